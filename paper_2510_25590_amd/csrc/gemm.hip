// bf16 GEMM on the CDNA4 matrix cores for the block's dense projections (QKV, attention
// output, MLP up/down; section "Region-Aware Generation": the DiT runs on [X^P, X^E] only).
//
//   C[m, n] = sum_k A[m, k] * W[n, k]      A: activations [M, K] row-major, W: weights, PACKED (see below)
//
// The number of rows M is the number of edited tokens (a few hundred to a few thousand), so the
// kernel is built around a 128-row tile: seven row tiles at 20 % of a 64x64 image.
//
//  * Weights never go through LDS.  regione_pack_weight stores them once in the register layout of
//    the "B" operand of v_mfma_f32_32x32x16_bf16: block (n/32, k/16) is 64 lanes x 16 bytes, lane l
//    holding W[32*(n/32) + l%32][16*(k/16) + 8*(l/32) .. +8].  A wave reads a fragment as one fully
//    coalesced 1 KiB load straight into VGPRs, three K-steps ahead of its use.
//  * The four waves of a workgroup split the tile along N only (wave tile 128 x 32*TN), so no weight
//    fragment is needed by two waves; the activation tile (128 x 64 per K-step) is shared through
//    LDS, XOR-swizzled so that ds_read_b128 of a fragment is conflict free, double buffered, its
//    global loads three K-steps ahead (L2 latency under load is about a microsecond, i.e.
//    more than two K-steps of matrix-core work).
//  * Few row tiles means few workgroups: GEMMs with a narrow N are split along K over blockIdx.y
//    into float partial sums, merged by a second kernel that applies the epilogue.
//  * Workgroups are numbered so that each XCD (blockIdx.x % 8) owns a contiguous range of weight
//    blocks: every weight byte then streams through one L2 only.
#include "common.h"
#include <math.h>
#include <type_traits>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // a native 16-byte vector: copies are single loads/stores
typedef __attribute__((ext_vector_type(8))) int i32x8;            // operand of the 8-bit MFMA: 32 E4M3 values per lane

constexpr int BM = 128;       // rows per workgroup tile
constexpr int TM = BM / 32;
constexpr int BK = 64;        // k elements per step
constexpr int kThreads = 256;
constexpr int A_PER_THREAD = BM * 8 / kThreads;  // 16-byte chunks of the A tile per thread
// K-steps between a global load and its use (four did not measure faster than three for the narrow tile)
template <int TN> struct Pipe { static constexpr int DEPTH = 3; static constexpr int NSETS = DEPTH + 1; };


__device__ __forceinline__ float gelu_tanh_f32(float x) {
    // 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3)
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    return x / (1.0f + __expf(-2.0f * u));
}

// Row of the key/value destination for output row `row` (its cache slot when a slot list is given).
template <int KIND>
__device__ __forceinline__ int64_t epilogue_kv_row(const GemmEpilogue& ep, int row) {
    if (KIND != EPI_QKV) return row;
    return ep.slot ? static_cast<int64_t>(ep.slot[row]) + ep.slot_offset : row;
}

template <int KIND>
__device__ __forceinline__ void epilogue_store(const GemmEpilogue& ep, int row, int64_t kv_row, int col, float acc, float bias, float gate) {
    float val = acc + bias;
    if (KIND == EPI_PLAIN) {
        if (ep.act == REGIONE_ACT_GELU_TANH && col >= ep.act_from) val = gelu_tanh_f32(val);
        const int64_t o = static_cast<int64_t>(row) * ep.ldy + col;
        if (ep.y_f32) static_cast<float*>(ep.y)[o] = val;
        else static_cast<bf16_t*>(ep.y)[o] = f32_to_bf16(val);
    } else if (KIND == EPI_QKV) {
        const int H = ep.hidden;
        if (col < H) {
            ep.q[static_cast<int64_t>(row) * ep.ldq + col] = f32_to_bf16(val);
        } else if (col < 3 * H) {
            if (col < 2 * H) ep.k[kv_row * ep.ldkv + (col - H)] = f32_to_bf16(val);
            else ep.v[kv_row * ep.ldkv + (col - 2 * H)] = f32_to_bf16(val);
        } else {
            if (ep.act == REGIONE_ACT_GELU_TANH) val = gelu_tanh_f32(val);
            static_cast<bf16_t*>(ep.y)[static_cast<int64_t>(row) * ep.ldy + ep.y_col0 + (col - 3 * H)] = f32_to_bf16(val);
        }
    } else if (KIND == EPI_VELOCITY) {
        // the velocity in its storage type, the cache takes it (Eq.9, fresh branch), the Euler update (Eq.4) with the
        // product and the difference rounded separately, and the row written where the merge by position puts it
        const int64_t o = static_cast<int64_t>(row) * ep.ldy + col;
        const int64_t full = ep.vel_index ? static_cast<int64_t>(ep.vel_index[row]) * ep.ldy + col : o;
        if (ep.y_f32) {
            if (ep.y) static_cast<float*>(ep.y)[o] = val;
            static_cast<float*>(ep.vel_ca)[o] = val;
            const float x = __fsub_rn(static_cast<float*>(ep.vel_xe)[o], __fmul_rn(ep.vel_dt, val));
            static_cast<float*>(ep.vel_xe)[o] = x;
            if (ep.vel_xfull) static_cast<float*>(ep.vel_xfull)[full] = x;
        } else {
            const bf16_t vb = f32_to_bf16(val);
            const float v = bf16_to_f32(vb);
            if (ep.y) static_cast<bf16_t*>(ep.y)[o] = vb;
            static_cast<bf16_t*>(ep.vel_ca)[o] = vb;
            const bf16_t xb = f32_to_bf16(__fsub_rn(bf16_to_f32(static_cast<bf16_t*>(ep.vel_xe)[o]), __fmul_rn(ep.vel_dt, v)));
            static_cast<bf16_t*>(ep.vel_xe)[o] = xb;
            if (ep.vel_xfull) static_cast<bf16_t*>(ep.vel_xfull)[full] = xb;
        }
    } else {  // EPI_RESID
        const int64_t ri = static_cast<int64_t>(row) * ep.ldr + col;
        const float res = ep.resid_f32 ? static_cast<const float*>(ep.resid)[ri] : bf16_to_f32(static_cast<const bf16_t*>(ep.resid)[ri]);
        val = res + gate * val;
        const int64_t o = static_cast<int64_t>(row) * ep.ldy + col;
        if (ep.y_f32) static_cast<float*>(ep.y)[o] = val;
        else static_cast<bf16_t*>(ep.y)[o] = f32_to_bf16(val);
    }
}

typedef __attribute__((ext_vector_type(4))) float f32x4;
constexpr int kMaxSplits = 8;   // largest K split the planner or a forced plan uses

typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;

// W = 4 or 8 consecutive elements: 16- or 32-byte (float32), 8- or 16-byte (bf16) pieces
template <int W>
__device__ __forceinline__ void store_vec(void* base, int64_t elem, int as_f32, const float (&v)[W]) {
    if (as_f32) {
        float* p = static_cast<float*>(base) + elem;
#pragma unroll
        for (int h = 0; h < W / 4; ++h) *reinterpret_cast<f32x4*>(p + 4 * h) = f32x4{v[4 * h], v[4 * h + 1], v[4 * h + 2], v[4 * h + 3]};
    } else if (W == 8) {
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = static_cast<__bf16>(v[e]);
        *reinterpret_cast<bf16x8*>(static_cast<bf16_t*>(base) + elem) = o;
    } else {
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = static_cast<__bf16>(v[e]);
        *reinterpret_cast<bf16x4*>(static_cast<bf16_t*>(base) + elem) = o;
    }
}
__device__ __forceinline__ void store8(void* base, int64_t elem, int as_f32, const float (&v)[8]) { store_vec<8>(base, elem, as_f32, v); }

// Epilogue for W consecutive columns col0..col0+W-1 of one row (all inside N, col0 a multiple of W, W = 4 or 8;
// the wide-epilogue conditions hold, so a group never straddles two destinations): wide loads and stores only.
template <int KIND, int W>
__device__ __forceinline__ void epilogue_store_vec(const GemmEpilogue& ep, int row, int col0, const float (&acc)[W],
                                                   const float (&bias)[W], const float (&gate)[W]) {
    float val[W];
#pragma unroll
    for (int e = 0; e < W; ++e) val[e] = acc[e] + bias[e];
    if (KIND == EPI_PLAIN) {
        if (ep.act == REGIONE_ACT_GELU_TANH) {
#pragma unroll
            for (int e = 0; e < W; ++e) if (col0 + e >= ep.act_from) val[e] = gelu_tanh_f32(val[e]);
        }
        store_vec<W>(ep.y, static_cast<int64_t>(row) * ep.ldy + col0, ep.y_f32, val);
    } else if (KIND == EPI_QKV) {
        const int H = ep.hidden;   // a multiple of 8
        if (col0 < H) {
            store_vec<W>(ep.q, static_cast<int64_t>(row) * ep.ldq + col0, 0, val);
        } else if (col0 < 3 * H) {
            const int64_t kv_row = epilogue_kv_row<KIND>(ep, row);
            if (col0 < 2 * H) store_vec<W>(ep.k, kv_row * ep.ldkv + (col0 - H), 0, val);
            else store_vec<W>(ep.v, kv_row * ep.ldkv + (col0 - 2 * H), 0, val);
        } else {
            if (ep.act == REGIONE_ACT_GELU_TANH) {
#pragma unroll
                for (int e = 0; e < W; ++e) val[e] = gelu_tanh_f32(val[e]);
            }
            store_vec<W>(ep.y, static_cast<int64_t>(row) * ep.ldy + ep.y_col0 + (col0 - 3 * H), 0, val);
        }
    } else {  // EPI_RESID
        const int64_t ri = static_cast<int64_t>(row) * ep.ldr + col0;
        float res[W];
        if (ep.resid_f32) {
#pragma unroll
            for (int h = 0; h < W / 4; ++h) {
                const f32x4 a = *reinterpret_cast<const f32x4*>(static_cast<const float*>(ep.resid) + ri + 4 * h);
#pragma unroll
                for (int e = 0; e < 4; ++e) res[4 * h + e] = a[e];
            }
        } else if (W == 8) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(static_cast<const bf16_t*>(ep.resid) + ri);
#pragma unroll
            for (int e = 0; e < 8; ++e) res[e] = static_cast<float>(a[e]);
        } else {
            const bf16x4 a = *reinterpret_cast<const bf16x4*>(static_cast<const bf16_t*>(ep.resid) + ri);
#pragma unroll
            for (int e = 0; e < 4; ++e) res[e] = static_cast<float>(a[e]);
        }
#pragma unroll
        for (int e = 0; e < W; ++e) val[e] = res[e] + gate[e] * val[e];
        store_vec<W>(ep.y, static_cast<int64_t>(row) * ep.ldy + col0, ep.y_f32, val);
    }
}
template <int KIND>
__device__ __forceinline__ void epilogue_store8(const GemmEpilogue& ep, int row, int col0, const float (&acc)[8],
                                                const float (&bias)[8], const float (&gate)[8]) {
    epilogue_store_vec<KIND, 8>(ep, row, col0, acc, bias, gate);
}

// Writes a wave's accumulators: the 128 x 32*TN tile whose first row is m0 and first column n0 + wn0.  `stage_lds`:
// 8 KiB of LDS per wave (indexed by the wave's number in the workgroup) that no wave reads any more once all waves
// have passed the barrier inside.  accumulator (i, j, r) of a lane: row = 8*(r/4) + 4*(lane/32) + r%4, column = lane%32
// of the 32x32 block (i, j) of the wave tile.
// SCALED (the 8-bit GEMM): every sum is first multiplied by ep.row_scale[row] * ep.col_scale[column], also on its way
// into a split-K partial result (the scaling is linear, so the merge needs no change).
template <int TN, int KIND, bool SCALED = false>
__device__ __forceinline__ void gemm_epilogue(f32x16 (&acc)[TM][TN], float* stage_lds, int M, int N, int m0, int n0, int wn0,
                                              float* __restrict__ partial, const GemmEpilogue& ep) {
    constexpr int WN = 32 * TN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    float* part_base = partial ? partial + (static_cast<int64_t>(blockIdx.y) * M) * N : nullptr;
    if (ep.vec_ok) {
        // Transpose through LDS, 32 rows at a time, so that every lane ends up with eight consecutive columns of one
        // row: bias, gate, residual and result then move in 16- or 32-byte pieces.  Each wave stages in its own 8 KiB.
        __syncthreads();   // every wave has finished reading the A tiles
        float* stage = stage_lds + wave * (32 * 64);
        constexpr int G = WN / 8;            // column groups per row
        constexpr int ROWS_PER_PASS = 64 / G;
        const int cg = lane % G, rsub = lane / G;
        const int col0 = n0 + wn0 + cg * 8;
        const bool col_live = col0 < N;      // N is a multiple of 8 on this path
        float bias[8], gate[8], cscale[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            bias[e] = (!partial && col_live && ep.bias) ? ep.bias[col0 + e] : 0.f;
            gate[e] = (!partial && col_live && KIND == EPI_RESID && ep.gate) ? ep.gate[col0 + e] : 1.f;
            cscale[e] = (SCALED && col_live) ? ep.col_scale[col0 + e] : 1.f;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    stage[(8 * (r >> 2) + 4 * lh + (r & 3)) * WN + j * 32 + l32] = acc[i][j][r];
#pragma unroll
            for (int p = 0; p < 32 / ROWS_PER_PASS; ++p) {
                const int rr = p * ROWS_PER_PASS + rsub;
                const int row = m0 + i * 32 + rr;
                const f32x4 lo = *reinterpret_cast<const f32x4*>(stage + rr * WN + cg * 8);
                const f32x4 hi = *reinterpret_cast<const f32x4*>(stage + rr * WN + cg * 8 + 4);
                float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                if (row < M && col_live) {
                    if (SCALED) {
                        const float rs = ep.row_scale[row];
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] *= rs * cscale[e];
                    }
                    if (partial) store8(part_base, static_cast<int64_t>(row) * N + col0, 1, v);
                    else epilogue_store8<KIND>(ep, row, col0, v, bias, gate);
                }
            }
        }
        return;
    }
    int col[TN];
    float bias[TN], gate[TN], cscale[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        col[j] = n0 + wn0 + j * 32 + l32;
        const bool live = col[j] < N;
        cscale[j] = (SCALED && live) ? ep.col_scale[col[j]] : 1.f;
        bias[j] = (!partial && live && ep.bias) ? ep.bias[col[j]] : 0.f;
        gate[j] = (!partial && live && KIND == EPI_RESID && ep.gate) ? ep.gate[col[j]] : 1.f;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = m0 + i * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
            if (row >= M) continue;
            const float rs = SCALED ? ep.row_scale[row] : 1.f;
            if (partial) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (col[j] < N) part_base[static_cast<int64_t>(row) * N + col[j]] = SCALED ? acc[i][j][r] * (rs * cscale[j]) : acc[i][j][r];
            } else {
                const int64_t kv_row = epilogue_kv_row<KIND>(ep, row);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (col[j] < N) epilogue_store<KIND>(ep, row, kv_row, col[j], SCALED ? acc[i][j][r] * (rs * cscale[j]) : acc[i][j][r], bias[j], gate[j]);
            }
        }
    }
}

// Tile order inside the launch: groups of `gh` row tiles; inside a group all column tiles, and for each column tile
// the group's row tiles consecutively.  The workgroups that run at the same time on an XCD then share a weight line
// among gh CUs and an activation line among the rest, instead of all of them hammering the same weight lines.
__device__ __forceinline__ void tile_coords(int tile, int m_tiles, int n_tiles, int gh, int& m_tile, int& n_tile) {
    const int per_group = gh * n_tiles;
    const int group = tile / per_group, rem = tile - group * per_group;
    int rows = m_tiles - group * gh;
    rows = rows < gh ? rows : gh;
    n_tile = rem / rows;
    m_tile = group * gh + (rem - n_tile * rows);
}

// Global loads of the pipeline are written in assembly and waited for by hand.  Left to the compiler, the rotating
// register sets made its wait-count insertion drain nearly every outstanding load at the top of a K-step (it reuses
// the registers of a consumed set for LDS fragments and then protects them against loads it believes pending), which
// shortened the prefetch distance from three steps to less than one.  An asm load is invisible to that pass; the
// matching rg_wait_loads below names the registers it makes valid, so no use can be scheduled above it.
__device__ __forceinline__ void rg_load16(u32x4& dst, const bf16_t* p) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(p));
}
template <int BYTES>
__device__ __forceinline__ void rg_load16_off(u32x4& dst, const bf16_t* p) {
    asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(dst) : "v"(p), "n"(BYTES));
}
// Waits until at most N of this wave's vector-memory loads are outstanding (they complete in issue order).
template <int N, int TN>
__device__ __forceinline__ void rg_wait_loads(u32x4 (&a)[4], u32x4 (&w)[TN * 4]) {
    if constexpr (TN == 1)
        asm volatile("s_waitcnt vmcnt(%8)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]) : "n"(N));
    else
        asm volatile("s_waitcnt vmcnt(%12)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]),
                     "+v"(w[4]), "+v"(w[5]), "+v"(w[6]), "+v"(w[7]) : "n"(N));
}

// Quarter q of the loads of one K-step: one 16-byte chunk of the A tile per thread (thread t owns chunk t & 7 of rows
// (t >> 3) + 32*q) and fragment q of every 32-column weight block of the wave.
template <int TN, int Q>
__device__ __forceinline__ void load_quarter(u32x4 (&areg)[A_PER_THREAD], u32x4 (&wreg)[TN * 4], const bf16_t* const (&a_rows)[A_PER_THREAD],
                                             const bf16_t* const (&w_blk)[TN], int step) {
    rg_load16(areg[Q], a_rows[Q] + step * BK);
#pragma unroll
    for (int j = 0; j < TN; ++j) rg_load16_off<Q * 1024>(wreg[j * 4 + Q], w_blk[j] + static_cast<int64_t>(step) * 2048);
}
template <int TN>
__device__ __forceinline__ void load_step(u32x4 (&areg)[A_PER_THREAD], u32x4 (&wreg)[TN * 4], const bf16_t* const (&a_rows)[A_PER_THREAD],
                                          const bf16_t* const (&w_blk)[TN], int step) {
    load_quarter<TN, 0>(areg, wreg, a_rows, w_blk, step);
    load_quarter<TN, 1>(areg, wreg, a_rows, w_blk, step);
    load_quarter<TN, 2>(areg, wreg, a_rows, w_blk, step);
    load_quarter<TN, 3>(areg, wreg, a_rows, w_blk, step);
}

__device__ __forceinline__ void a_store(bf16_t* lds, const u32x4 (&regs)[A_PER_THREAD]) {
    const int r0 = threadIdx.x >> 3, c = threadIdx.x & 7;
#pragma unroll
    for (int i = 0; i < A_PER_THREAD; ++i) {
        const int r = r0 + 32 * i;
        *reinterpret_cast<u32x4*>(lds + r * BK + ((c ^ ((r >> 1) & 7)) << 3)) = regs[i];
    }
}
__device__ __forceinline__ bf16x8 a_frag(const bf16_t* tile, int row, int chunk) {
    // rows are 128 bytes: 16 consecutive rows x one logical chunk cover all 64 banks exactly once
    return *reinterpret_cast<const bf16x8*>(tile + row * BK + ((chunk ^ ((row >> 1) & 7)) << 3));
}

template <int TN, int KIND>
__global__ void __launch_bounds__(kThreads)
gemm_bf16_kernel(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ Wp,
                 int M, int N, int K, int m_tiles, int n_tiles, int tiles_per_xcd, int group_rows,
                 int steps_per_split, float* __restrict__ partial, GemmEpilogue ep) {
    constexpr int WN = 32 * TN, BN = 4 * WN;
    __shared__ __attribute__((aligned(16))) bf16_t a_lds[2][BM * BK];

    // XCD-aware tile numbering: consecutive tiles (same weight columns, all row tiles) stay on one XCD
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int tile = xcd * tiles_per_xcd + local;
    if (local >= tiles_per_xcd || tile >= m_tiles * n_tiles) return;
    int n_tile, m_tile;
    tile_coords(tile, m_tiles, n_tiles, group_rows, m_tile, n_tile);
    const int m0 = m_tile * BM, n0 = n_tile * BN;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int wn0 = wave * WN;

    const int total_steps = K / BK;           // K is a multiple of 64 (checked by the launcher)
    const int ks_begin = blockIdx.y * steps_per_split;
    int nks = total_steps - ks_begin;
    nks = nks < steps_per_split ? nks : steps_per_split;

    // per-thread source rows of the A tile (rows past M repeat the last row; their results are never stored)
    const bf16_t* a_rows[A_PER_THREAD];
#pragma unroll
    for (int i = 0; i < A_PER_THREAD; ++i) {
        int r = m0 + (threadIdx.x >> 3) + 32 * i;
        r = r < M ? r : M - 1;
        a_rows[i] = A + static_cast<int64_t>(r) * lda + (threadIdx.x & 7) * 8;
    }
    // per-wave weight blocks (blocks past N repeat the last block)
    const int n_blocks = (N + 31) >> 5;
    const int64_t blk_stride = static_cast<int64_t>(K >> 4) * 512;  // elements per 32-column block
    const bf16_t* w_blk[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int nb = ((n0 + wn0) >> 5) + j;
        nb = nb < n_blocks ? nb : n_blocks - 1;
        w_blk[j] = Wp + nb * blk_stride + lane * 8;
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // The K-steps run in groups of four through a software pipeline without any branch inside (so that the order of
    // its loads and waits is the same on every path, which the build verifies on the machine code); the up to three
    // steps that remain run one at a time behind it.
    constexpr int DEPTH = Pipe<TN>::DEPTH, NSETS = Pipe<TN>::NSETS;
    static_assert(NSETS == 4, "the unrolled schedule below rotates four register sets");
    const int n4 = nks & ~3;
    if (n4 > 0) {
        u32x4 areg[NSETS][A_PER_THREAD];
        u32x4 wreg[NSETS][TN * 4];
        constexpr int L = A_PER_THREAD + 4 * TN;        // loads per thread and K-step
        // steps past the end of the pipelined part re-load its last step (keeps the number of loads in flight constant)
#pragma unroll
        for (int p = 0; p < DEPTH; ++p) load_step<TN>(areg[p], wreg[p], a_rows, w_blk, ks_begin + (p < n4 ? p : n4 - 1));
        rg_wait_loads<(DEPTH - 1) * L, TN>(areg[0], wreg[0]);
        a_store(a_lds[0], areg[0]);
        __syncthreads();

        // One K-step.  S = j % NSETS names the register set that holds step j; the loads of step j + DEPTH go to the
        // set freed by step j - 1; they are issued a quarter at a time in front of each quarter's MFMAs, together with
        // the LDS reads of the next quarter, so that the memory pipes work in the shadow of the matrix cores.
        // Nothing of the hand-over between two steps stands at the step boundary: the A tile of step j+1 is stored
        // right after the first quarter of step j (its loads landed long ago, and the buffer it goes to was last read
        // before the barrier of step j-1); the one barrier of a step stands before its fourth quarter, when every
        // wave has stored its part of the next tile and issued its last reads of this one; and the first fragments of
        // step j+1 are read behind that barrier, under the MFMAs of the fourth quarter.  (With the store, the barrier
        // and the first read all at the boundary the same kernel ran 1-8 % slower, bit-identical results.)
        // (Macros, not lambdas: captured arrays would live in memory.)
        bf16x8 af[2][TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) af[0][i] = a_frag(a_lds[0], i * 32 + l32, lh);
#define RG_GEMM_QUARTER(KK, S, SD)                                                                        \
    {                                                                                                     \
        /* memory instructions of this quarter first, then its MFMAs: they run under the MFMAs */           \
        if (KK < 3) {                                                                                     \
            _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                \
                af[(KK + 1) & 1][i] = a_frag(at, i * 32 + l32, (KK + 1) * 2 + lh);                        \
        } else {                                                                                          \
            _Pragma("unroll") for (int i = 0; i < TM; ++i) af[0][i] = a_frag(nx, i * 32 + l32, lh);       \
        }                                                                                                 \
        load_quarter<TN, KK>(areg[SD], wreg[SD], a_rows, w_blk, st_);                                     \
        _Pragma("unroll") for (int jn = 0; jn < TN; ++jn) {                                               \
            const bf16x8 wf = __builtin_bit_cast(bf16x8, wreg[S][jn * 4 + KK]);                           \
            _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                \
                acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[KK & 1][i], wf, acc[i][jn], 0, 0, 0); \
        }                                                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                                \
    }
#define RG_GEMM_STEP(J, S, S1, SD)                                                                        \
    {                                                                                                     \
        const int j_ = (J);                                                                               \
        const int st_ = ks_begin + (j_ + DEPTH < n4 ? j_ + DEPTH : n4 - 1);                               \
        const bf16_t* at = a_lds[j_ & 1];                                                                 \
        bf16_t* nx = a_lds[(j_ + 1) & 1];                                                                 \
        RG_GEMM_QUARTER(0, S, SD)                                                                         \
        /* in flight: steps j+1, j+2 and the first quarter of step j+3; step j+1 is wanted (its A tile now, its */ \
        /* weights in the next step) */                                                                   \
        rg_wait_loads<L + 1 + TN, TN>(areg[S1], wreg[S1]);                                                \
        a_store(nx, areg[S1]);                                                                            \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        RG_GEMM_QUARTER(1, S, SD)                                                                         \
        RG_GEMM_QUARTER(2, S, SD)                                                                         \
        __syncthreads();                                                                                  \
        RG_GEMM_QUARTER(3, S, SD)                                                                         \
    }
        for (int j = 0; j < n4; j += 4) {
            RG_GEMM_STEP(j, 0, 1, 3)
            RG_GEMM_STEP(j + 1, 1, 2, 0)
            RG_GEMM_STEP(j + 2, 2, 3, 1)
            RG_GEMM_STEP(j + 3, 3, 0, 2)
        }
#undef RG_GEMM_STEP
#undef RG_GEMM_QUARTER
        // the loads issued for steps past the end are still in flight; they must land before their registers are reused
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    // remaining steps, one at a time: A tile through registers into LDS, weight fragments into registers, then the MFMAs
    for (int j = n4; j < nks; ++j) {
        const int st = ks_begin + j;
        u32x4 ar[A_PER_THREAD];
        bf16x8 wf[TN][4];
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) ar[i] = *reinterpret_cast<const u32x4*>(a_rows[i] + st * BK);
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                wf[jn][kk] = *reinterpret_cast<const bf16x8*>(w_blk[jn] + static_cast<int64_t>(st) * 2048 + kk * 512);
        __syncthreads();   // every wave has finished reading the tile of the step before
        a_store(a_lds[0], ar);
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 af[TM];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = a_frag(a_lds[0], i * 32 + l32, kk * 2 + lh);
#pragma unroll
            for (int jn = 0; jn < TN; ++jn)
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[jn][kk], acc[i][jn], 0, 0, 0);
        }
    }

    gemm_epilogue<TN, KIND>(acc, reinterpret_cast<float*>(&a_lds[0][0]), M, N, m0, n0, wn0, partial, ep);
}

// ---------------------------------------------------------------------------------------------------------------
// Second GEMM kernel: both operands through LDS by asynchronous global-to-LDS copies, no staging registers.
// 128 x (128*TN) workgroup tile, four waves split N as above, K in stages of 32.  Without register sets for the
// pipeline a wave needs fewer than 256 registers, so two workgroups share a CU: while one waits at a barrier or on
// LDS, the other keeps the matrix cores busy.
//   stage = A tile [128 rows x 32 k] (rows of 64 bytes, 16-byte chunk c of row r stored at chunk c ^ ((r >> 2) & 3):
//           the 16 rows of a ds_read_b128 phase then cover all 64 banks once)
//         + per wave, TN blocks x 2 k-groups of packed-weight fragments (1 KiB each, lane l's 16 bytes at 16*l:
//           exactly what the packed layout holds, so the copy is linear and the read conflict-free)
constexpr int LK = 32;                 // k elements per stage
constexpr int L_STAGES = 3;
// WM = 1: 128-row workgroup tile, 4 waves.  WM = 2: 256 rows, 8 waves as 2 (rows) x 4 (columns); the two waves of a
// column group share their weight fragments, which cuts the bytes fetched per FLOP by a third.
template <int TN, int WM> struct LdsGemm {
    static constexpr int ROWS = BM * WM;
    static constexpr int THREADS = kThreads * WM;
    static constexpr unsigned A_BYTES = ROWS * LK * 2;               // 8 KiB per 128 rows
    static constexpr unsigned W_BYTES = 4 * TN * 2 * 1024;           // 8 KiB per 32 columns of wave tile
    static constexpr unsigned STAGE_BYTES = A_BYTES + W_BYTES;
    static constexpr unsigned EPI_BYTES = 4 * WM * 8192;             // epilogue staging: 8 KiB per wave
    static constexpr unsigned LDS_BYTES = (L_STAGES * STAGE_BYTES > EPI_BYTES ? L_STAGES * STAGE_BYTES : EPI_BYTES);
    static constexpr int A_COPIES = ROWS * 4 / THREADS;              // 16-byte slots of the A tile per thread (= 2)
    static constexpr int W_FRAGS = 4 * TN * 2;                       // 1 KiB fragments per stage
    static constexpr int W_COPIES = W_FRAGS / (4 * WM);              // per wave
    static constexpr int COPIES = A_COPIES + W_COPIES;               // asynchronous copies per thread and stage
};

// lane l of the wave writes LDS[lds_base + 16*l .. +16) from src (wave-uniform lds_base); counted in vmcnt
__device__ __forceinline__ void rg_async_copy16(const bf16_t* src, unsigned lds_base_bytes) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(src), "s"(lds_base_bytes) : "memory", "m0");
}

// FP8 = true: the same bytes hold E4M3 values (A, lda, K and every k index of this kernel then count PAIRS of
// them, i.e. 2 bytes).  A stage is ONE k-step of v_mfma_f32_32x32x64_f8f6f4: a lane's 32 operand bytes are the two
// 16-byte pieces that the bf16 path feeds to two MFMAs, bytes [16*(lane/32), +16) and [32 + 16*(lane/32), +16) of the
// stage's 64-byte row.  Which k of the instruction each byte becomes does not matter: activations and weights are laid
// out alike, and the sum over k does not depend on its order.
template <int TN, int WM, int KIND, bool FP8 = false>
__global__ void __launch_bounds__(kThreads * WM) __attribute__((amdgpu_waves_per_eu(2, 2)))
gemm_lds_kernel(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ Wp,
                int M, int N, int K, int m_tiles, int n_tiles, int tiles_per_xcd, int group_rows,
                int steps_per_split, float* __restrict__ partial, GemmEpilogue ep) {
    using G = LdsGemm<TN, WM>;
    constexpr int WN = 32 * TN, BN = 4 * WN;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const unsigned lds0 = static_cast<unsigned>(reinterpret_cast<size_t>((__attribute__((address_space(3))) void*)(lds_raw)));

    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int tile = xcd * tiles_per_xcd + local;
    if (local >= tiles_per_xcd || tile >= m_tiles * n_tiles) return;
    int n_tile, m_tile;
    tile_coords(tile, m_tiles, n_tiles, group_rows, m_tile, n_tile);
    const int m0_wg = m_tile * G::ROWS, n0 = n_tile * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int wn = wave & 3, wm = wave >> 2;     // column group and row half of this wave
    const int wn0 = wn * WN;
    const int m0 = m0_wg + wm * BM;              // first row of the wave tile

    const int total_steps = K / BK;            // split-K bookkeeping stays in steps of 64
    const int ks_begin = blockIdx.y * steps_per_split;
    int nks = total_steps - ks_begin;
    nks = nks < steps_per_split ? nks : steps_per_split;
    const int n_stages = nks * (BK / LK);
    const int k_begin = ks_begin * BK;

    // copy sources.  A: thread t owns LDS slots t and t + THREADS of the stage's A tile (slot = row*4 + physical chunk);
    // the swizzle is applied on the global side: the lane that owns physical chunk p of a row loads logical chunk
    // p ^ ((row >> 2) & 3).  Rows past M repeat the last row; their results are never stored.
    const bf16_t* a_src[G::A_COPIES];
#pragma unroll
    for (int i = 0; i < G::A_COPIES; ++i) {
        const int slot = threadIdx.x + G::THREADS * i;
        const int row = slot >> 2, phys = slot & 3;
        int r = m0_wg + row;
        r = r < M ? r : M - 1;
        a_src[i] = A + static_cast<int64_t>(r) * lda + k_begin + ((phys ^ ((row >> 2) & 3)) << 3);
    }
    // W: the stage holds fragment f = (column group * TN + block) * 2 + k-group; wave w copies fragments
    // w * W_COPIES .. + W_COPIES - 1 (with WM = 1 exactly the fragments it reads itself)
    const int n_blocks = (N + 31) >> 5;
    const int64_t blk_stride = static_cast<int64_t>(K >> 4) * 512;   // elements per 32-column block
    const bf16_t* w_src[G::W_COPIES];
#pragma unroll
    for (int c = 0; c < G::W_COPIES; ++c) {
        const int f = wave * G::W_COPIES + c;
        const int g = f & 1, blk = f >> 1;                           // blk = column group * TN + block inside the group
        int nb = (n0 >> 5) + blk;
        nb = nb < n_blocks ? nb : n_blocks - 1;                      // blocks past N repeat the last block
        w_src[c] = Wp + nb * blk_stride + (static_cast<int64_t>(k_begin >> 4) + g) * 512 + lane * 8;
    }
    const unsigned a_dst = __builtin_amdgcn_readfirstlane(lds0 + static_cast<unsigned>(wave) * 1024u);
    const unsigned w_dst = __builtin_amdgcn_readfirstlane(lds0 + G::A_BYTES + static_cast<unsigned>(wave * G::W_COPIES) * 1024u);
    auto issue = [&](int st, unsigned stage_off) __attribute__((always_inline)) {   // st: stage index, clamped by the caller
#pragma unroll
        for (int i = 0; i < G::A_COPIES; ++i)
            rg_async_copy16(a_src[i] + st * LK, a_dst + stage_off + static_cast<unsigned>(i) * (G::THREADS * 16u));
#pragma unroll
        for (int c = 0; c < G::W_COPIES; ++c)
            rg_async_copy16(w_src[c] + static_cast<int64_t>(st) * 1024, w_dst + stage_off + static_cast<unsigned>(c) * 1024u);
    };

    // fragment read offsets (bytes inside a stage)
    unsigned a_off[2][TM];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = wm * BM + i * 32 + l32;
            a_off[kk][i] = static_cast<unsigned>(row) * 64u + static_cast<unsigned>(((2 * kk + lh) ^ ((row >> 2) & 3)) << 4);
        }
    const unsigned w_off = G::A_BYTES + static_cast<unsigned>(wn) * (TN * 2048u) + static_cast<unsigned>(lane) * 16u;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    if constexpr (FP8) {
        // Three LDS stages, copies three stages ahead.  A stage is one k-step; its MFMAs run in two halves (row blocks
        // 0-1, then 2-3) with the same hand-over between them as in the bf16 schedule below:
        //   first half : read the A fragments of row blocks 2-3 of stage t, run the MFMAs of row blocks 0-1
        //   middle     : wait for the copies of stage t+1, barrier, issue the copies of stage t+3 into the buffer of
        //                stage t, read the weight fragments and the A fragments of row blocks 0-1 of stage t+1
        //   second half: run the MFMAs of row blocks 2-3.
        static_assert(L_STAGES == 3 && TM == 4, "the schedule below rotates three buffers and splits four row blocks");
        auto clamp_stage = [&](int t) __attribute__((always_inline)) { return t < n_stages ? t : n_stages - 1; };
#pragma unroll
        for (int p = 0; p < L_STAGES; ++p) issue(clamp_stage(p), p * G::STAGE_BYTES);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * G::COPIES) : "memory");
        __syncthreads();
        u32x4 a8[TM][2], w8[2][TN][2];      // [..][kk]: the two 16-byte pieces of an operand
#define RG_F8_AFRAGS(I0, S)                                                                               \
    {                                                                                                     \
        const unsigned char* st_ = lds_raw + (S) * G::STAGE_BYTES;                                        \
        _Pragma("unroll") for (int i = (I0); i < (I0) + 2; ++i)                                           \
            _Pragma("unroll") for (int kk = 0; kk < 2; ++kk)                                              \
                a8[i][kk] = *reinterpret_cast<const u32x4*>(st_ + a_off[kk][i]);                          \
    }
#define RG_F8_WFRAGS(P, S)                                                                                \
    {                                                                                                     \
        const unsigned char* st_ = lds_raw + (S) * G::STAGE_BYTES;                                        \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                    \
            _Pragma("unroll") for (int kk = 0; kk < 2; ++kk)                                              \
                w8[P][j][kk] = *reinterpret_cast<const u32x4*>(st_ + w_off + (j * 2 + kk) * 1024);        \
    }
#define RG_F8_MFMAS(I0, P)                                                                                \
    _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                        \
        _Pragma("unroll") for (int i = (I0); i < (I0) + 2; ++i) {                                         \
            const i32x8 av = {(int)a8[i][0][0], (int)a8[i][0][1], (int)a8[i][0][2], (int)a8[i][0][3],     \
                              (int)a8[i][1][0], (int)a8[i][1][1], (int)a8[i][1][2], (int)a8[i][1][3]};    \
            const i32x8 wv = {(int)w8[P][j][0][0], (int)w8[P][j][0][1], (int)w8[P][j][0][2], (int)w8[P][j][0][3], \
                              (int)w8[P][j][1][0], (int)w8[P][j][1][1], (int)w8[P][j][1][2], (int)w8[P][j][1][3]}; \
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, wv, acc[i][j], 0, 0, 0, 0, 0, 0); \
        }
#define RG_F8_STAGE(T, S, P)                                                                              \
    {                                                                                                     \
        const int t_ = (T);                                                                               \
        RG_F8_AFRAGS(2, S)                                                                                \
        RG_F8_MFMAS(0, P)                                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(G::COPIES) : "memory");                                  \
        __syncthreads();                                                                                  \
        issue(clamp_stage(t_ + L_STAGES), (S) * G::STAGE_BYTES);                                          \
        RG_F8_WFRAGS((P) ^ 1, ((S) + 1) % L_STAGES)                                                       \
        RG_F8_AFRAGS(0, ((S) + 1) % L_STAGES)                                                             \
        RG_F8_MFMAS(2, P)                                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                                \
    }
        RG_F8_WFRAGS(0, 0)
        RG_F8_AFRAGS(0, 0)
        for (int t = 0; t < n_stages; t += 6) {
            RG_F8_STAGE(t, 0, 0)
            if (t + 1 < n_stages) RG_F8_STAGE(t + 1, 1, 1)
            if (t + 2 < n_stages) RG_F8_STAGE(t + 2, 2, 0)
            if (t + 3 < n_stages) RG_F8_STAGE(t + 3, 0, 1)
            if (t + 4 < n_stages) RG_F8_STAGE(t + 4, 1, 0)
            if (t + 5 < n_stages) RG_F8_STAGE(t + 5, 2, 1)
        }
#undef RG_F8_STAGE
#undef RG_F8_MFMAS
#undef RG_F8_WFRAGS
#undef RG_F8_AFRAGS
    } else {
    // Three LDS stages, copies three stages ahead, fragments one half-stage ahead.  A stage is two MFMA k-steps:
    //   first half : read the second k-step's fragments of stage t, run the MFMAs of its first k-step (fragments read
    //                during stage t-1)
    //   middle     : wait until the copies of stage t+1 have landed, barrier (publishes them; every wave has finished
    //                reading stage t, so its buffer is free), issue the copies of stage t+3 into that buffer, read the
    //                first k-step's fragments of stage t+1
    //   second half: run the MFMAs of the second k-step, which hide the latency of what the middle part issued.
    // Stages past the end re-copy the last one, so the copy count per stage is constant.
    static_assert(L_STAGES == 3, "the schedule below rotates three buffers");
    auto clamp_stage = [&](int t) __attribute__((always_inline)) { return t < n_stages ? t : n_stages - 1; };
#pragma unroll
    for (int p = 0; p < L_STAGES; ++p) issue(clamp_stage(p), p * G::STAGE_BYTES);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * G::COPIES) : "memory");
    __syncthreads();
    bf16x8 af[2][TM], wf[2][TN];
#define RG_LDS_FRAGS(KK, S)                                                                               \
    {                                                                                                     \
        const unsigned char* st_ = lds_raw + (S) * G::STAGE_BYTES;                                        \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                    \
            af[KK][i] = *reinterpret_cast<const bf16x8*>(st_ + a_off[KK][i]);                             \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                    \
            wf[KK][j] = *reinterpret_cast<const bf16x8*>(st_ + w_off + (j * 2 + KK) * 1024);              \
    }
#define RG_LDS_MFMAS(KK)                                                                                  \
    _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                        \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                    \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[KK][i], wf[KK][j], acc[i][j], 0, 0, 0);
#define RG_LDS_STAGE(T, S)                                                                                \
    {                                                                                                     \
        const int t_ = (T);                                                                               \
        RG_LDS_FRAGS(1, S)                                                                                \
        RG_LDS_MFMAS(0)                                                                                   \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(G::COPIES) : "memory");                                  \
        __syncthreads();                                                                                  \
        issue(clamp_stage(t_ + L_STAGES), (S) * G::STAGE_BYTES);                                          \
        RG_LDS_FRAGS(0, (S + 1) % L_STAGES)                                                               \
        RG_LDS_MFMAS(1)                                                                                   \
        __builtin_amdgcn_sched_barrier(0);                                                                \
    }
    RG_LDS_FRAGS(0, 0)
    for (int t = 0; t < n_stages; t += 3) {
        RG_LDS_STAGE(t, 0)
        if (t + 1 < n_stages) RG_LDS_STAGE(t + 1, 1)
        if (t + 2 < n_stages) RG_LDS_STAGE(t + 2, 2)
    }
#undef RG_LDS_STAGE
#undef RG_LDS_MFMAS
#undef RG_LDS_FRAGS
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing may still be writing LDS when the epilogue reuses it
    gemm_epilogue<TN, KIND, FP8>(acc, reinterpret_cast<float*>(lds_raw), M, N, m0, n0, wn0, partial, ep);
}

// Sums the split-K partial results and applies the epilogue.  One thread per output element, columns fastest.
template <int KIND>
__global__ void __launch_bounds__(kThreads)
splitk_epilogue_kernel(const float* __restrict__ partial, int splits, int M, int N, GemmEpilogue ep) {
    const int64_t total = static_cast<int64_t>(M) * N;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; e < total; e += stride) {
        const int row = static_cast<int>(e / N), col = static_cast<int>(e - static_cast<int64_t>(row) * N);
        float s = 0.f;
        for (int p = 0; p < splits; ++p) s += partial[p * total + e];
        const float bias = ep.bias ? ep.bias[col] : 0.f;
        const float gate = (KIND == EPI_RESID && ep.gate) ? ep.gate[col] : 1.f;
        epilogue_store<KIND>(ep, row, epilogue_kv_row<KIND>(ep, row), col, s, bias, gate);
    }
}

// The same with the wide epilogue's conditions (N a multiple of 8, aligned rows): one thread per group of FOUR
// columns, so that every load of a wave is one contiguous kilobyte; the partial sums of all splits are requested
// before the first is used.
template <int KIND>
__global__ void __launch_bounds__(kThreads)
splitk_epilogue4_kernel(const float* __restrict__ partial, int splits, int M, int N, GemmEpilogue ep) {
    const int groups = N >> 2;
    const int64_t gid = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (gid >= static_cast<int64_t>(M) * groups) return;
    const int row = static_cast<int>(gid / groups), col0 = static_cast<int>(gid - static_cast<int64_t>(row) * groups) * 4;
    const int64_t total = static_cast<int64_t>(M) * N;
    const float* src = partial + static_cast<int64_t>(row) * N + col0;
    f32x4 part[kMaxSplits];
#pragma unroll
    for (int p = 0; p < kMaxSplits; ++p)
        if (p < splits) part[p] = *reinterpret_cast<const f32x4*>(src + p * total);
    float bias[4] = {0.f, 0.f, 0.f, 0.f}, gate[4] = {1.f, 1.f, 1.f, 1.f};
    if (ep.bias) {
        const f32x4 b = *reinterpret_cast<const f32x4*>(ep.bias + col0);
#pragma unroll
        for (int e = 0; e < 4; ++e) bias[e] = b[e];
    }
    if (KIND == EPI_RESID && ep.gate) {
        const f32x4 g = *reinterpret_cast<const f32x4*>(ep.gate + col0);
#pragma unroll
        for (int e = 0; e < 4; ++e) gate[e] = g[e];
    }
    float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < kMaxSplits; ++p)
        if (p < splits) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += part[p][e];
        }
    epilogue_store_vec<KIND, 4>(ep, row, col0, v, bias, gate);
}

// [n, k] row-major -> fragment-major packed layout (rows past n are zero)
__global__ void __launch_bounds__(kThreads)
pack_weight_kernel(const bf16_t* __restrict__ w, int n, int k, bf16_t* __restrict__ wp) {
    const int64_t chunks = static_cast<int64_t>((n + 31) >> 5) * (k >> 4) * 64;   // 16-byte chunks of the packed array
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    for (int64_t c = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; c < chunks; c += stride) {
        const int lane = static_cast<int>(c & 63);
        const int64_t blk = c >> 6;
        const int kb = static_cast<int>(blk % (k >> 4));
        const int nb = static_cast<int>(blk / (k >> 4));
        const int row = nb * 32 + (lane & 31), col = kb * 16 + 8 * (lane >> 5);
        uint4 x = make_uint4(0, 0, 0, 0);
        if (row < n) x = *reinterpret_cast<const uint4*>(w + static_cast<int64_t>(row) * k + col);
        *reinterpret_cast<uint4*>(wp + c * 8) = x;
    }
}

struct GemmPlan { int tn; int splits; int variant; };   // variant 0: register-direct weights; 1, 2: both operands through LDS, 128 / 256 rows

// Picks the wave-tile width and the K split that finish soonest under a model fitted to measurements on MI355X:
// a K-step of a 128 x 256 workgroup takes about 1.05 us; a 128 x 128 workgroup takes 0.65 us alone on a CU and
// 1.1 us when two share one (its registers allow that); split-K adds a pass over the float partial sums.
GemmPlan plan_gemm(const regione_ctx* ctx, int m, int n, int k) {
    if (ctx->gemm_force_tn > 0)
        return {(ctx->gemm_force_tn - 1) % 2 + 1, ctx->gemm_force_splits > 0 ? ctx->gemm_force_splits : 1, (ctx->gemm_force_tn - 1) / 2};
    // Many rows (the full forward of a storing step) and a narrow result: the 256-row tile with both operands through
    // LDS fetches a third fewer bytes per FLOP and measured 4-5 % faster than the register kernel at 8704 rows and
    // 3072 columns.  For wide results (9216, 12288 columns) the register kernel with the wide wave tile is level or
    // up to 14 % faster at 4096-8704 rows, and at 2048 rows the eight row tiles of the 256-row kernel leave CUs idle.
    if (m >= 3072 && n >= 512 && n < 6144) return {2, 1, 2};
    const int m_tiles = (m + BM - 1) / BM, steps = k / BK;
    GemmPlan best = {2, 1, 0};
    double best_t = 1e30;
    for (int tn = 1; tn <= 2; ++tn) {
        const int n_tiles = (n + 128 * tn - 1) / (128 * tn);
        for (int s : {1, 2, 3, 4, 6, 8}) {
            if (s > 1 && (steps / s < 8 || static_cast<size_t>(s) * m * n * sizeof(float) > ctx->gemm_part_bytes)) continue;
            const int per = (steps + s - 1) / s;
            const long wgs = static_cast<long>(m_tiles) * n_tiles * s;
            const long cap = tn == 1 ? 512 : 256;
            const long full = wgs / cap, rem = wgs % cap;
            const double t_wide = s > 1 ? 1.6 : 1.05;   // measured: the wide tile loses more than the narrow one under split-K
            const double t_full = tn == 1 ? 1.1 : t_wide;
            const double t_rem = tn == 1 ? (rem <= 256 ? 0.65 : 1.1) : t_wide;
            double t = per * (full * t_full + (rem > 0 ? t_rem : 0.0)) + 4.0;
            if (s > 1) t += 3.0 + (s + 1.0) * m * n * 4.0 / 3.0e6;
            if (t < best_t) { best_t = t; best = {tn, s, 0}; }
        }
    }
    return best;
}

template <int TN, int KIND, int VARIANT>
int launch_gemm(regione_ctx* ctx, const bf16_t* a, int lda, const bf16_t* wp, int m, int n, int k, int splits, const GemmEpilogue& ep) {
    constexpr int BN = 128 * TN;
    constexpr int WM = VARIANT == 2 ? 2 : 1;
    constexpr int ROWS = BM * WM;
    const int m_tiles = (m + ROWS - 1) / ROWS, n_tiles = (n + BN - 1) / BN;
    const int tiles = m_tiles * n_tiles;
    const int tiles_per_xcd = (tiles + 7) / 8;
    const int steps = k / BK;
    const int per = (steps + splits - 1) / splits;
    const int used_splits = (steps + per - 1) / per;
    if (used_splits > 1 && static_cast<size_t>(used_splits) * m * n * sizeof(float) > ctx->gemm_part_bytes)
        RG_FAIL(REGIONE_ERR_WORKSPACE, "gemm: %d K-splits of a %d x %d result exceed the workspace", used_splits, m, n);
    float* partial = used_splits > 1 ? ctx->gemm_part : nullptr;
    // many row tiles: groups of four (measured 2-19 % faster on the 8704-row GEMMs than all row tiles of a column tile
    // in a row); few row tiles: one group, the previous order
    const int group_rows = m_tiles > 8 ? 4 : m_tiles;
    if (VARIANT != 0) {
        constexpr unsigned lds_bytes = LdsGemm<TN, WM>::LDS_BYTES;
        constexpr uint32_t grant_bit = 1u << ((TN - 1) + 2 * (WM - 1) + 4 * KIND);   // bits 0-11
        if (!(ctx->lds_grant_mask & grant_bit)) {   // per instantiation: more than 64 KiB of LDS has to be granted explicitly
            RG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_lds_kernel<TN, WM, KIND>), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes)));
            ctx->lds_grant_mask |= grant_bit;
        }
        hipLaunchKernelGGL((gemm_lds_kernel<TN, WM, KIND>), dim3(tiles_per_xcd * 8, used_splits), dim3(kThreads * WM), lds_bytes, ctx->stream,
                           a, lda, wp, m, n, k, m_tiles, n_tiles, tiles_per_xcd, group_rows, per, partial, ep);
    } else {
        hipLaunchKernelGGL((gemm_bf16_kernel<TN, KIND>), dim3(tiles_per_xcd * 8, used_splits), dim3(kThreads), 0, ctx->stream,
                           a, lda, wp, m, n, k, m_tiles, n_tiles, tiles_per_xcd, group_rows, per, partial, ep);
    }
    RG_LAUNCH_CHECK();
    if (used_splits > 1) {
        const int64_t total = static_cast<int64_t>(m) * n;
        const bool wide = ep.vec_ok && used_splits <= kMaxSplits && (!ep.bias || rg_aligned16(ep.bias)) && (!ep.gate || rg_aligned16(ep.gate));
        if (ep.merge_kind == EPI_VELOCITY) {
            int64_t blocks = (total + kThreads - 1) / kThreads;
            if (blocks > 256 * 16) blocks = 256 * 16;
            hipLaunchKernelGGL((splitk_epilogue_kernel<EPI_VELOCITY>), dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, ctx->stream,
                               partial, used_splits, m, n, ep);
        } else if (wide) {
            const int64_t blocks = (total / 4 + kThreads - 1) / kThreads;
            hipLaunchKernelGGL((splitk_epilogue4_kernel<KIND>), dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, ctx->stream,
                               partial, used_splits, m, n, ep);
        } else {
            int64_t blocks = (total + kThreads - 1) / kThreads;
            if (blocks > 256 * 16) blocks = 256 * 16;
            hipLaunchKernelGGL((splitk_epilogue_kernel<KIND>), dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, ctx->stream,
                               partial, used_splits, m, n, ep);
        }
        RG_LAUNCH_CHECK();
    }
    return REGIONE_OK;
}

// Results of at most 64 columns (the velocity head: hidden -> latent channels): a workgroup owns 32 rows x 32 columns,
// its sixteen waves split K, fragments come straight from global memory (A rows as the MFMA's row operand, the packed
// weights as they lie), the partial tiles meet in LDS and are added in wave order, and the epilogue runs on the sums.
// Such a launch is a chain of memory round trips, not arithmetic: with K over sixteen waves a wave has all its loads
// in flight at once (four waves per workgroup, twelve round trips each: 25 us at 820 x 64 x 3072 inside the step,
// slower than the general kernel's K split + merge launch, 15 + 5 us).
// KIND: EPI_PLAIN, or EPI_VELOCITY (the fresh region step's velocity cache, Euler update and latent merge).
constexpr int kSkinnyWaves = 16;
template <int KIND>
__global__ void __launch_bounds__(kSkinnyWaves * 64)
gemm_skinny_kernel(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ Wp, int M, int N, int K, GemmEpilogue ep) {
    constexpr int LDR = 32;                      // row stride of a partial tile in LDS
    __shared__ float red[kSkinnyWaves][32 * LDR];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int m0 = blockIdx.x * 32, nb = blockIdx.y;
    const int steps = K >> 4, per = (steps + kSkinnyWaves - 1) / kSkinnyWaves;
    const int s0 = wave * per;
    const int s1 = s0 + per < steps ? s0 + per : steps;
    int row = m0 + l32;
    row = row < M ? row : M - 1;                 // rows past the end repeat the last one; their sums are not stored
    const bf16_t* ap = A + static_cast<int64_t>(row) * lda + 8 * lh;
    const bf16_t* wp = Wp + (static_cast<int64_t>(nb) * steps * 64 + lane) * 8;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    // all loads of a chunk of ten K-steps are issued before its first MFMA: one memory round trip per chunk
    constexpr int CH = 10;
    for (int base = s0; base < s1; base += CH) {
        bf16x8 a[CH], w[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int sidx = base + i < s1 ? base + i : s1 - 1;     // past the end: a valid address, the product is dropped below
            a[i] = *reinterpret_cast<const bf16x8*>(ap + sidx * 16);
            w[i] = *reinterpret_cast<const bf16x8*>(wp + static_cast<int64_t>(sidx) * 512);
        }
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (base + i < s1) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], w[i], acc, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) red[wave][(8 * (r >> 2) + 4 * lh + (r & 3)) * LDR + l32] = acc[r];
    __syncthreads();
    {
        const int i = threadIdx.x;               // 32 x 32 sums, one per thread
        const int rr = i >> 5, cc = i & 31;
        const int at = rr * LDR + cc;
        float sum = red[0][at];
#pragma unroll
        for (int w = 1; w < kSkinnyWaves; ++w) sum += red[w][at];
        const int grow = m0 + rr, gcol = nb * 32 + cc;
        if (grow < M && gcol < N) epilogue_store<KIND>(ep, grow, grow, gcol, sum, ep.bias ? ep.bias[gcol] : 0.f, 1.f);
    }
}

template <int KIND>
int launch_gemm_skinny(regione_ctx* ctx, const bf16_t* a, int lda, const bf16_t* wp, int m, int n, int k, const GemmEpilogue& ep) {
    hipLaunchKernelGGL((gemm_skinny_kernel<KIND>), dim3(static_cast<unsigned>((m + 31) / 32), static_cast<unsigned>((n + 31) / 32)), dim3(kSkinnyWaves * 64), 0, ctx->stream,
                       a, lda, wp, m, n, k, ep);
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}
// the shapes the small-N kernel takes: narrow results, unless a comparison forces a plan of the general kernels
bool skinny_shape(const regione_ctx* ctx, int n) { return n <= 64 && ctx->gemm_force_tn == 0 && ctx->gemm_force_splits == 0; }

template <int KIND>
int dispatch(regione_ctx* ctx, const bf16_t* a, int lda, const bf16_t* wp, int m, int n, int k, const GemmEpilogue& ep) {
    GemmPlan p = plan_gemm(ctx, m, n, k);
    if (ep.merge_kind == EPI_VELOCITY && p.splits < 2) p.splits = 2;   // the velocity step lives in the merge kernel: there has to be one
    if (p.variant == 2) {
        if (p.tn == 1) return launch_gemm<1, KIND, 2>(ctx, a, lda, wp, m, n, k, p.splits, ep);
        return launch_gemm<2, KIND, 2>(ctx, a, lda, wp, m, n, k, p.splits, ep);
    }
    if (p.variant == 1) {
        if (p.tn == 1) return launch_gemm<1, KIND, 1>(ctx, a, lda, wp, m, n, k, p.splits, ep);
        return launch_gemm<2, KIND, 1>(ctx, a, lda, wp, m, n, k, p.splits, ep);
    }
    if (p.tn == 1) return launch_gemm<1, KIND, 0>(ctx, a, lda, wp, m, n, k, p.splits, ep);
    return launch_gemm<2, KIND, 0>(ctx, a, lda, wp, m, n, k, p.splits, ep);
}


// the wide epilogue needs every eight-column group whole (n % 8, checked by the caller) and every touched row 16-byte aligned
bool wide_epilogue_ok(const GemmEpilogue& ep, int n) {
    if (ep.kind == EPI_PLAIN) return (ep.ldy % 8 == 0) && rg_aligned16(ep.y) && (ep.act_from % 8 == 0);
    if (ep.kind == EPI_QKV) return (ep.hidden % 8 == 0) && (ep.ldq % 8 == 0) && (ep.ldkv % 8 == 0) && rg_aligned16(ep.q) && rg_aligned16(ep.k) && rg_aligned16(ep.v) &&
                                   (n <= 3 * ep.hidden || ((ep.ldy % 8 == 0) && (ep.y_col0 % 8 == 0) && rg_aligned16(ep.y)));
    if (ep.kind == EPI_RESID) return (ep.ldy % 8 == 0) && (ep.ldr % 8 == 0) && rg_aligned16(ep.y) && rg_aligned16(ep.resid);
    return false;
}

// The 8-bit GEMM: 128-row LDS kernel only.  k2 = K in pairs of E4M3 values (the kernel's unit).
template <int TN, int KIND>
int launch_gemm_fp8(regione_ctx* ctx, const bf16_t* a, int lda2, const bf16_t* wp, int m, int n, int k2, int splits, const GemmEpilogue& ep) {
    constexpr int BN = 128 * TN;
    const int m_tiles = (m + BM - 1) / BM, n_tiles = (n + BN - 1) / BN;
    const int tiles = m_tiles * n_tiles;
    const int tiles_per_xcd = (tiles + 7) / 8;
    const int steps = k2 / BK;
    const int per = (steps + splits - 1) / splits;
    const int used_splits = (steps + per - 1) / per;
    if (used_splits > 1 && static_cast<size_t>(used_splits) * m * n * sizeof(float) > ctx->gemm_part_bytes)
        RG_FAIL(REGIONE_ERR_WORKSPACE, "gemm_fp8: %d K-splits of a %d x %d result exceed the workspace", used_splits, m, n);
    float* partial = used_splits > 1 ? ctx->gemm_part : nullptr;
    const int group_rows = m_tiles > 8 ? 4 : m_tiles;
    constexpr unsigned lds_bytes = LdsGemm<TN, 1>::LDS_BYTES;
    constexpr uint32_t grant_bit = 1u << (12 + (TN - 1));   // bits 12-13: one grant covers the three epilogue kinds of a width
    if (!(ctx->lds_grant_mask & grant_bit)) {
        RG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_lds_kernel<TN, 1, EPI_PLAIN, true>), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes)));
        RG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_lds_kernel<TN, 1, EPI_QKV, true>), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes)));
        RG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_lds_kernel<TN, 1, EPI_RESID, true>), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes)));
        ctx->lds_grant_mask |= grant_bit;
    }
    hipLaunchKernelGGL((gemm_lds_kernel<TN, 1, KIND, true>), dim3(tiles_per_xcd * 8, used_splits), dim3(kThreads), lds_bytes, ctx->stream,
                       a, lda2, wp, m, n, k2, m_tiles, n_tiles, tiles_per_xcd, group_rows, per, partial, ep);
    RG_LAUNCH_CHECK();
    if (used_splits > 1) {
        const int64_t total = static_cast<int64_t>(m) * n;
        const bool wide = ep.vec_ok && used_splits <= kMaxSplits && (!ep.bias || rg_aligned16(ep.bias));
        if (wide) {
            const int64_t blocks = (total / 4 + kThreads - 1) / kThreads;
            hipLaunchKernelGGL((splitk_epilogue4_kernel<KIND>), dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, ctx->stream,
                               partial, used_splits, m, n, ep);
        } else {
            int64_t blocks = (total + kThreads - 1) / kThreads;
            if (blocks > 256 * 16) blocks = 256 * 16;
            hipLaunchKernelGGL((splitk_epilogue_kernel<KIND>), dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, ctx->stream,
                               partial, used_splits, m, n, ep);
        }
        RG_LAUNCH_CHECK();
    }
    return REGIONE_OK;
}

}  // namespace

int rg_gemm_fp8(regione_ctx* ctx, const uint8_t* a, int lda, const uint8_t* wp, int m, int n, int k, const GemmEpilogue& ep_in) {
    if (m <= 0 || n <= 0) return REGIONE_OK;
    if (k <= 0 || (k % (2 * BK)) || (lda & 15)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "gemm_fp8: k=%d must be a positive multiple of 128 and lda=%d of 16", k, lda);
    if (!rg_aligned16(a) || !rg_aligned16(wp)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "gemm_fp8: operands must be 16-byte aligned");
    if (!ep_in.row_scale || !ep_in.col_scale) RG_FAIL(REGIONE_ERR_INVALID_ARG, "gemm_fp8: both scales are needed");
    if (ep_in.kind != EPI_PLAIN && ep_in.kind != EPI_QKV && ep_in.kind != EPI_RESID) RG_FAIL(REGIONE_ERR_INVALID_ARG, "gemm_fp8: epilogue kind %d", ep_in.kind);
    ProfScope prof(ctx, REGIONE_PROF_GEMM);
    GemmEpilogue ep = ep_in;
    ep.vec_ok = (n % 8 == 0) && rg_aligned16(ep.col_scale) && wide_epilogue_ok(ep, n);
    const int k2 = k / 2, steps = k2 / BK;
    const int m_tiles = (m + BM - 1) / BM;
    // Wave tile: the wide one (fewer LDS bytes per MFMA) once it gives most CUs a workgroup; measured at 820 rows:
    // 9216 columns 34 us wide / 37 us narrow, 3072 columns 26 / 19 us.  K is split only when the narrow tile still
    // leaves half the CUs idle (every split adds a pass over float32 partial sums, which at 820 x 3072 x 12288
    // already costs what it gains).
    int tn = (static_cast<long>(m_tiles) * ((n + 255) / 256) >= 200) ? 2 : 1;
    int splits = 1;
    if (ctx->gemm_force_tn > 0) tn = (ctx->gemm_force_tn - 1) % 2 + 1;
    const long wgs = static_cast<long>(m_tiles) * ((n + 128 * tn - 1) / (128 * tn));
    while (splits < kMaxSplits && wgs * splits < 128 && steps / (splits + 1) >= 8 &&
           static_cast<size_t>(splits + 1) * m * n * sizeof(float) <= ctx->gemm_part_bytes) ++splits;
    if (ctx->gemm_force_splits > 0) splits = ctx->gemm_force_splits;
    const bf16_t* a2 = reinterpret_cast<const bf16_t*>(a);
    const bf16_t* w2 = reinterpret_cast<const bf16_t*>(wp);
#define RG_FP8(KIND) (tn == 1 ? launch_gemm_fp8<1, KIND>(ctx, a2, lda / 2, w2, m, n, k2, splits, ep) : launch_gemm_fp8<2, KIND>(ctx, a2, lda / 2, w2, m, n, k2, splits, ep))
    if (ep.kind == EPI_QKV) return RG_FP8(EPI_QKV);
    if (ep.kind == EPI_RESID) return RG_FP8(EPI_RESID);
    return RG_FP8(EPI_PLAIN);
#undef RG_FP8
}

int rg_gemm_velocity(regione_ctx* ctx, const void* a_any, int lda, const void* wp_any, int m, int n, int k, const GemmEpilogue& ep_in) {
    if (m <= 0 || n <= 0) return REGIONE_OK;
    if (ctx->f32) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "gemm: the fused velocity step is a bf16-context path");
    if (k < 2 * BK || (k % BK) || (lda & 7)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "gemm: k=%d must be a multiple of 64, at least 128, and lda=%d a multiple of 8", k, lda);
    if (!rg_aligned16(a_any) || !rg_aligned16(wp_any)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "gemm: operands must be 16-byte aligned");
    if (static_cast<size_t>(2) * m * n * sizeof(float) > ctx->gemm_part_bytes) RG_FAIL(REGIONE_ERR_WORKSPACE, "gemm: the partial sums of a %d x %d result exceed the workspace", m, n);
    ProfScope prof(ctx, REGIONE_PROF_GEMM);
    GemmEpilogue ep = ep_in;
    ep.kind = EPI_PLAIN; ep.merge_kind = EPI_VELOCITY; ep.vec_ok = 0;
    if (skinny_shape(ctx, n)) return launch_gemm_skinny<EPI_VELOCITY>(ctx, static_cast<const bf16_t*>(a_any), lda, static_cast<const bf16_t*>(wp_any), m, n, k, ep);
    return dispatch<EPI_PLAIN>(ctx, static_cast<const bf16_t*>(a_any), lda, static_cast<const bf16_t*>(wp_any), m, n, k, ep);
}

int rg_gemm(regione_ctx* ctx, const void* a_any, int lda, const void* wp_any, int m, int n, int k, const GemmEpilogue& ep_in) {
    if (m <= 0 || n <= 0) return REGIONE_OK;
    if (ctx->f32) return rg_gemm_f32(ctx, static_cast<const float*>(a_any), lda, static_cast<const float*>(wp_any), m, n, k, ep_in);
    const bf16_t* a = static_cast<const bf16_t*>(a_any);
    const bf16_t* wp = static_cast<const bf16_t*>(wp_any);
    if (k <= 0 || (k % BK) || (lda & 7)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "gemm: k=%d must be a positive multiple of 64 and lda=%d of 8", k, lda);
    if (!rg_aligned16(a) || !rg_aligned16(wp)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "gemm: operands must be 16-byte aligned");
    ProfScope prof(ctx, REGIONE_PROF_GEMM);
    GemmEpilogue ep = ep_in;
    ep.vec_ok = (n % 8 == 0) && wide_epilogue_ok(ep, n);
    if (ep.kind == EPI_PLAIN && skinny_shape(ctx, n)) return launch_gemm_skinny<EPI_PLAIN>(ctx, a, lda, wp, m, n, k, ep);
    switch (ep.kind) {
        case EPI_PLAIN: return dispatch<EPI_PLAIN>(ctx, a, lda, wp, m, n, k, ep);
        case EPI_QKV: return dispatch<EPI_QKV>(ctx, a, lda, wp, m, n, k, ep);
        case EPI_RESID: return dispatch<EPI_RESID>(ctx, a, lda, wp, m, n, k, ep);
    }
    RG_FAIL(REGIONE_ERR_INVALID_ARG, "gemm: bad epilogue kind %d", ep.kind);
}

extern "C" int64_t regione_packed_weight_elems(int32_t n, int32_t k) {
    if (n <= 0 || k <= 0) return 0;
    return static_cast<int64_t>((n + 31) / 32) * 32 * k;
}

extern "C" int regione_pack_weight(regione_ctx* ctx, const void* w, int32_t n, int32_t k, void* w_packed) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "pack_weight: null context");
    if (n <= 0 || k <= 0 || (k % BK)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "pack_weight: n=%d, k=%d (k must be a multiple of 64)", n, k);
    if (!w || !w_packed || !rg_aligned16(w) || !rg_aligned16(w_packed)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "pack_weight: null or unaligned tensor");
    if (w == w_packed) RG_FAIL(REGIONE_ERR_INVALID_ARG, "pack_weight: cannot pack in place");
    if (ctx->f32) return rg_pack_weight_f32(ctx, static_cast<const float*>(w), n, k, static_cast<float*>(w_packed));
    const int64_t chunks = regione_packed_weight_elems(n, k) / 8;
    int64_t blocks = (chunks + kThreads - 1) / kThreads;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(pack_weight_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, ctx->stream,
                       static_cast<const bf16_t*>(w), n, k, static_cast<bf16_t*>(w_packed));
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

extern "C" int regione_tune_gemm(regione_ctx* ctx, int32_t wave_tile_blocks, int32_t k_splits) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "tune_gemm: null context");
    if (wave_tile_blocks < 0 || wave_tile_blocks > 6 || k_splits < 0 || k_splits > 16) RG_FAIL(REGIONE_ERR_INVALID_ARG, "tune_gemm: wave_tile_blocks in 0..6, k_splits in 0..16");
    ctx->gemm_force_tn = wave_tile_blocks;
    ctx->gemm_force_splits = k_splits;
    return REGIONE_OK;
}

extern "C" int regione_linear(regione_ctx* ctx, const void* x, const void* w_packed, const float* b_opt,
                              int32_t m, int32_t n, int32_t k, int32_t act, int32_t out_dtype, void* y) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear: null context");
    if (m < 0 || n <= 0 || k <= 0) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear: m=%d n=%d k=%d", m, n, k);
    if (act != REGIONE_ACT_NONE && act != REGIONE_ACT_GELU_TANH) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear: bad act %d", act);
    if (out_dtype != REGIONE_BF16 && out_dtype != REGIONE_FP32) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear: bad out_dtype %d", out_dtype);
    if (k % BK) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "linear: k=%d must be a multiple of 64", k);
    if (m == 0) return REGIONE_OK;
    if (!x || !w_packed || !y) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear: null tensor");
    GemmEpilogue ep = {};
    ep.kind = EPI_PLAIN; ep.bias = b_opt; ep.act = act; ep.act_from = 0;
    ep.y = y; ep.ldy = n; ep.y_f32 = out_dtype == REGIONE_FP32;
    return rg_gemm(ctx, x, k, w_packed, m, n, k, ep);
}
