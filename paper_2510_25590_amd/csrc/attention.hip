// Attention with the Region-Instruction KV cache, Eq.6:
//   O = softmax(Q [K_fresh; K_cache]^T * scale) [V_fresh; V_cache]        (per head)
// Queries are the fresh (edited / text) rows only; the key list is the fresh rows followed by the
// cache rows in use, addressed as one virtual list so that a tile may straddle the two.
//
// Flash-style streaming with an online softmax.  A workgroup of NW waves owns NW*QB*32 query rows of
// one head; each wave owns QB blocks of 32 queries, whose Q fragments stay in registers.  Keys and
// values are staged 64 rows at a time in LDS by asynchronous global->LDS copies, three stages deep.  The scores are computed
// TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: a lane then holds, for ONE query
// (column lane%32), 16 of every 32 keys, so the running maximum and the rescaling factor are
// per-lane scalars, and the exponentiated scores are already in the register layout of the "B"
// operand of the second product O^T = V^T P^T.  The V^T "A" operand (8 consecutive keys per lane
// for one d) is read from the row-major V tile with ds_read_b64_tr_b16, the transposing LDS read
// of gfx950.  The k-slot of the second product pairs lane-half h, slot s of both operands, so the
// only requirement is that both sides enumerate keys identically: slot s of half h of MFMA (kb,j)
// is key kb*32 + 16*j + 8*(s/4) + 4*h + s%4, which is exactly the row order of the S^T accumulator.
#include <cmath>
#include "common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kThreads = 256;
constexpr int KT = 64;  // keys per tile

struct AttnArgs {
    const bf16_t* q; int ldq; int n_q;
    const bf16_t* k0; const bf16_t* v0; int ldkv0; int n0;       // fresh rows
    const bf16_t* k1; const bf16_t* v1; int ldkv1; int n1;       // cache rows
    const int32_t* idx1;                                        // optional row list into the cache
    int heads; float scale_log2e;
    bf16_t* out; int ldo;
    // split-KV
    int splits; int tiles_per_split; float* part;  // [splits][heads][n_q_pad][D + 4] when splits > 1: O, maximum, sum, two unused (rows stay 16-byte aligned)
    int n_q_pad;
    int q_tiles;
};

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;   // native 16-byte vector (plain loads/stores, no memcpy)

// LDS swizzles (16-byte chunk index -> physical chunk).  K tile: the 16 rows read together with one logical chunk
// must cover all 64 banks once; rows are 256 bytes (D = 128) or 128 bytes (D = 64).  V tile: a transposing read
// touches, per lane half, 4 consecutive keys x 4 consecutive chunks.
template <int D> __device__ __forceinline__ int k_swz(int row, int chunk) {
    return D == 128 ? (chunk ^ (row & 15)) : (chunk ^ ((row >> 1) & 7));
}
template <int D> __device__ __forceinline__ int v_swz(int row, int chunk) {
    return D == 128 ? (chunk ^ ((row & 3) << 2)) : (chunk ^ (((row >> 1) & 1) << 2));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
constexpr float kRescaleSlack = 8.0f;   // log2 of the largest probability weight kept without moving the reference
// Three-input maximum in assembly (plain fmaxf costs an extra canonicalising instruction per MFMA result).  The
// compiler does not check what an assembly statement reads against the MFMAs still in flight, so the FIRST read of an
// accumulator after its last MFMA must be an ordinary expression (first_max below), which gets the required wait
// states; everything chained behind it is late enough.
__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float first_max(float a, float b) { return __builtin_fmaxf(a, b); }
// The value of lane l and of lane l ^ 32, in both lanes: gfx950's v_permlane32_swap exchanges the upper half of its
// first operand with the lower half of its second, so two copies of x become (x of the lower lane, x of the upper
// lane) everywhere.  A vector ALU instruction: no trip through the LDS as with a bpermute.
__device__ __forceinline__ void both_halves(float x, float& lo, float& hi) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const unsigned a = r[0], b = r[1];   // elements copied out before the casts: a bit cast applied to r[1] directly reads r[0]
    lo = __uint_as_float(a);
    hi = __uint_as_float(b);
}
__device__ __forceinline__ float max_across_halves(float x) { float lo, hi; both_halves(x, lo, hi); return max3(lo, hi, hi); }
__device__ __forceinline__ float sum_across_halves(float x) { float lo, hi; both_halves(x, lo, hi); return lo + hi; }

// Asynchronous global -> LDS copy of one 16-byte chunk per lane (gfx950 global_load_lds_dwordx4): lane l of the wave
// writes LDS[lds_base + 16*l].  The copy bypasses the VGPRs and is counted in vmcnt; it is written in assembly so
// that the compiler's wait-count pass does not see it (it would wait for it before every later LDS read); the kernel
// waits by hand before the barrier that publishes a stage.
__device__ __forceinline__ void async_copy16(const bf16_t* src, unsigned lds_base_bytes) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(src), "s"(lds_base_bytes) : "memory", "m0");
}

// Same copy with the address split into a wave-uniform 64-bit base (scalar registers) and a 32-bit byte offset per
// lane: the base moves from tile to tile with scalar arithmetic and the lanes' offsets never change.
__device__ __forceinline__ void async_copy16_sbase(unsigned lane_off_bytes, const bf16_t* base, unsigned lds_base_bytes) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" :: "v"(lane_off_bytes), "s"(base), "s"(lds_base_bytes) : "memory", "m0");
}

// Which rows a call reads: one contiguous array (fresh rows only, or the whole cache), fresh rows followed by cache
// rows, or cache rows picked by an index list.
enum { SRC_CONTIG = 0, SRC_TWO = 1, SRC_INDEXED = 2 };

// Issues the copies of one 64-key tile into an LDS stage.  The tile is 64 * CPR chunks; wave w issues blocks
// b = w*LD_N + i of 64 consecutive chunk positions, position P = row*CPR + physical chunk.  Since the LDS side is
// linear in the lane, the swizzle is applied on the global side: the lane that owns physical chunk p of a row loads
// the logical chunk p ^ f(row) (both swizzles are XORs, hence their own inverses).
template <int D, int NW, int MODE>
__device__ __forceinline__ void kv_tile_issue(const AttnArgs& a, int head, int key0, int n_keys, unsigned stage_base_bytes) {
    constexpr int CPR = D / 8, LD_N = KT * CPR / (NW * 64), TILE = KT * D;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // All addresses first, the copies afterwards: an index entry is an ordinary load, and a wait for it placed between
    // two copies would wait for the earlier copy as well.
    const bf16_t* ksrc[LD_N];
    const bf16_t* vsrc[LD_N];
#pragma unroll
    for (int i = 0; i < LD_N; ++i) {
        const int pos = (wave * LD_N + i) * 64 + lane;
        const int row = pos / CPR, phys = pos % CPR;
        int key = key0 + row;
        key = key < n_keys ? key : n_keys - 1;   // tail rows repeat a valid row; their scores are masked
        const bool fresh = key < a.n0;
        int64_t grow = fresh ? key : key - a.n0;
        if (MODE == SRC_INDEXED) { if (!fresh) grow = a.idx1[grow]; }
        const int64_t base = grow * (fresh ? a.ldkv0 : a.ldkv1) + head * D;
        ksrc[i] = (fresh ? a.k0 : a.k1) + base + (k_swz<D>(row, phys) << 3);
        vsrc[i] = (fresh ? a.v0 : a.v1) + base + (v_swz<D>(row, phys) << 3);
    }
#pragma unroll
    for (int i = 0; i < LD_N; ++i) asm volatile("" : "+v"(ksrc[i]), "+v"(vsrc[i]));   // pins the order: addresses, then copies
#pragma unroll
    for (int i = 0; i < LD_N; ++i) {
        const unsigned lds_blk = __builtin_amdgcn_readfirstlane(stage_base_bytes + static_cast<unsigned>(wave * LD_N + i) * 1024u);
        async_copy16(ksrc[i], lds_blk);
        async_copy16(vsrc[i], lds_blk + TILE * 2u);
    }
}
// At most N of this wave's copies still in flight.  The wait is the compiler's own builtin, not assembly: its
// wait-count pass then knows that its own earlier loads (query fragments, index entries) have landed too and does
// not put waits of its own for them into the tile loop, where they would also wait for the copies just issued.
template <int N> __device__ __forceinline__ void wait_async_copies() {
    static_assert(N >= 0 && N < 64, "vmcnt is a six-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));   // vmcnt(N), other counters untouched
    asm volatile("" ::: "memory");
}

// One 64-key tile for the QB*32 queries of a wave.  STAGE selects the LDS buffer (compile time, so that every LDS
// address is a per-lane constant plus an immediate).  K and V fragments are read once and used for all QB query blocks.
template <int D, int STAGE, int QB, bool MASK>
__device__ __forceinline__ void attn_tile(const bf16_t* smem, int t, int n_keys, float c, int lh,
                                          const int (&koff)[D / 16], const int (&voff)[D / 32], const bf16x8 (&qf)[QB][D / 16],
                                          f32x16 (&o)[QB][D / 32], float (&m_run)[QB], float (&l_run)[QB]) {
    constexpr int DB = D / 32, KK = D / 16, TILE = KT * D;
    const bf16_t* kt = smem + STAGE * 2 * TILE;
    const bf16_t* vt = kt + TILE;

    // ---- S^T = K Q^T for the two 32-key blocks
    f32x16 s[QB][2];
    f32x16 zero;
#pragma unroll
    for (int r = 0; r < 16; ++r) zero[r] = 0.f;   // becomes the inline constant 0 of the first MFMA's accumulator operand
    // K fragments are fetched two k-steps (four reads) ahead of their MFMAs
    constexpr int PF = 2;
    bf16x8 kf[KK][2];
#pragma unroll
    for (int kk = 0; kk < PF; ++kk)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) kf[kk][kb] = *reinterpret_cast<const bf16x8*>(kt + koff[kk] + kb * 32 * D);
    s16x4 vlo[DB], vhi[DB];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        if (kk + PF < KK) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) kf[kk + PF][kb] = *reinterpret_cast<const bf16x8*>(kt + koff[kk + PF] + kb * 32 * D);
        } else if (kk + PF == KK) {
            // first group of V^T fragments: in flight during the last MFMAs of S and the softmax
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                vlo[db] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vt + voff[db]));
                vhi[db] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vt + voff[db] + 8 * D));
            }
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
                s[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk][kb], qf[qb][kk], kk == 0 ? zero : s[qb][kb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- online softmax on raw scores; accumulator r of block kb is key t*64 + kb*32 + 8*(r/4) + 4*lh + r%4
    if (MASK) {   // only the last tile of the key list can run past it: the kernel peels that tile off its main loop
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (t * KT + kb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3) >= n_keys) s[qb][kb][r] = -INFINITY;
    }
    bf16x8 pf[QB][2][2];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        // maximum of the lane's 32 scores with three-input maxima (plain fmaxf costs an extra canonicalising
        // instruction per MFMA result); -inf entries of a masked tail are ordinary operands
        float mx = first_max(s[qb][0][0], s[qb][0][1]);   // waits for the last MFMA of block 0
#pragma unroll
        for (int r = 2; r < 16; r += 2) mx = max3(mx, s[qb][0][r], s[qb][0][r + 1]);
        mx = first_max(mx, s[qb][1][0]);                  // and of block 1, issued later
        mx = max3(mx, s[qb][1][1], s[qb][1][15]);
#pragma unroll
        for (int r = 2; r < 14; r += 2) mx = max3(mx, s[qb][1][r], s[qb][1][r + 1]);
        mx = max3(mx, s[qb][1][14], s[qb][1][14]);
        mx = max_across_halves(mx);
        // m_run is the REFERENCE of the exponentials, not the exact running maximum: it only moves when the tile's
        // maximum exceeds it by more than kRescaleSlack (in the log2 domain), so exp2((s - m_run) c) <= 2^kRescaleSlack
        // and the 64-multiplication rescale of the accumulators becomes rare.  Any reference gives the same quotient
        // O / l; the probabilities keep their relative precision in bf16 whatever their scale.
        const bool move = (mx - m_run[qb]) * c > kRescaleSlack;     // the first tile: m_run = -inf, always true
        float m_new = m_run[qb];
        if (__builtin_amdgcn_ballot_w64(move) != 0) {               // wave-uniform branch
            m_new = move ? mx : m_run[qb];                          // finite: every tile holds at least one live key
            const float alpha = move ? fast_exp2((m_run[qb] - m_new) * c) : 1.0f;
            l_run[qb] *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[qb][db][r] *= alpha;
            m_run[qb] = m_new;
        }
        const float neg_mc = -m_new * c;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float p = fast_exp2(__builtin_fmaf(s[qb][kb][8 * j + e], c, neg_mc));
                    psum += p;
                    pf[qb][kb][j][e] = static_cast<__bf16>(p);
                }
        l_run[qb] += psum;
    }

    // ---- O^T += V^T P^T, one (kb, j) group of DB*QB MFMAs at a time, the next group's fragments in flight
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int kb = g >> 1, j = g & 1;
        bf16x8 vf[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const s16x8 both = {vlo[db][0], vlo[db][1], vlo[db][2], vlo[db][3], vhi[db][0], vhi[db][1], vhi[db][2], vhi[db][3]};
            vf[db] = __builtin_bit_cast(bf16x8, both);
        }
        if (g < 3) {
            const int row_off = (((g + 1) >> 1) * 32 + 16 * ((g + 1) & 1)) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                vlo[db] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vt + voff[db] + row_off));
                vhi[db] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vt + voff[db] + row_off + 8 * D));
            }
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int db = 0; db < DB; ++db) o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db], pf[qb][kb][j], o[qb][db], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// NW waves per workgroup, QB blocks of 32 queries per wave, NSTAGE LDS stages.
template <int D, int NW, int QB, int NSTAGE, int WPE, int MODE>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
attn_kvcache_kernel(AttnArgs a) {
    constexpr int DB = D / 32;   // 32-wide d blocks of the output
    constexpr int KK = D / 16;   // k-steps of the first product
    constexpr int CPR = D / 8, LD_N = KT * CPR / (NW * 64), TILE = KT * D;
    constexpr int COPIES = 2 * LD_N;                    // asynchronous copies per thread and tile
    constexpr int QW = NW * QB * 32;                    // queries per workgroup
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];   // NSTAGE stages of (K tile, V tile)
    bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
    const unsigned smem_bytes0 = static_cast<unsigned>(reinterpret_cast<size_t>((__attribute__((address_space(3))) void*)(smem_raw)));   // LDS byte address

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    // XCD-aware numbering (workgroup i runs on XCD i % 8): all query tiles of one (head, key split) get consecutive
    // slots on ONE XCD, so that the K/V range they share is filled into a single L2 once instead of once per query tile.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int group = (local / a.q_tiles) * 8 + xcd;            // (head, split) pair
    if (group >= a.heads * a.splits) return;
    const int q_tile = local % a.q_tiles;
    const int head = group % a.heads;
    const int split = group / a.heads;
    const int q_base = q_tile * QW + wave * (QB * 32);
    const int n_keys = a.n0 + a.n1;
    const int n_tiles = (n_keys + KT - 1) / KT;
    const int tile_begin = split * a.tiles_per_split;
    int tile_end = tile_begin + a.tiles_per_split;
    tile_end = tile_end < n_tiles ? tile_end : n_tiles;

    // Q fragments ("B" operand): lane holds query l32 of the block, d = kk*16 + 8*lh + 0..7
    bf16x8 qf[QB][KK];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int qrow = q_base + qb * 32 + l32;
        qrow = qrow < a.n_q ? qrow : a.n_q - 1;
        const bf16_t* qp = a.q + static_cast<int64_t>(qrow) * a.ldq + head * D + 8 * lh;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qf[qb][kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16);
    }

    // per-lane LDS offsets (elements) of the fragment reads
    int koff[KK], voff[DB];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) koff[kk] = l32 * D + (k_swz<D>(l32, kk * 2 + lh) << 3);
    {
        const int src_key = 4 * lh + ((lane & 15) >> 2);      // row this lane addresses in a transposing read (plus a multiple of 8)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int d_src = db * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);   // 4 consecutive d = 8 bytes
            voff[db] = src_key * D + (v_swz<D>(src_key, d_src >> 3) << 3) + (d_src & 7);
        }
    }

    f32x16 o[QB][DB];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[qb][db][r] = 0.f;
    }
    const float c = a.scale_log2e;

    // Two LDS stages, copies one tile ahead.  Per tile: wait until this tile's copies have landed, barrier (publishes
    // them and retires the stage read one tile ago), issue the copies of the next tile into that retired stage, compute.
    // Tiles past the end re-copy the last tile so that the copy count per tile is constant.
    static_assert(NSTAGE == 2, "the tile loop below alternates two stages");
    constexpr unsigned STAGE_BYTES = 2u * TILE * 2u;
    // contiguous source: per-lane byte offsets of this thread's chunk positions inside a tile, for K and for V
    const bf16_t* const src_k = a.n0 > 0 ? a.k0 : a.k1;
    const bf16_t* const src_v = a.n0 > 0 ? a.v0 : a.v1;
    const int src_ld = a.n0 > 0 ? a.ldkv0 : a.ldkv1;
    unsigned off_k[LD_N], off_v[LD_N];
    if (MODE == SRC_CONTIG) {
#pragma unroll
        for (int i = 0; i < LD_N; ++i) {
            const int pos = (wave * LD_N + i) * 64 + lane;
            const int row = pos / CPR, phys = pos % CPR;
            const unsigned row_off = static_cast<unsigned>(row) * static_cast<unsigned>(src_ld) + static_cast<unsigned>(head * D);
            off_k[i] = (row_off + static_cast<unsigned>(k_swz<D>(row, phys) << 3)) * 2u;
            off_v[i] = (row_off + static_cast<unsigned>(v_swz<D>(row, phys) << 3)) * 2u;
        }
    }
    const unsigned wave_lds = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(wave * LD_N) * 1024u);
    auto issue_tile = [&](int t, unsigned stage_bytes) __attribute__((always_inline)) {
        const int tc = t < tile_end ? t : tile_end - 1;
        if (MODE == SRC_CONTIG && (tc + 1) * KT <= n_keys) {     // a full tile of one array: scalar base + fixed lane offsets
            const bf16_t* kb = src_k + static_cast<int64_t>(tc) * KT * src_ld;
            const bf16_t* vb = src_v + static_cast<int64_t>(tc) * KT * src_ld;
#pragma unroll
            for (int i = 0; i < LD_N; ++i) {
                const unsigned lds_blk = stage_bytes + wave_lds + static_cast<unsigned>(i) * 1024u;
                async_copy16_sbase(off_k[i], kb, lds_blk);
                async_copy16_sbase(off_v[i], vb, lds_blk + TILE * 2u);
            }
        } else {
            kv_tile_issue<D, NW, MODE == SRC_CONTIG ? SRC_TWO : MODE>(a, head, tc * KT, n_keys, stage_bytes);
        }
    };
    if (tile_begin < tile_end) issue_tile(tile_begin, smem_bytes0);
#define RG_ATTN_TILE(T, STAGE, MASK)                                                                      \
    {                                                                                                     \
        const int t_ = (T);                                                                               \
        wait_async_copies<0>();                                                                           \
        __syncthreads();                                                                                  \
        issue_tile(t_ + 1, smem_bytes0 + ((STAGE) ^ 1) * STAGE_BYTES);                                    \
        attn_tile<D, STAGE, QB, MASK>(smem, t_, n_keys, c, lh, koff, voff, qf, o, m_run, l_run);          \
    }
    // only the very last tile of the key list can be partial; it runs outside the main loop with the masking code
    const bool last_partial = tile_end * KT > n_keys;
    const int full_end = last_partial ? tile_end - 1 : tile_end;
    for (int t = tile_begin; t < full_end; t += 2) {
        RG_ATTN_TILE(t, 0, false)
        if (t + 1 < full_end) RG_ATTN_TILE(t + 1, 1, false)
    }
    if (full_end < tile_end && tile_begin < tile_end) {   // its stage follows from the number of full tiles before it
        if (((full_end - tile_begin) & 1) == 0) RG_ATTN_TILE(full_end, 0, true) else RG_ATTN_TILE(full_end, 1, true)
    }
#undef RG_ATTN_TILE
    wait_async_copies<0>();   // nothing may still be writing LDS when the workgroup ends

    // ---- finish: O^T accumulator r of d-block db: d = db*32 + 8*(r/4) + 4*lh + r%4, query = l32
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int qrow = q_base + qb * 32 + l32;
        const float l_tot = sum_across_halves(l_run[qb]);
        if (qrow >= a.n_q) continue;
        if (a.splits == 1) {
            const float inv = 1.0f / l_tot;
            bf16_t* op = a.out + static_cast<int64_t>(qrow) * a.ldo + head * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int d = db * 32 + 8 * g + 4 * lh;
                    bf16x4 pk;
#pragma unroll
                    for (int e = 0; e < 4; ++e) pk[e] = static_cast<__bf16>(o[qb][db][4 * g + e] * inv);
                    *reinterpret_cast<bf16x4*>(op + d) = pk;
                }
        } else {
            // partial result: unnormalised O, running max (log2 domain) and sum
            float* pp = a.part + ((static_cast<int64_t>(split) * a.heads + head) * a.n_q_pad + qrow) * (D + 4);
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int d = db * 32 + 8 * g + 4 * lh;
                    *reinterpret_cast<f32x4*>(pp + d) = f32x4{o[qb][db][4 * g], o[qb][db][4 * g + 1], o[qb][db][4 * g + 2], o[qb][db][4 * g + 3]};
                }
            if (lh == 0) { pp[D] = m_run[qb] * c; pp[D + 1] = l_tot; }   // maximum in the log2 domain, as the merge kernel expects
        }
    }
}

// Merges the split-KV partial results: out = sum_s 2^(m_s - m) O_s / sum_s 2^(m_s - m) l_s.
template <int D>
__global__ void __launch_bounds__(kThreads)
attn_combine_kernel(const float* __restrict__ part, int splits, int heads, int n_q, int n_q_pad, bf16_t* __restrict__ out, int ldo) {
    // one thread per (query, head, 4 d's)
    constexpr int G = D / 4;
    const int64_t gid = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t total = static_cast<int64_t>(n_q) * heads * G;
    if (gid >= total) return;
    const int g = static_cast<int>(gid % G);
    const int head = static_cast<int>((gid / G) % heads);
    const int qrow = static_cast<int>(gid / (static_cast<int64_t>(G) * heads));
    // every split's row is requested before the first value is used; a wave's loads of one split are contiguous
    constexpr int kMaxSplits = 8;
    float ms[kMaxSplits], ls[kMaxSplits];
    f32x4 val[kMaxSplits];
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s)
        if (s < splits) {
            const float* pp = part + ((static_cast<int64_t>(s) * heads + head) * n_q_pad + qrow) * (D + 4);
            const float2 ml = *reinterpret_cast<const float2*>(pp + D);
            ms[s] = ml.x; ls[s] = ml.y;
            val[s] = *reinterpret_cast<const f32x4*>(pp + 4 * g);
        }
    float m = -INFINITY;
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s)
        if (s < splits && ls[s] > 0.f) m = fmaxf(m, ms[s]);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
#pragma unroll
    for (int s = 0; s < kMaxSplits; ++s)
        if (s < splits && ls[s] > 0.f) {   // a split with l = 0 saw no key
            const float w = fast_exp2(ms[s] - m);
            l += w * ls[s];
            acc[0] += w * val[s][0]; acc[1] += w * val[s][1]; acc[2] += w * val[s][2]; acc[3] += w * val[s][3];
        }
    const float inv = 1.0f / l;
    bf16x4 pk;
#pragma unroll
    for (int e = 0; e < 4; ++e) pk[e] = static_cast<__bf16>(acc[e] * inv);
    *reinterpret_cast<bf16x4*>(out + static_cast<int64_t>(qrow) * ldo + head * D + 4 * g) = pk;
}

template <int D, int NW, int QB, int NSTAGE, int WPE>
int launch_attention(regione_ctx* ctx, AttnArgs a) {
    constexpr int QW = NW * QB * 32;
    const int q_tiles = (a.n_q + QW - 1) / QW;
    const int n_tiles = (a.n0 + a.n1 + KT - 1) / KT;
    // Key-range splits: the choice that minimises a small cost model.  The chip holds `slots` workgroups at a time;
    // a pass of workgroups costs its tiles plus a fixed prologue/epilogue (in tile times, about 2 us each with a full
    // CU); partial results cost their write and re-read.
    constexpr int wg_per_cu = WPE * 4 / NW;
    const double slots = 256.0 * wg_per_cu;
    const double wgs = static_cast<double>(q_tiles) * a.heads;
    int splits = 1;
    double best = 0.0;
    for (int s = 1; s <= 8 && (s == 1 || s * 4 <= n_tiles); ++s) {
        const double load = wgs * s / slots;
        const double passes = load <= 1.0 ? 1.0 : 0.5 * (ceil(load) + load);   // a last, partly filled pass runs faster
        const double fill = wgs * s <= 256.0 ? 0.68 : 1.0;                      // a CU with one workgroup runs it faster
        double t = passes * ((n_tiles + s - 1) / s + 4) * 2.0 * fill;
        if (s > 1) t += 3.0 + 1.5 * static_cast<double>(s) * a.n_q * a.heads * (D + 4) * 8.0 / 4.0e6;
        if (s == 1 || t < best) { best = t; splits = s; }
    }
    if (ctx->attn_force_splits > 0 && ctx->attn_force_splits * 2 <= n_tiles) splits = ctx->attn_force_splits;
    a.n_q_pad = a.n_q;
    if (splits > 1) {
        const size_t need = static_cast<size_t>(splits) * a.heads * a.n_q_pad * (D + 4) * sizeof(float);
        if (need > ctx->attn_part_bytes) splits = 1;
    }
    a.splits = splits;
    a.tiles_per_split = (n_tiles + splits - 1) / splits;
    a.part = ctx->attn_part;
    a.q_tiles = q_tiles;
    const int groups_per_xcd = (a.heads * splits + 7) / 8;
    const dim3 grid(static_cast<unsigned>(groups_per_xcd) * q_tiles * 8);
    constexpr size_t lds_bytes = static_cast<size_t>(NSTAGE) * 2 * KT * D * sizeof(bf16_t);
    constexpr uint32_t grant_bit = 1u << (24 + (D == 128 ? 1 : 0));   // bits 0-23 belong to the GEMM kernels
    if (!(ctx->lds_grant_mask & grant_bit)) {   // per instantiation: more than 64 KiB of LDS has to be granted explicitly
        RG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(attn_kvcache_kernel<D, NW, QB, NSTAGE, WPE, SRC_INDEXED>), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes)));
        RG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(attn_kvcache_kernel<D, NW, QB, NSTAGE, WPE, SRC_TWO>), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes)));
        RG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(attn_kvcache_kernel<D, NW, QB, NSTAGE, WPE, SRC_CONTIG>), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes)));
        ctx->lds_grant_mask |= grant_bit;
    }
    // a lane's byte offset inside a tile of a contiguous source has to fit 32 bits
    const int64_t src_ld = a.n0 > 0 ? a.ldkv0 : a.ldkv1;
    const bool contig = !a.idx1 && (a.n0 == 0 || a.n1 == 0) && (KT * src_ld + a.heads * D) * 2 < (int64_t{1} << 31);
    if (a.idx1) hipLaunchKernelGGL((attn_kvcache_kernel<D, NW, QB, NSTAGE, WPE, SRC_INDEXED>), grid, dim3(NW * 64), lds_bytes, ctx->stream, a);
    else if (contig) hipLaunchKernelGGL((attn_kvcache_kernel<D, NW, QB, NSTAGE, WPE, SRC_CONTIG>), grid, dim3(NW * 64), lds_bytes, ctx->stream, a);
    else hipLaunchKernelGGL((attn_kvcache_kernel<D, NW, QB, NSTAGE, WPE, SRC_TWO>), grid, dim3(NW * 64), lds_bytes, ctx->stream, a);
    RG_LAUNCH_CHECK();
    if (splits > 1) {
        const int64_t total = static_cast<int64_t>(a.n_q) * a.heads * (D / 4);
        hipLaunchKernelGGL((attn_combine_kernel<D>), dim3(static_cast<unsigned>((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, ctx->stream,
                           a.part, splits, a.heads, a.n_q, a.n_q_pad, a.out, a.ldo);
        RG_LAUNCH_CHECK();
    }
    return REGIONE_OK;
}

}  // namespace

extern "C" int regione_tune_attention(regione_ctx* ctx, int32_t key_splits) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "tune_attention: null context");
    if (key_splits < 0 || key_splits > 8) RG_FAIL(REGIONE_ERR_INVALID_ARG, "tune_attention: key_splits=%d must be 0..8", key_splits);
    ctx->attn_force_splits = key_splits;
    return REGIONE_OK;
}

int rg_attention(regione_ctx* ctx, const void* q_any, int ldq, int n_q,
                 const void* k0_any, const void* v0_any, int ldkv0, int n0,
                 const void* k1_any, const void* v1_any, int ldkv1, int n1, const int32_t* idx1,
                 int heads, int d, float scale, void* out_any, int ldo) {
    if (n_q <= 0) return REGIONE_OK;
    if (ctx->f32)
        return rg_attention_f32(ctx, static_cast<const float*>(q_any), ldq, n_q, static_cast<const float*>(k0_any), static_cast<const float*>(v0_any), ldkv0, n0,
                                static_cast<const float*>(k1_any), static_cast<const float*>(v1_any), ldkv1, n1, idx1, heads, d, scale, static_cast<float*>(out_any), ldo);
    const bf16_t* q = static_cast<const bf16_t*>(q_any);
    const bf16_t* k0 = static_cast<const bf16_t*>(k0_any); const bf16_t* v0 = static_cast<const bf16_t*>(v0_any);
    const bf16_t* k1 = static_cast<const bf16_t*>(k1_any); const bf16_t* v1 = static_cast<const bf16_t*>(v1_any);
    bf16_t* out = static_cast<bf16_t*>(out_any);
    if (n0 + n1 <= 0) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "attention: %d queries but no key", n_q);
    if (d != 64 && d != 128) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "attention: head dimension %d (64 or 128 supported)", d);
    if ((ldq & 7) || (ldo & 3) || (n0 > 0 && (ldkv0 & 7)) || (n1 > 0 && (ldkv1 & 7)))
        RG_FAIL(REGIONE_ERR_BAD_SHAPE, "attention: row strides must keep 16-byte alignment");
    ProfScope prof(ctx, REGIONE_PROF_ATTENTION);
    AttnArgs a = {};
    a.q = q; a.ldq = ldq; a.n_q = n_q;
    a.k0 = k0; a.v0 = v0; a.ldkv0 = ldkv0; a.n0 = n0;
    a.k1 = k1; a.v1 = v1; a.ldkv1 = ldkv1; a.n1 = n1; a.idx1 = idx1;
    a.heads = heads;
    a.scale_log2e = (scale > 0.f ? scale : 1.0f / sqrtf(static_cast<float>(d))) * 1.4426950408889634f;
    a.out = out; a.ldo = ldo;
    if (d == 64) return launch_attention<64, 4, 1, 2, 2>(ctx, a);
    return launch_attention<128, 4, 1, 2, 2>(ctx, a);
}

extern "C" int regione_attn_kvcache(regione_ctx* ctx, const void* q, int32_t n_q,
                                    const void* k_fresh, const void* v_fresh, int32_t n_fresh,
                                    const void* k_cache, const void* v_cache, int32_t n_c,
                                    const int32_t* cache_index_opt, int32_t n_cache_index,
                                    int32_t heads, int32_t d, float scale, void* out) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "attn_kvcache: null context");
    if (n_q < 0 || n_fresh < 0 || n_c < 0 || heads <= 0 || n_cache_index < 0)
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "attn_kvcache: n_q=%d n_fresh=%d n_c=%d heads=%d", n_q, n_fresh, n_c, heads);
    if (d != 64 && d != 128) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "attn_kvcache: head dimension %d (64 or 128 supported)", d);
    if (n_q == 0) return REGIONE_OK;
    if (!q || !out) RG_FAIL(REGIONE_ERR_INVALID_ARG, "attn_kvcache: null q or out");
    if (n_fresh > 0 && (!k_fresh || !v_fresh)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "attn_kvcache: null fresh K/V");
    if (n_c > 0 && (!k_cache || !v_cache)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "attn_kvcache: null cache");
    const int n1 = cache_index_opt ? n_cache_index : n_c;
    if (cache_index_opt && n_c == 0 && n_cache_index > 0) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "attn_kvcache: index list into an empty cache");
    if (n_fresh + n1 == 0) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "attn_kvcache: %d queries but no key", n_q);
    if (!rg_aligned16(q) || !rg_aligned16(out) || !rg_aligned16(k_fresh) || !rg_aligned16(v_fresh) || !rg_aligned16(k_cache) || !rg_aligned16(v_cache))
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "attn_kvcache: tensors must be 16-byte aligned");
    const int ld = heads * d;
    return rg_attention(ctx, q, ld, n_q, k_fresh, v_fresh, ld, n_fresh, k_cache, v_cache, ld, n1, cache_index_opt, heads, d, scale, out, ld);
}
