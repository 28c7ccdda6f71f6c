// bf16 GEMM on the CDNA4 matrix cores for the block's dense projections (QKV, attention
// output, MLP up/down; section "Region-Aware Generation": the DiT runs on [X^P, X^E] only).
//
//   C[m, n] = sum_k A[m, k] * W[n, k]      A: activations [M, K], W: weights [N, K] (both K-contiguous)
//
// One workgroup (4 waves) computes a BM x BN tile with v_mfma_f32_32x32x16_bf16.  K is walked in
// steps of 64; the A and W tiles of a step are staged in LDS as rows of eight 16-byte chunks whose
// position is XOR-swizzled with the row so that the ds_read_b128 of a fragment is conflict free,
// double buffered, with the next step's global loads in flight during the MFMAs.  The MFMA "A"
// operand is the activation tile and "B" the weight tile, so a lane's accumulators belong to one
// output column and the lanes of a half-wave write 32 consecutive columns of a row.
// Workgroups are numbered so that each XCD (blockIdx % 8) owns a contiguous range of weight rows:
// every weight tile then streams through one L2 only.
#include "common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BK = 64;        // k elements per step (8 chunks of 16 bytes per row)
constexpr int kThreads = 256;

__device__ __forceinline__ float gelu_tanh_f32(float x) {
    // 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3)
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    return x / (1.0f + __expf(-2.0f * u));
}

template <int KIND>
__device__ __forceinline__ void epilogue_store(const GemmEpilogue& ep, int row, int col, float acc, float bias, float gate) {
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
            const int64_t r = ep.slot ? static_cast<int64_t>(ep.slot[row]) + ep.slot_offset : row;
            if (col < 2 * H) ep.k[r * ep.ldkv + (col - H)] = f32_to_bf16(val);
            else ep.v[r * ep.ldkv + (col - 2 * H)] = f32_to_bf16(val);
        } else {
            if (ep.act == REGIONE_ACT_GELU_TANH) val = gelu_tanh_f32(val);
            static_cast<bf16_t*>(ep.y)[static_cast<int64_t>(row) * ep.ldy + ep.y_col0 + (col - 3 * H)] = f32_to_bf16(val);
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

// Tile loader: ROWS x 64 bf16 from a K-contiguous matrix into swizzled LDS, through registers.
template <int ROWS>
struct TileLoader {
    static constexpr int PER_THREAD = ROWS * 8 / kThreads;
    uint4 regs[PER_THREAD];
    template <bool KTAIL>
    __device__ __forceinline__ void load(const bf16_t* __restrict__ base, int ld, int row0, int nrows, int k0, int K) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int idx = threadIdx.x + i * kThreads;
            const int r = idx >> 3, c = idx & 7;
            int gr = row0 + r;
            gr = gr < nrows ? gr : nrows - 1;  // rows past the end repeat the last row; their results are never stored
            const int gk = k0 + c * 8;
            if (KTAIL) {  // K not a multiple of 64: chunks past its end contribute zeros
                const bool live = gk < K;
                uint4 x = *reinterpret_cast<const uint4*>(base + static_cast<int64_t>(gr) * ld + (live ? gk : 0));
                if (!live) x = make_uint4(0, 0, 0, 0);
                regs[i] = x;
            } else {
                regs[i] = *reinterpret_cast<const uint4*>(base + static_cast<int64_t>(gr) * ld + gk);
            }
        }
    }
    __device__ __forceinline__ void store(bf16_t* lds) const {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int idx = threadIdx.x + i * kThreads;
            const int r = idx >> 3, c = idx & 7;
            *reinterpret_cast<uint4*>(lds + r * BK + ((c ^ (r & 7)) << 3)) = regs[i];
        }
    }
};

__device__ __forceinline__ bf16x8 lds_frag(const bf16_t* tile, int row, int chunk) {
    return *reinterpret_cast<const bf16x8*>(tile + row * BK + ((chunk ^ (row & 7)) << 3));
}

template <int BM, int BN, int WGM, int WGN, int KIND, bool KTAIL>
__global__ void __launch_bounds__(kThreads)
gemm_bf16_kernel(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ W, int ldw,
                 int M, int N, int K, int m_tiles, int n_tiles, int tiles_per_xcd, GemmEpilogue ep) {
    static_assert(WGM * WGN == 4, "four waves");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 32, TN = WN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    // stage s: A tile at s*STAGE, W tile right after it.  Addresses are formed from the shared base by integer
    // offsets only, so that every access is an LDS (ds_*) instruction and never a flat one.
    bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
    constexpr int STAGE = (BM + BN) * BK;

    // XCD-aware tile numbering: consecutive tiles (same weight rows, all row tiles) stay on one XCD
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    if (local >= tiles_per_xcd) return;
    const int tile = xcd * tiles_per_xcd + local;
    if (tile >= m_tiles * n_tiles) return;
    const int n_tile = tile / m_tiles, m_tile = tile - n_tile * m_tiles;
    const int m0 = m_tile * BM, n0 = n_tile * BN;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
    const int l32 = lane & 31, lh = lane >> 5;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    TileLoader<BM> la;
    TileLoader<BN> lw;
    const int k_steps = (K + BK - 1) / BK;
    la.template load<KTAIL>(A, lda, m0, M, 0, K);
    lw.template load<KTAIL>(W, ldw, n0, N, 0, K);
    la.store(smem);
    lw.store(smem + BM * BK);
    __syncthreads();
    for (int ks = 0; ks < k_steps; ++ks) {
        const int cur = ks & 1;
        // The last step re-loads its own tiles into the idle stage: unconditional code keeps the staging registers in VGPRs.
        const int k_next = (ks + 1 < k_steps ? ks + 1 : ks) * BK;
        la.template load<KTAIL>(A, lda, m0, M, k_next, K);
        lw.template load<KTAIL>(W, ldw, n0, N, k_next, K);
        const bf16_t* at = smem + cur * STAGE;
        const bf16_t* wt = at + BM * BK;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[TM], wf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = lds_frag(at, wm0 + i * 32 + l32, kk * 2 + lh);
#pragma unroll
            for (int j = 0; j < TN; ++j) wf[j] = lds_frag(wt, wn0 + j * 32 + l32, kk * 2 + lh);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[j], acc[i][j], 0, 0, 0);
        }
        la.store(smem + (cur ^ 1) * STAGE);
        lw.store(smem + (cur ^ 1) * STAGE + BM * BK);
        __syncthreads();
    }

    // accumulator (i, j, r) of a lane: row = 8*(r/4) + 4*(lane/32) + r%4, column = lane%32 of the 32x32 block
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn0 + j * 32 + l32;
        if (col >= N) continue;
        const float bias = ep.bias ? ep.bias[col] : 0.f;
        const float gate = (KIND == EPI_RESID && ep.gate) ? ep.gate[col] : 1.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm0 + i * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (row < M) epilogue_store<KIND>(ep, row, col, acc[i][j][r], bias, gate);
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN, int KIND, bool KTAIL>
int launch_gemm_k(regione_ctx* ctx, const bf16_t* a, int lda, const bf16_t* w, int ldw, int m, int n, int k, const GemmEpilogue& ep) {
    const int m_tiles = (m + BM - 1) / BM, n_tiles = (n + BN - 1) / BN;
    const int tiles = m_tiles * n_tiles;
    const int tiles_per_xcd = (tiles + 7) / 8;
    const size_t lds_bytes = static_cast<size_t>(2) * (BM + BN) * BK * sizeof(bf16_t);
    auto kern = gemm_bf16_kernel<BM, BN, WGM, WGN, KIND, KTAIL>;
    static bool attr_set = false;  // per instantiation
    if (!attr_set) {
        RG_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes)));
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(tiles_per_xcd * 8), dim3(kThreads), lds_bytes, ctx->stream,
                       a, lda, w, ldw, m, n, k, m_tiles, n_tiles, tiles_per_xcd, ep);
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

template <int BM, int BN, int WGM, int WGN, int KIND>
int launch_gemm(regione_ctx* ctx, const bf16_t* a, int lda, const bf16_t* w, int ldw, int m, int n, int k, const GemmEpilogue& ep) {
    if (k % BK) return launch_gemm_k<BM, BN, WGM, WGN, KIND, true>(ctx, a, lda, w, ldw, m, n, k, ep);
    return launch_gemm_k<BM, BN, WGM, WGN, KIND, false>(ctx, a, lda, w, ldw, m, n, k, ep);
}

template <int KIND>
int dispatch_tile(regione_ctx* ctx, const bf16_t* a, int lda, const bf16_t* w, int ldw, int m, int n, int k, const GemmEpilogue& ep) {
    // Pick the tile that keeps the most CUs busy with the least padding.
    const long t_big = static_cast<long>((m + 127) / 128) * ((n + 255) / 256);
    if (t_big >= 200 || m > 2048) return launch_gemm<128, 256, 2, 2, KIND>(ctx, a, lda, w, ldw, m, n, k, ep);
    const long t_mid = static_cast<long>((m + 127) / 128) * ((n + 127) / 128);
    if (t_mid >= 160 || m > 64) return launch_gemm<128, 128, 2, 2, KIND>(ctx, a, lda, w, ldw, m, n, k, ep);
    return launch_gemm<64, 128, 2, 2, KIND>(ctx, a, lda, w, ldw, m, n, k, ep);
}

}  // namespace

int rg_gemm(regione_ctx* ctx, const bf16_t* a, int lda, const bf16_t* w, int ldw, int m, int n, int k, const GemmEpilogue& ep) {
    if (m <= 0 || n <= 0) return REGIONE_OK;
    if (k <= 0 || (k & 7) || (lda & 7) || (ldw & 7)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "gemm: k=%d lda=%d ldw=%d must be positive multiples of 8", k, lda, ldw);
    if (!rg_aligned16(a) || !rg_aligned16(w)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "gemm: operands must be 16-byte aligned");
    ProfScope prof(ctx, REGIONE_PROF_GEMM);
    switch (ep.kind) {
        case EPI_PLAIN: return dispatch_tile<EPI_PLAIN>(ctx, a, lda, w, ldw, m, n, k, ep);
        case EPI_QKV: return dispatch_tile<EPI_QKV>(ctx, a, lda, w, ldw, m, n, k, ep);
        case EPI_RESID: return dispatch_tile<EPI_RESID>(ctx, a, lda, w, ldw, m, n, k, ep);
    }
    RG_FAIL(REGIONE_ERR_INVALID_ARG, "gemm: bad epilogue kind %d", ep.kind);
}

extern "C" int regione_linear(regione_ctx* ctx, const void* x, const void* w, const float* b_opt,
                              int32_t m, int32_t n, int32_t k, int32_t act, int32_t out_dtype, void* y) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear: null context");
    if (m < 0 || n <= 0 || k <= 0) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear: m=%d n=%d k=%d", m, n, k);
    if (act != REGIONE_ACT_NONE && act != REGIONE_ACT_GELU_TANH) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear: bad act %d", act);
    if (out_dtype != REGIONE_BF16 && out_dtype != REGIONE_FP32) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear: bad out_dtype %d", out_dtype);
    if (k % 8) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "linear: k=%d must be a multiple of 8", k);
    if (m == 0) return REGIONE_OK;
    if (!x || !w || !y) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear: null tensor");
    GemmEpilogue ep = {};
    ep.kind = EPI_PLAIN; ep.bias = b_opt; ep.act = act; ep.act_from = 0;
    ep.y = y; ep.ldy = n; ep.y_f32 = out_dtype == REGIONE_FP32;
    return rg_gemm(ctx, static_cast<const bf16_t*>(x), k, static_cast<const bf16_t*>(w), k, m, n, k, ep);
}
