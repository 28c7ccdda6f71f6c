// The float32 context: dense projections on v_mfma_f32_32x32x2_f32 and attention with the Region-Instruction KV
// cache (Eq.6) with float32 operands, float32 sums and a float32 softmax.  This is the arithmetic of the small
// float32 configuration on which the method's path is first checked against the CPU definition at a tight
// tolerance; one simple tile shape each, written for correctness, not speed (the bf16 kernels are the fast path).
#include <cmath>
#include "common.h"

namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kThreads = 256;
constexpr int FB = 64;   // rows and columns of a workgroup tile: four waves, one 32 x 32 block each
constexpr int FK = 16;   // k elements per step

__device__ __forceinline__ float gelu_tanh_exact(float x) {
    return 0.5f * x * (1.0f + tanhf(0.7978845608028654f * (x + 0.044715f * x * x * x)));
}

__device__ __forceinline__ void put(void* base, int64_t elem, int as_f32, float v) {
    if (as_f32) static_cast<float*>(base)[elem] = v;
    else static_cast<bf16_t*>(base)[elem] = f32_to_bf16(v);
}

// The epilogue kinds of the bf16 GEMM with float32 activations: q, k, v (and y, resid where flagged) are float arrays.
template <int KIND>
__device__ __forceinline__ void store_f32(const GemmEpilogue& ep, int row, int col, float acc) {
    float val = acc + (ep.bias ? ep.bias[col] : 0.f);
    if (KIND == EPI_PLAIN) {
        if (ep.act == REGIONE_ACT_GELU_TANH && col >= ep.act_from) val = gelu_tanh_exact(val);
        put(ep.y, static_cast<int64_t>(row) * ep.ldy + col, ep.y_f32, val);
    } else if (KIND == EPI_QKV) {
        const int H = ep.hidden;
        if (col < H) {
            reinterpret_cast<float*>(ep.q)[static_cast<int64_t>(row) * ep.ldq + col] = val;
        } else if (col < 3 * H) {
            const int64_t kv_row = ep.slot ? static_cast<int64_t>(ep.slot[row]) + ep.slot_offset : row;
            if (col < 2 * H) reinterpret_cast<float*>(ep.k)[kv_row * ep.ldkv + (col - H)] = val;
            else reinterpret_cast<float*>(ep.v)[kv_row * ep.ldkv + (col - 2 * H)] = val;
        } else {
            if (ep.act == REGIONE_ACT_GELU_TANH) val = gelu_tanh_exact(val);
            put(ep.y, static_cast<int64_t>(row) * ep.ldy + ep.y_col0 + (col - 3 * H), ep.y_f32, val);
        }
    } else {  // EPI_RESID
        const int64_t ri = static_cast<int64_t>(row) * ep.ldr + col;
        const float res = ep.resid_f32 ? static_cast<const float*>(ep.resid)[ri] : bf16_to_f32(static_cast<const bf16_t*>(ep.resid)[ri]);
        const float gate = ep.gate ? ep.gate[col] : 1.f;
        put(ep.y, static_cast<int64_t>(row) * ep.ldy + col, ep.y_f32, res + gate * val);
    }
}

// C[m, n] = sum_k A[m, k] W[n, k]; A row-major float32 (lda a multiple of 4), W row-major [n, k], K a multiple of 16.
// Rows past M and columns past N are computed on a repeated valid row and never stored.
template <int KIND>
__global__ void __launch_bounds__(kThreads)
gemm_f32_kernel(const float* __restrict__ A, int lda, const float* __restrict__ W, int M, int N, int K, GemmEpilogue ep) {
    __shared__ float a_lds[FB][FK + 1];   // odd row stride: the 32 rows a fragment read touches fall into 32 banks
    __shared__ float w_lds[FB][FK + 1];
    const int m0 = blockIdx.y * FB, n0 = blockIdx.x * FB;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = threadIdx.x >> 2, c4 = (threadIdx.x & 3) * 4;
    int ar = m0 + lrow; ar = ar < M ? ar : M - 1;
    int wr = n0 + lrow; wr = wr < N ? wr : N - 1;
    const float* ap = A + static_cast<int64_t>(ar) * lda + c4;
    const float* wp = W + static_cast<int64_t>(wr) * K + c4;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    for (int k0 = 0; k0 < K; k0 += FK) {
        const f32x4 av = *reinterpret_cast<const f32x4*>(ap + k0);
        const f32x4 wv = *reinterpret_cast<const f32x4*>(wp + k0);
        __syncthreads();   // every wave has finished reading the tiles of the step before
#pragma unroll
        for (int e = 0; e < 4; ++e) { a_lds[lrow][c4 + e] = av[e]; w_lds[lrow][c4 + e] = wv[e]; }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < FK / 2; ++kk) {
            // operand layout of the 32x32x2 instruction: lane l holds row (column) l % 32 at k = l / 32
            const float a = a_lds[wm * 32 + l32][2 * kk + lh];
            const float b = w_lds[wn * 32 + l32][2 * kk + lh];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
    }
    // accumulator r of a lane: row 8*(r/4) + 4*(lane/32) + r%4, column lane%32 of the wave's 32 x 32 block
    const int col = n0 + wn * 32 + l32;
    if (col >= N) return;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
        if (row < M) store_f32<KIND>(ep, row, col, acc[r]);
    }
}

__global__ void __launch_bounds__(kThreads)
pack_weight_f32_kernel(const float* __restrict__ w, int n, int n_pad, int k, float* __restrict__ wp) {
    const int64_t total = static_cast<int64_t>(n_pad) * k;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < total; i += stride)
        wp[i] = (i / k) < n ? w[i] : 0.f;
}

struct AttnF32Args {
    const float* q; int ldq; int n_q;
    const float* k0; const float* v0; int ldkv0; int n0;
    const float* k1; const float* v1; int ldkv1; int n1; const int32_t* idx1;
    float scale; float* out; int ldo;
};

// Eq.6 for one (query row, head) per wave: the key list is the fresh rows followed by the cache rows in use.  Lane j of
// the wave scores key j of a group of 64, the softmax runs online over the groups (running maximum and sum are the
// same in every lane), and lane l accumulates output elements l and l + 64.
template <int D>
__global__ void __launch_bounds__(64)
attn_f32_kernel(AttnF32Args a) {
    __shared__ float q_lds[D];
    __shared__ float p_lds[64];
    const int lane = threadIdx.x;
    const int qrow = blockIdx.x, head = blockIdx.y;
    const int n_keys = a.n0 + a.n1;
    const float* qp = a.q + static_cast<int64_t>(qrow) * a.ldq + head * D;
    for (int d = lane; d < D; d += 64) q_lds[d] = qp[d];
    __syncthreads();
    auto key_row = [&](int key, const float*& kp, const float*& vp) {
        if (key < a.n0) {
            const int64_t off = static_cast<int64_t>(key) * a.ldkv0 + head * D;
            kp = a.k0 + off; vp = a.v0 + off;
        } else {
            int64_t r = key - a.n0;
            if (a.idx1) r = a.idx1[r];
            const int64_t off = r * a.ldkv1 + head * D;
            kp = a.k1 + off; vp = a.v1 + off;
        }
    };
    float m_run = -INFINITY, l_run = 0.f;
    float o[D / 64];
#pragma unroll
    for (int i = 0; i < D / 64; ++i) o[i] = 0.f;
    for (int key0 = 0; key0 < n_keys; key0 += 64) {
        const int key = key0 + lane;
        float s = -INFINITY;
        if (key < n_keys) {
            const float* kp; const float* vp;
            key_row(key, kp, vp);
            float dot = 0.f;
#pragma unroll 8
            for (int d = 0; d < D; d += 4) {
                const f32x4 kv = *reinterpret_cast<const f32x4*>(kp + d);
                dot = fmaf(q_lds[d], kv[0], dot); dot = fmaf(q_lds[d + 1], kv[1], dot);
                dot = fmaf(q_lds[d + 2], kv[2], dot); dot = fmaf(q_lds[d + 3], kv[3], dot);
            }
            s = dot * a.scale;
        }
        float mx = s;
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
        const float m_new = fmaxf(m_run, mx);            // finite: every group holds at least one key
        const float alpha = expf(m_run - m_new);         // 0 for the first group
        const float p = key < n_keys ? expf(s - m_new) : 0.f;
        float psum = p;
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) psum += __shfl_xor(psum, m, 64);
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int i = 0; i < D / 64; ++i) o[i] *= alpha;
        p_lds[lane] = p;
        __syncthreads();
        const int live = n_keys - key0 < 64 ? n_keys - key0 : 64;
        for (int j = 0; j < live; ++j) {
            const float* kp; const float* vp;
            key_row(key0 + j, kp, vp);
            const float pj = p_lds[j];
#pragma unroll
            for (int i = 0; i < D / 64; ++i) o[i] = fmaf(pj, vp[lane + 64 * i], o[i]);
        }
        __syncthreads();   // p_lds is rewritten by the next group
    }
    float* op = a.out + static_cast<int64_t>(qrow) * a.ldo + head * D;
    const float inv = 1.0f / l_run;
#pragma unroll
    for (int i = 0; i < D / 64; ++i) op[lane + 64 * i] = o[i] * inv;
}

}  // namespace

int rg_pack_weight_f32(regione_ctx* ctx, const float* w, int n, int k, float* w_packed) {
    const int n_pad = (n + 31) / 32 * 32;
    int64_t blocks = (static_cast<int64_t>(n_pad) * k + kThreads - 1) / kThreads;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(pack_weight_f32_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, ctx->stream, w, n, n_pad, k, w_packed);
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

int rg_gemm_f32(regione_ctx* ctx, const float* a, int lda, const float* w, int m, int n, int k, const GemmEpilogue& ep) {
    if (m <= 0 || n <= 0) return REGIONE_OK;
    if (k <= 0 || (k % FK) || (lda & 3)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "gemm (float32): k=%d must be a positive multiple of 16 and lda=%d of 4", k, lda);
    if (!rg_aligned16(a) || !rg_aligned16(w)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "gemm (float32): operands must be 16-byte aligned");
    ProfScope prof(ctx, REGIONE_PROF_GEMM);
    const dim3 grid((n + FB - 1) / FB, (m + FB - 1) / FB);
    if (grid.y > 65535) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "gemm (float32): %d rows exceed this simple kernel's grid", m);
    switch (ep.kind) {
        case EPI_PLAIN: hipLaunchKernelGGL((gemm_f32_kernel<EPI_PLAIN>), grid, dim3(kThreads), 0, ctx->stream, a, lda, w, m, n, k, ep); break;
        case EPI_QKV: hipLaunchKernelGGL((gemm_f32_kernel<EPI_QKV>), grid, dim3(kThreads), 0, ctx->stream, a, lda, w, m, n, k, ep); break;
        case EPI_RESID: hipLaunchKernelGGL((gemm_f32_kernel<EPI_RESID>), grid, dim3(kThreads), 0, ctx->stream, a, lda, w, m, n, k, ep); break;
        default: RG_FAIL(REGIONE_ERR_INVALID_ARG, "gemm (float32): bad epilogue kind %d", ep.kind);
    }
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

int rg_attention_f32(regione_ctx* ctx, const float* q, int ldq, int n_q,
                     const float* k0, const float* v0, int ldkv0, int n0,
                     const float* k1, const float* v1, int ldkv1, int n1, const int32_t* idx1,
                     int heads, int d, float scale, float* out, int ldo) {
    if (n_q <= 0) return REGIONE_OK;
    if (n0 + n1 <= 0) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "attention: %d queries but no key", n_q);
    if (d != 64 && d != 128) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "attention: head dimension %d (64 or 128 supported)", d);
    if ((n0 > 0 && (ldkv0 & 3)) || (n1 > 0 && (ldkv1 & 3))) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "attention (float32): row strides must keep 16-byte alignment");
    if (heads > 65535) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "attention (float32): %d heads", heads);
    ProfScope prof(ctx, REGIONE_PROF_ATTENTION);
    AttnF32Args a = {q, ldq, n_q, k0, v0, ldkv0, n0, k1, v1, ldkv1, n1, idx1, scale > 0.f ? scale : 1.0f / sqrtf(static_cast<float>(d)), out, ldo};
    const dim3 grid(static_cast<unsigned>(n_q), static_cast<unsigned>(heads));
    if (d == 64) hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(64), 0, ctx->stream, a);
    else hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(64), 0, ctx->stream, a);
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}
