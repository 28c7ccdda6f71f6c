// 8-bit floating point (OCP E4M3) variant of the dense projections on the edited rows (section "Region-Aware
// Generation"); an extension, the paper itself computes in the model's precision.  This file: per-row quantisation
// and the entry points; the matrix-core kernel is the 8-bit form of the LDS GEMM in gemm.hip.
#include "common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

constexpr float kE4M3Max = 448.0f;

// TPR threads per row (64: four rows per workgroup, 256: one); the row stays in registers between the maximum and the
// conversion (up to 8 16-byte pieces per thread, so 4096 columns per wave and 16384 per workgroup).
//   amax = max |x|;  scale = amax / 448;  code = e4m3(clamp(x * (448 / amax), +-448)), round to nearest even
// (v_cvt_pk_fp8_f32).  The divisions are IEEE float32 divisions, the product a float32 product.
template <int TPR>
__global__ void __launch_bounds__(256)
quantize_rows_fp8_kernel(const bf16_t* __restrict__ x, int64_t rows, int cols, uint8_t* __restrict__ q, float* __restrict__ scale) {
    constexpr int MAXV = 8, RPB = 256 / TPR;
    __shared__ float wave_max[4];
    const int t = threadIdx.x % TPR;
    const int64_t row = static_cast<int64_t>(blockIdx.x) * RPB + threadIdx.x / TPR;
    const bool live_row = row < rows;      // (a workgroup of TPR = 256 has one row, so the barrier below is uniform)
    const int pieces = cols >> 3;
    const bf16x8* src = reinterpret_cast<const bf16x8*>(x + (live_row ? row : 0) * cols);
    bf16x8 v[MAXV];
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int p = i * TPR + t;
        if (live_row && p < pieces) {
            v[i] = src[p];
#pragma unroll
            for (int e = 0; e < 8; ++e) amax = __builtin_fmaxf(amax, __builtin_fabsf(static_cast<float>(v[i][e])));
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = __builtin_fmaxf(amax, __shfl_xor(amax, off, 64));
    if (TPR == 256) {
        if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = amax;
        __syncthreads();
        amax = __builtin_fmaxf(__builtin_fmaxf(wave_max[0], wave_max[1]), __builtin_fmaxf(wave_max[2], wave_max[3]));
    }
    if (!live_row) return;
    const bool live = amax > 0.f;
    const float mult = live ? kE4M3Max / amax : 1.0f;
    if (t == 0) scale[row] = live ? amax / kE4M3Max : 1.0f;
    uint2* dst = reinterpret_cast<uint2*>(q + row * cols);
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int p = i * TPR + t;
        if (p < pieces) {
            float y[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = __builtin_fminf(__builtin_fmaxf(static_cast<float>(v[i][e]) * mult, -kE4M3Max), kE4M3Max);
            unsigned lo = 0, hi = 0;
            lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], lo, false);
            lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], lo, true);
            hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], hi, false);
            hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], hi, true);
            dst[p] = make_uint2(lo, hi);
        }
    }
}

// LayerNorm + modulation (as layernorm_mod_vec_kernel in rows.hip: no affine, biased variance, eps 1e-6, two passes in
// float32, u = y * (1 + scale) + shift) with the row quantisation above applied to its float32 result while the row is
// still in registers: the bf16 rounding of u, its store and the quantiser's load of it fall away.  One wave per row.
typedef __attribute__((ext_vector_type(4))) float q_f32x4;
template <typename T> __device__ __forceinline__ void q_ld8(const T* p, float (&v)[8]);
template <> __device__ __forceinline__ void q_ld8<bf16_t>(const bf16_t* p, float (&v)[8]) {
    const bf16x8 x = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = static_cast<float>(x[e]);
}
template <> __device__ __forceinline__ void q_ld8<float>(const float* p, float (&v)[8]) {
    const q_f32x4 a = *reinterpret_cast<const q_f32x4*>(p), b = *reinterpret_cast<const q_f32x4*>(p + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { v[e] = a[e]; v[4 + e] = b[e]; }
}

template <typename T, int MAXV>
__global__ void __launch_bounds__(256)
layernorm_mod_fp8_kernel(const T* __restrict__ h, int n, int hidden, const float* __restrict__ shift, const float* __restrict__ scale,
                         uint8_t* __restrict__ q, float* __restrict__ row_scale) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    const T* hr = h + static_cast<int64_t>(row) * hidden;
    const int groups = hidden >> 3;
    float x[MAXV][8];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int g = lane + 64 * i;
        if (g < groups) {
            q_ld8<T>(hr + g * 8, x[i]);
#pragma unroll
            for (int e = 0; e < 8; ++e) sum += x[i][e];
        }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, 64);
    const float mean = sum / hidden;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        if (lane + 64 * i < groups) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float d = x[i][e] - mean; sq += d * d; }
        }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) sq += __shfl_xor(sq, m, 64);
    const float rstd = rsqrtf(sq / hidden + 1e-6f);
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int g = lane + 64 * i;
        if (g < groups) {
            float sc[8], sh[8];
            if (scale) q_ld8<float>(scale + g * 8, sc);
            if (shift) q_ld8<float>(shift + g * 8, sh);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float y = (x[i][e] - mean) * rstd;
                y = y * (1.f + (scale ? sc[e] : 0.f)) + (shift ? sh[e] : 0.f);
                x[i][e] = y;
                amax = __builtin_fmaxf(amax, __builtin_fabsf(y));
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = __builtin_fmaxf(amax, __shfl_xor(amax, off, 64));
    const bool live = amax > 0.f;
    const float mult = live ? kE4M3Max / amax : 1.0f;
    if (lane == 0) row_scale[row] = live ? amax / kE4M3Max : 1.0f;
    uint2* dst = reinterpret_cast<uint2*>(q + static_cast<int64_t>(row) * hidden);
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int g = lane + 64 * i;
        if (g < groups) {
            float y[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = __builtin_fminf(__builtin_fmaxf(x[i][e] * mult, -kE4M3Max), kE4M3Max);
            unsigned lo = 0, hi = 0;
            lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], lo, false);
            lo = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], lo, true);
            hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], hi, false);
            hi = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], hi, true);
            dst[g] = make_uint2(lo, hi);
        }
    }
}

}  // namespace

int rg_layernorm_mod_fp8(regione_ctx* ctx, const void* h, int h_f32, int n, int hidden, const float* shift, const float* scale,
                         uint8_t* q, float* row_scale) {
    if (n <= 0) return REGIONE_OK;
    if ((hidden & 7) || hidden > 4096 || hidden <= 0) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "layernorm_fp8: hidden=%d (a multiple of 8, at most 4096)", hidden);
    if (!rg_aligned16(h) || !rg_aligned16(q) || (shift && !rg_aligned16(shift)) || (scale && !rg_aligned16(scale)))
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "layernorm_fp8: tensors must be 16-byte aligned");
    ProfScope prof(ctx, REGIONE_PROF_LAYERNORM);
    const dim3 grid((n + 3) / 4);
    if (h_f32) hipLaunchKernelGGL((layernorm_mod_fp8_kernel<float, 8>), grid, dim3(256), 0, ctx->stream, static_cast<const float*>(h), n, hidden, shift, scale, q, row_scale);
    else hipLaunchKernelGGL((layernorm_mod_fp8_kernel<bf16_t, 8>), grid, dim3(256), 0, ctx->stream, static_cast<const bf16_t*>(h), n, hidden, shift, scale, q, row_scale);
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

extern "C" int regione_quantize_rows_fp8(regione_ctx* ctx, const void* x, int64_t rows, int32_t cols, void* q, float* scale) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "quantize_rows_fp8: null context");
    if (rows < 0 || cols <= 0 || (cols & 7) || cols > 16384) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "quantize_rows_fp8: rows=%lld, cols=%d (a multiple of 8, at most 16384)", (long long)rows, cols);
    if (rows == 0) return REGIONE_OK;
    if (rows > (int64_t(1) << 31)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "quantize_rows_fp8: rows=%lld too many", (long long)rows);
    if (!x || !q || !scale || !rg_aligned16(x) || !rg_aligned16(q)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "quantize_rows_fp8: null or unaligned tensor");
    ProfScope prof(ctx, REGIONE_PROF_ROWS);
    const bf16_t* xs = static_cast<const bf16_t*>(x);
    uint8_t* qs = static_cast<uint8_t*>(q);
    // short rows: a wave per row; long rows (or few of them): a workgroup per row, so that the launch fills the chip
    if (cols <= 2048 || (cols <= 4096 && rows >= 4096))
        hipLaunchKernelGGL(quantize_rows_fp8_kernel<64>, dim3(static_cast<unsigned>((rows + 3) / 4)), dim3(256), 0, ctx->stream, xs, rows, cols, qs, scale);
    else
        hipLaunchKernelGGL(quantize_rows_fp8_kernel<256>, dim3(static_cast<unsigned>(rows)), dim3(256), 0, ctx->stream, xs, rows, cols, qs, scale);
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

extern "C" int regione_pack_weight_fp8(regione_ctx* ctx, const void* wq, int32_t n, int32_t k, void* wq_packed) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "pack_weight_fp8: null context");
    if (ctx->f32) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "pack_weight_fp8: the 8-bit projections belong to bf16 contexts");
    if (n <= 0 || k <= 0 || (k % 128)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "pack_weight_fp8: n=%d, k=%d (k must be a multiple of 128)", n, k);
    // the 8-bit layout is the 16-bit one with every pair of codes taken as one element
    return regione_pack_weight(ctx, wq, n, k / 2, wq_packed);
}

extern "C" int regione_linear_fp8(regione_ctx* ctx, const void* xq, const float* x_scale, const void* wq_packed, const float* w_scale,
                                  const float* b_opt, int32_t m, int32_t n, int32_t k, int32_t act, int32_t out_dtype, void* y) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear_fp8: null context");
    if (ctx->f32) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "linear_fp8: the 8-bit projections belong to bf16 contexts");
    if (m < 0 || n <= 0 || k <= 0) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear_fp8: m=%d n=%d k=%d", m, n, k);
    if (act != REGIONE_ACT_NONE && act != REGIONE_ACT_GELU_TANH) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear_fp8: bad act %d", act);
    if (out_dtype != REGIONE_BF16 && out_dtype != REGIONE_FP32) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear_fp8: bad out_dtype %d", out_dtype);
    if (k % 128) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "linear_fp8: k=%d must be a multiple of 128", k);
    if (m == 0) return REGIONE_OK;
    if (!xq || !x_scale || !wq_packed || !w_scale || !y) RG_FAIL(REGIONE_ERR_INVALID_ARG, "linear_fp8: null tensor");
    GemmEpilogue ep = {};
    ep.kind = EPI_PLAIN; ep.bias = b_opt; ep.act = act; ep.act_from = 0;
    ep.y = y; ep.ldy = n; ep.y_f32 = out_dtype == REGIONE_FP32;
    ep.row_scale = x_scale; ep.col_scale = w_scale;
    return rg_gemm_fp8(ctx, static_cast<const uint8_t*>(xq), k, static_cast<const uint8_t*>(wq_packed), m, n, k, ep);
}
