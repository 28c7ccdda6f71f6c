// Matrix-core peak probe (measurement aid, not part of the method): register-only MFMA loops, timed like every other
// launch of the library, so that the achieved TFLOP/s of the GEMM and attention kernels can be read against what the
// chip sustains at the clock it holds under load instead of the nominal 2.4 GHz figure.
#include "common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ unsigned mix(unsigned x) {   // a small integer hash: operand bits that differ per lane
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

template <int FORMAT>
__global__ void __launch_bounds__(256)
mfma_peak_kernel(int iters, float* __restrict__ out) {
    const unsigned gid = blockIdx.x * 256 + threadIdx.x;
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    if (FORMAT == 0) {
        // bf16 pairs with biased exponent 120-123 (|x| in [2^-7, 2^-3)): random mantissas and signs, no NaN, no infinity
        bf16x8 a[4], b;
        u32x4 raw;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int e = 0; e < 4; ++e) raw[e] = (mix(gid * 16 + j * 4 + e) & 0x81ff81ffu) | 0x3c003c00u;
            a[j] = __builtin_bit_cast(bf16x8, raw);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) raw[e] = (mix(gid * 16 + 77 + e) & 0x81ff81ffu) | 0x3c003c00u;
        b = __builtin_bit_cast(bf16x8, raw);
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b, acc[j], 0, 0, 0);
        }
    } else {
        // E4M3 bytes with bit 6 cleared: |x| < 2, never the NaN code
        i32x8 a[4], b;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) a[j][e] = static_cast<int>(mix(gid * 64 + j * 8 + e) & 0xbfbfbfbfu);
#pragma unroll
        for (int e = 0; e < 8; ++e) b[e] = static_cast<int>(mix(gid * 64 + 99 + e) & 0xbfbfbfbfu);
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[j], b, acc[j], 0, 0, 0, 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    out[gid] = s;
}

}  // namespace

extern "C" int regione_mfma_peak_probe(regione_ctx* ctx, int32_t format, int32_t iters, int32_t n_workgroups, float* out, double* flops_host) {
    if (!ctx || !out || !flops_host) RG_FAIL(REGIONE_ERR_INVALID_ARG, "mfma_peak_probe: null argument");
    if ((format != 0 && format != 1) || iters < 1 || iters > (1 << 22) || n_workgroups < 1 || n_workgroups > (1 << 16))
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "mfma_peak_probe: format=%d iters=%d n_workgroups=%d", format, iters, n_workgroups);
    ProfScope prof(ctx, REGIONE_PROF_GEMM);
    if (format == 0) hipLaunchKernelGGL(mfma_peak_kernel<0>, dim3(n_workgroups), dim3(256), 0, ctx->stream, iters, out);
    else hipLaunchKernelGGL(mfma_peak_kernel<1>, dim3(n_workgroups), dim3(256), 0, ctx->stream, iters, out);
    RG_LAUNCH_CHECK();
    *flops_host = static_cast<double>(n_workgroups) * 4.0 * iters * 4.0 * 2.0 * 32.0 * 32.0 * (format == 0 ? 16.0 : 64.0);
    return REGIONE_OK;
}
