// Query/key extras of real editing transformers, which the paper leaves inside its black-box DiT: RMS normalisation
// over the head dimension and rotary position embedding.  A token's angles belong to its position in the FULL cached
// sequence [P | X | I], so a gathered (edited) token is rotated exactly as in the full forward and its key can be
// compared with cached keys written steps ago.
//
// Both are applied in place to the rows the QKV projection has just written (queries in the workspace, keys in their
// cache slots), one pass: 16 bytes per lane in, 16 bytes out.
#include "common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxAxes = 8;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

struct RopeAxes { int n_axes; int dims[kMaxAxes]; };

// table[row, 0:d/2] = cos(angle), table[row, d/2:d] = sin(angle); pair j of an axis of dimension a turns by
// pos * theta^(-2j/a), the axes' pairs follow each other.  Angles in double, rounded once to float32.
__global__ void __launch_bounds__(kThreads)
rope_table_kernel(const int32_t* __restrict__ pos_ids, int64_t n, RopeAxes axes, int half, double theta, float* __restrict__ table) {
    const int64_t gid = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (gid >= n * half) return;
    const int64_t row = gid / half;
    int j = static_cast<int>(gid - row * half);
    const int pair = j;
    int ax = 0;
    while (ax < axes.n_axes - 1 && j >= axes.dims[ax] / 2) { j -= axes.dims[ax] / 2; ++ax; }
    const double freq = pow(theta, -2.0 * j / axes.dims[ax]);
    const double angle = static_cast<double>(pos_ids[row * axes.n_axes + ax]) * freq;
    table[row * 2 * half + pair] = static_cast<float>(cos(angle));
    table[row * 2 * half + half + pair] = static_cast<float>(sin(angle));
}

struct QkArgs {
    bf16_t* q; int ldq;                 // [n, heads*D] rows of queries
    bf16_t* k; int ldkv;                // keys: row kv_slot[i] + slot_offset (row i when kv_slot is null)
    const int32_t* kv_slot;
    const int32_t* pos_slot; int pos0;  // table row of row i: pos_slot[i] + slot_offset, or pos0 + i
    int slot_offset;
    int n, heads;
    const float* q_norm; const float* k_norm;   // [D] or null (no normalisation of that side)
    const float* table; int table_rows;         // [table_rows, D] or null (no rotation)
    float eps;
};

// D/8 lanes per (row, query-or-key, head) vector.
template <int D>
__global__ void __launch_bounds__(kThreads)
qk_norm_rope_kernel(QkArgs a) {
    constexpr int LPV = D / 8, VPW = kThreads / LPV;
    const int sub = threadIdx.x % LPV;
    const int64_t vec = static_cast<int64_t>(blockIdx.x) * VPW + threadIdx.x / LPV;
    const int64_t total = static_cast<int64_t>(a.n) * 2 * a.heads;
    if (vec >= total) return;           // whole lane groups leave together: the shuffles below stay inside a group
    const int head = static_cast<int>(vec % a.heads);
    const int which = static_cast<int>((vec / a.heads) & 1);
    const int row = static_cast<int>(vec / (2 * a.heads));
    const float* w = which ? a.k_norm : a.q_norm;
    if (!w && !a.table) return;
    bf16_t* p;
    if (which == 0) p = a.q + static_cast<int64_t>(row) * a.ldq + head * D + sub * 8;
    else {
        const int64_t kv_row = a.kv_slot ? static_cast<int64_t>(a.kv_slot[row]) + a.slot_offset : row;
        p = a.k + kv_row * a.ldkv + head * D + sub * 8;
    }
    const bf16x8 in = *reinterpret_cast<const bf16x8*>(p);
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = static_cast<float>(in[e]);
    if (w) {
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += x[e] * x[e];
#pragma unroll
        for (int m = 1; m < LPV; m <<= 1) ss += __shfl_xor(ss, m, 64);
        const float rinv = rsqrtf(ss / D + a.eps);
        const f32x4 w0 = *reinterpret_cast<const f32x4*>(w + sub * 8), w1 = *reinterpret_cast<const f32x4*>(w + sub * 8 + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { x[e] *= rinv * w0[e]; x[4 + e] *= rinv * w1[e]; }
    }
    if (a.table) {
        int64_t pos = a.pos_slot ? static_cast<int64_t>(a.pos_slot[row]) + a.slot_offset : a.pos0 + row;
        pos = pos < 0 ? 0 : (pos >= a.table_rows ? a.table_rows - 1 : pos);   // never read outside the table
        const float* t = a.table + pos * D + sub * 4;
        const f32x4 c = *reinterpret_cast<const f32x4*>(t), s = *reinterpret_cast<const f32x4*>(t + D / 2);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float u = x[2 * j], v = x[2 * j + 1];
            x[2 * j] = u * c[j] - v * s[j];
            x[2 * j + 1] = u * s[j] + v * c[j];
        }
    }
    bf16x8 out;
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = static_cast<__bf16>(x[e]);
    *reinterpret_cast<bf16x8*>(p) = out;
}

}  // namespace

int rg_qk_norm_rope(regione_ctx* ctx, bf16_t* q, int ldq, bf16_t* k, int ldkv, const int32_t* kv_slot,
                    const int32_t* pos_slot, int pos0, int slot_offset, int n, int heads, int d,
                    const float* q_norm, const float* k_norm, const float* table, int table_rows) {
    if (n <= 0 || (!q_norm && !k_norm && !table)) return REGIONE_OK;
    if (d != 64 && d != 128) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "qk_norm_rope: head dimension %d (64 or 128 supported)", d);
    if ((ldq & 7) || (ldkv & 7) || !rg_aligned16(q) || !rg_aligned16(k)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "qk_norm_rope: rows must keep 16-byte alignment");
    if ((q_norm && !rg_aligned16(q_norm)) || (k_norm && !rg_aligned16(k_norm)) || (table && !rg_aligned16(table)))
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "qk_norm_rope: weights and table must be 16-byte aligned");
    if (table && table_rows <= 0) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "qk_norm_rope: a rotation table with %d rows", table_rows);
    ProfScope prof(ctx, REGIONE_PROF_LAYERNORM);
    QkArgs a = {q, ldq, k, ldkv, kv_slot, pos_slot, pos0, slot_offset, n, heads, q_norm, k_norm, table, table_rows, 1e-6f};
    const int64_t total = static_cast<int64_t>(n) * 2 * heads;
    if (d == 128) {
        const int64_t blocks = (total + kThreads / 16 - 1) / (kThreads / 16);
        hipLaunchKernelGGL(qk_norm_rope_kernel<128>, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, ctx->stream, a);
    } else {
        const int64_t blocks = (total + kThreads / 8 - 1) / (kThreads / 8);
        hipLaunchKernelGGL(qk_norm_rope_kernel<64>, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, ctx->stream, a);
    }
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

extern "C" int regione_rope_table(regione_ctx* ctx, const int32_t* pos_ids, int64_t n, int32_t n_axes,
                                  const int32_t* axes_dims_host, float theta, float* table) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "rope_table: null context");
    if (n < 0 || n_axes <= 0 || n_axes > kMaxAxes || !axes_dims_host) RG_FAIL(REGIONE_ERR_INVALID_ARG, "rope_table: n=%lld n_axes=%d (1..%d)", static_cast<long long>(n), n_axes, kMaxAxes);
    if (!(theta > 1.0f)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "rope_table: theta=%g must exceed 1", static_cast<double>(theta));
    RopeAxes axes = {};
    axes.n_axes = n_axes;
    int sum = 0;
    for (int i = 0; i < n_axes; ++i) {
        if (axes_dims_host[i] <= 0 || (axes_dims_host[i] & 1)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "rope_table: axis %d owns %d elements (a positive even number is needed)", i, axes_dims_host[i]);
        axes.dims[i] = axes_dims_host[i];
        sum += axes_dims_host[i];
    }
    if (sum != ctx->dims.head_dim) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "rope_table: the axes own %d elements, the head dimension is %d", sum, ctx->dims.head_dim);
    if (n == 0) return REGIONE_OK;
    if (!pos_ids || !table) RG_FAIL(REGIONE_ERR_INVALID_ARG, "rope_table: null positions or table");
    const int half = sum / 2;
    const int64_t blocks = (n * half + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(rope_table_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, ctx->stream, pos_ids, n, axes, half, static_cast<double>(theta), table);
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}
