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
    int slot_period, slot_branch_rows;  // period > 0: rows [b*period, (b+1)*period) are branch b; its slots and positions repeat, its keys sit slot_branch_rows further
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
        const int branch = a.slot_period > 0 ? row / a.slot_period : 0;
        const int64_t kv_row = a.kv_slot ? static_cast<int64_t>(a.kv_slot[row - branch * a.slot_period]) + a.slot_offset + static_cast<int64_t>(branch) * a.slot_branch_rows : row;
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
        const int local = a.slot_period > 0 ? row % a.slot_period : row;   // a branch's rows sit at the same positions
        int64_t pos = a.pos_slot ? static_cast<int64_t>(a.pos_slot[local]) + a.slot_offset : a.pos0 + local;
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
                    const int32_t* pos_slot, int pos0, int slot_offset, int slot_period, int slot_branch_rows, int n, int heads, int d,
                    const float* q_norm, const float* k_norm, const float* table, int table_rows) {
    if (n <= 0 || (!q_norm && !k_norm && !table)) return REGIONE_OK;
    if (d != 64 && d != 128) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "qk_norm_rope: head dimension %d (64 or 128 supported)", d);
    if ((ldq & 7) || (ldkv & 7) || !rg_aligned16(q) || !rg_aligned16(k)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "qk_norm_rope: rows must keep 16-byte alignment");
    if ((q_norm && !rg_aligned16(q_norm)) || (k_norm && !rg_aligned16(k_norm)) || (table && !rg_aligned16(table)))
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "qk_norm_rope: weights and table must be 16-byte aligned");
    if (table && table_rows <= 0) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "qk_norm_rope: a rotation table with %d rows", table_rows);
    ProfScope prof(ctx, REGIONE_PROF_LAYERNORM);
    QkArgs a = {q, ldq, k, ldkv, kv_slot, pos_slot, pos0, slot_offset, slot_period, slot_branch_rows, n, heads, q_norm, k_norm, table, table_rows, 1e-6f};
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

namespace {
// out[b*n + i] = slot[i] + b * branch_rows: the slot list of every branch of a batched block call
__global__ void __launch_bounds__(kThreads)
expand_slots_kernel(const int32_t* __restrict__ slot, int n, int n_branches, int branch_rows, int32_t* __restrict__ out) {
    const int gid = blockIdx.x * kThreads + threadIdx.x;
    if (gid >= n * n_branches) return;
    const int b = gid / n;
    out[gid] = slot[gid - b * n] + b * branch_rows;
}
}  // namespace

int rg_expand_slots(regione_ctx* ctx, const int32_t* slot, int n, int n_branches, int branch_rows, int32_t* out) {
    if (n <= 0 || n_branches <= 0) return REGIONE_OK;
    if (static_cast<int64_t>(n_branches) * branch_rows > INT32_MAX) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "block_forward: %d branches of %d cache rows exceed 32-bit row numbers", n_branches, branch_rows);
    hipLaunchKernelGGL(expand_slots_kernel, dim3((n * n_branches + kThreads - 1) / kThreads), dim3(kThreads), 0, ctx->stream, slot, n, n_branches, branch_rows, out);
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

namespace {
// slots of the fresh rows of a region step whose text rows are recomputed: [0, n_txt) for the text rows, then
// index[i] + n_txt for the edited rows (image rows sit behind the text rows in the cached sequence)
__global__ void __launch_bounds__(kThreads)
fresh_slots_kernel(const int32_t* __restrict__ index, const int32_t* __restrict__ n_dev, int64_t n_max, int n_txt, int32_t* __restrict__ out) {
    int64_t n = n_max;
    if (n_dev) { const int64_t nd = *n_dev; n = nd < n_max ? (nd < 0 ? 0 : nd) : n_max; }
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (i < n_txt) out[i] = static_cast<int32_t>(i);
    else if (i < n_txt + n) out[i] = index[i - n_txt] + n_txt;
}
// out = b + t * b_time, the product and the sum rounded separately
__global__ void __launch_bounds__(kThreads)
time_bias_kernel(const float* __restrict__ b, const float* __restrict__ b_time, float t, float* __restrict__ out, int n) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i < n) out[i] = __fadd_rn(b[i], __fmul_rn(t, b_time[i]));
}
}  // namespace

extern "C" int regione_fresh_slots(regione_ctx* ctx, const int32_t* index, const int32_t* n_dev, int64_t n_max, int32_t n_txt, int32_t* slots) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "fresh_slots: null context");
    if (n_max < 0 || n_txt < 0 || n_max + n_txt > INT32_MAX) RG_FAIL(REGIONE_ERR_INVALID_ARG, "fresh_slots: n_max=%lld n_txt=%d", static_cast<long long>(n_max), n_txt);
    if (n_max + n_txt == 0) return REGIONE_OK;
    if (!slots || (n_max > 0 && !index)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "fresh_slots: null list");
    const int64_t blocks = (n_max + n_txt + kThreads - 1) / kThreads;
    ProfScope prof(ctx, REGIONE_PROF_ROWS);
    hipLaunchKernelGGL(fresh_slots_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, ctx->stream, index, n_dev, n_max, n_txt, slots);
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

extern "C" int regione_time_bias(regione_ctx* ctx, const float* b, const float* b_time, float t, float* out, int32_t n) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "time_bias: null context");
    if (n < 0) RG_FAIL(REGIONE_ERR_INVALID_ARG, "time_bias: n=%d", n);
    if (n == 0) return REGIONE_OK;
    if (!b || !b_time || !out) RG_FAIL(REGIONE_ERR_INVALID_ARG, "time_bias: null vector");
    hipLaunchKernelGGL(time_bias_kernel, dim3((n + kThreads - 1) / kThreads), dim3(kThreads), 0, ctx->stream, b, b_time, t, out, n);
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

// ---- conditioning path: a block's modulation vectors come from ONE conditioning vector per step (time embedding
// through SiLU and a [6H, H] or [3H, H] matrix).  With a single input row there is nothing for the matrix cores to
// reuse: the product is bound by reading the matrix once from HBM (2 bytes per multiply-add).
namespace {

constexpr int kVecRowsPerWave = 4;

// y[r] = sum_c W[r, c] act(x[c]) + b[r].  act(x) is staged once per workgroup in LDS as float32; every wave owns
// kVecRowsPerWave consecutive rows and streams them 16 bytes per lane and row, so four independent loads are in
// flight per lane and iteration.
template <int ACT>
__global__ void __launch_bounds__(kThreads)
vec_linear_kernel(const float* __restrict__ x, const bf16_t* __restrict__ w, const float* __restrict__ b, int n, int k, float* __restrict__ y) {
    extern __shared__ __attribute__((aligned(16))) float xs[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row0 = (blockIdx.x * (kThreads / 64) + wave) * kVecRowsPerWave;
    const bf16_t* wrow[kVecRowsPerWave];
#pragma unroll
    for (int r = 0; r < kVecRowsPerWave; ++r) {
        const int row = row0 + r < n ? row0 + r : n - 1;       // rows past the end repeat the last one; never stored
        wrow[r] = w + static_cast<int64_t>(row) * k;
    }
    // the first chunk of the matrix rows is requested before the vector is staged: it does not depend on it
    int c0 = lane * 8;                                         // k is a multiple of 8: a lane's chunk is whole or absent
    bf16x8 wv[kVecRowsPerWave] = {};
    if (c0 < k) {
#pragma unroll
        for (int r = 0; r < kVecRowsPerWave; ++r) wv[r] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(wrow[r] + c0));
    }
    for (int c = threadIdx.x; c < k; c += kThreads) {
        float v = x[c];
        if (ACT == REGIONE_ACT_SILU) v = v / (1.0f + __expf(-v));
        xs[c] = v;
    }
    __syncthreads();
    float acc[kVecRowsPerWave] = {};
    while (c0 < k) {
        const int c1 = c0 + 64 * 8;
        bf16x8 wn[kVecRowsPerWave] = {};
        if (c1 < k) {                                          // the next chunk is in flight while this one is used
#pragma unroll
            for (int r = 0; r < kVecRowsPerWave; ++r) wn[r] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(wrow[r] + c1));
        }
        const f32x4 x0 = *reinterpret_cast<const f32x4*>(xs + c0), x1 = *reinterpret_cast<const f32x4*>(xs + c0 + 4);
#pragma unroll
        for (int r = 0; r < kVecRowsPerWave; ++r) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[r] += static_cast<float>(wv[r][e]) * x0[e];
                acc[r] += static_cast<float>(wv[r][4 + e]) * x1[e];
            }
            wv[r] = wn[r];
        }
        c0 = c1;
    }
#pragma unroll
    for (int r = 0; r < kVecRowsPerWave; ++r) {
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) acc[r] += __shfl_xor(acc[r], m, 64);
        if (lane == 0 && row0 + r < n) y[row0 + r] = acc[r] + (b ? b[row0 + r] : 0.f);
    }
}

// out[j] = cos(t f_j), out[dim/2 + j] = sin(t f_j), f_j = max_period^(-j / (dim/2)); formed in float64.
__global__ void __launch_bounds__(kThreads)
timestep_embedding_kernel(double t, int half, double max_period, float* __restrict__ out) {
    const int j = blockIdx.x * kThreads + threadIdx.x;
    if (j >= half) return;
    const double f = pow(max_period, -static_cast<double>(j) / half);
    out[j] = static_cast<float>(cos(t * f));
    out[half + j] = static_cast<float>(sin(t * f));
}

}  // namespace

extern "C" int regione_vec_linear(regione_ctx* ctx, const float* x, int32_t pre_act, const void* w, const float* b_opt,
                                  int32_t n, int32_t k, float* y) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "vec_linear: null context");
    if (n < 0 || k <= 0) RG_FAIL(REGIONE_ERR_INVALID_ARG, "vec_linear: n=%d k=%d", n, k);
    if (pre_act != REGIONE_ACT_NONE && pre_act != REGIONE_ACT_SILU) RG_FAIL(REGIONE_ERR_INVALID_ARG, "vec_linear: activation %d (none or SiLU on the input)", pre_act);
    if (k % 8 || k > 16384) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "vec_linear: k=%d must be a multiple of 8, at most 16384", k);
    if (n == 0) return REGIONE_OK;
    if (!x || !w || !y) RG_FAIL(REGIONE_ERR_INVALID_ARG, "vec_linear: null operand");
    if (!rg_aligned16(w)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "vec_linear: the matrix must be 16-byte aligned");
    ProfScope prof(ctx, REGIONE_PROF_GEMM);
    const int rows_per_wg = (kThreads / 64) * kVecRowsPerWave;
    const dim3 grid(static_cast<unsigned>((n + rows_per_wg - 1) / rows_per_wg));
    const size_t lds = static_cast<size_t>(k) * sizeof(float);
    const bf16_t* wb = static_cast<const bf16_t*>(w);
    if (pre_act == REGIONE_ACT_SILU) hipLaunchKernelGGL(vec_linear_kernel<REGIONE_ACT_SILU>, grid, dim3(kThreads), lds, ctx->stream, x, wb, b_opt, n, k, y);
    else hipLaunchKernelGGL(vec_linear_kernel<REGIONE_ACT_NONE>, grid, dim3(kThreads), lds, ctx->stream, x, wb, b_opt, n, k, y);
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

extern "C" int regione_timestep_embedding(regione_ctx* ctx, double t, int32_t dim, double max_period, float* out) {
    if (!ctx || !out) RG_FAIL(REGIONE_ERR_INVALID_ARG, "timestep_embedding: null context or output");
    if (dim <= 0 || (dim & 1)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "timestep_embedding: dim=%d must be positive and even", dim);
    if (!(max_period > 1.0)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "timestep_embedding: max_period=%g must exceed 1", max_period);
    const int half = dim / 2;
    hipLaunchKernelGGL(timestep_embedding_kernel, dim3((half + kThreads - 1) / kThreads), dim3(kThreads), 0, ctx->stream, t, half, max_period, out);
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}
