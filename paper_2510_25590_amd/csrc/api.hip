// Context and the composition of one transformer block out of the library's kernels.  (Error reporting and the pure
// host functions - stage plan, cache decisions, gamma fit - live in host_logic.cpp, which needs no GPU toolchain.)
#include <cstdlib>
#include <functional>
#include <algorithm>
#include <vector>
#include "common.h"
#include <string.h>
#include <new>
#include <math.h>

namespace {
template <typename T>
int dev_alloc(T** p, size_t count) {
    *p = nullptr;
    if (count == 0) return REGIONE_OK;
    RG_HIP(hipMalloc(reinterpret_cast<void**>(p), count * sizeof(T)));
    return REGIONE_OK;
}
void free_all(regione_ctx* c) {
    void* ptrs[] = {c->part_counts, c->u, c->q, c->kf, c->vf, c->a, c->h1, c->m, c->slot_all, c->mod_ws, c->attn_part, c->gemm_part, c->q8, c->q8_scale};
    for (void* p : ptrs) if (p) (void)hipFree(p);
    if (c->n_edited_pinned) (void)hipHostFree(c->n_edited_pinned);
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    if (c->side_stream) (void)hipStreamDestroy(c->side_stream);
    if (c->prof_ev) {
        for (int i = 0; i < 2 * c->prof_cap; ++i) if (c->prof_ev[i]) (void)hipEventDestroy(c->prof_ev[i]);
        delete[] c->prof_ev;
    }
    delete[] c->prof_class;
}
}  // namespace

extern "C" int regione_create(regione_ctx** out, const regione_dims* dims, void* hip_stream) {
    if (!out || !dims) RG_FAIL(REGIONE_ERR_INVALID_ARG, "create: null argument");
    *out = nullptr;
    if (dims->hidden <= 0 || dims->heads <= 0 || dims->head_dim <= 0 || dims->mlp <= 0 || dims->max_fresh < 0 || dims->max_tokens < 0)
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "create: sizes must be positive");
    if (dims->hidden != dims->heads * dims->head_dim)
        RG_FAIL(REGIONE_ERR_BAD_SHAPE, "create: hidden %d != heads %d * head_dim %d", dims->hidden, dims->heads, dims->head_dim);
    if (dims->head_dim != 64 && dims->head_dim != 128)
        RG_FAIL(REGIONE_ERR_UNSUPPORTED, "create: head dimension %d (64 or 128 supported)", dims->head_dim);
    if (dims->hidden % 64 || dims->mlp % 64) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "create: hidden and mlp must be multiples of 64");
    if (dims->compute_dtype != REGIONE_BF16 && dims->compute_dtype != REGIONE_FP32)
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "create: compute_dtype %d (REGIONE_BF16 or REGIONE_FP32)", dims->compute_dtype);
    regione_ctx* c = new (std::nothrow) regione_ctx();
    if (!c) RG_FAIL(REGIONE_ERR_HIP, "create: out of host memory");
    memset(c, 0, sizeof(*c));
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->dims = *dims;
    c->f32 = dims->compute_dtype == REGIONE_FP32;
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; RG_FAIL(REGIONE_ERR_HIP, "create: no HIP device"); }
    const size_t n = static_cast<size_t>(dims->max_fresh), H = dims->hidden, M = dims->mlp;
    const size_t es = c->f32 ? 4 : 2;   // bytes per activation element
    c->part_counts_cap = rg_partition_scratch_ints(dims->max_tokens);   // per-block counts and one decision bit per token
    const size_t split_rows = n < 2048 ? n : 2048;
    c->attn_part_bytes = static_cast<size_t>(8) * dims->heads * split_rows * (dims->head_dim + 4) * sizeof(float);
    int rc = dev_alloc(&c->part_counts, static_cast<size_t>(c->part_counts_cap));
    if (rc == REGIONE_OK) rc = dev_alloc(&c->u, n * H * es);
    if (rc == REGIONE_OK) rc = dev_alloc(&c->q, n * H * es);
    if (rc == REGIONE_OK) rc = dev_alloc(&c->kf, n * H * es);
    if (rc == REGIONE_OK) rc = dev_alloc(&c->vf, n * H * es);
    if (rc == REGIONE_OK) rc = dev_alloc(&c->a, n * (H + M) * es);
    if (rc == REGIONE_OK) rc = dev_alloc(&c->h1, n * H);
    if (rc == REGIONE_OK) rc = dev_alloc(&c->m, n * M * es);
    if (rc == REGIONE_OK) rc = dev_alloc(&c->slot_all, n);
    if (rc == REGIONE_OK) rc = dev_alloc(&c->mod_ws, static_cast<size_t>(12) * H);
    if (rc == REGIONE_OK) rc = dev_alloc(reinterpret_cast<char**>(&c->attn_part), c->attn_part_bytes);
    c->gemm_part_bytes = n > 0 ? static_cast<size_t>(128) << 20 : 0;
    if (rc == REGIONE_OK) rc = dev_alloc(reinterpret_cast<char**>(&c->gemm_part), c->gemm_part_bytes);
    if (rc == REGIONE_OK) {   // pinned, device-visible host word for the edited-token count (saves the device-to-host copy)
        void* host = nullptr; void* dev = nullptr;
        if (hipHostMalloc(&host, 64, hipHostMallocMapped) != hipSuccess || hipHostGetDevicePointer(&dev, host, 0) != hipSuccess) {
            if (host) (void)hipHostFree(host);
            free_all(c); delete c;
            RG_FAIL(REGIONE_ERR_HIP, "create: cannot allocate pinned host memory");
        }
        c->n_edited_pinned = static_cast<int32_t*>(host);
        c->n_edited_pinned_dev = static_cast<int32_t*>(dev);
        c->n_edited_pinned[0] = 0;      // the count ...
        c->n_edited_pinned[1] = 0;      // ... and the ticket of the call it belongs to (recycled pinned memory may hold an old context's ticket)
    }
    if (rc == REGIONE_OK) rc = rg_partition_static_warm();   // so that regione_partition_static's first call has nothing to set up
    if (rc != REGIONE_OK) { free_all(c); delete c; return rc; }
    *out = c;
    return REGIONE_OK;
}

extern "C" int regione_destroy(regione_ctx* ctx) {
    if (!ctx) return REGIONE_OK;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->side_stream) (void)hipStreamSynchronize(ctx->side_stream);
    free_all(ctx);
    delete ctx;
    return REGIONE_OK;
}

extern "C" int regione_profile_enable(regione_ctx* ctx, int32_t on) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "profile_enable: null context");
    if (on && !ctx->prof_ev) {
        ctx->prof_cap = 8192;
        ctx->prof_ev = new (std::nothrow) hipEvent_t[2 * ctx->prof_cap]();
        ctx->prof_class = new (std::nothrow) int[ctx->prof_cap]();
        if (!ctx->prof_ev || !ctx->prof_class) RG_FAIL(REGIONE_ERR_HIP, "profile_enable: out of host memory");
        for (int i = 0; i < 2 * ctx->prof_cap; ++i) RG_HIP(hipEventCreate(&ctx->prof_ev[i]));
    }
    ctx->prof_on = on ? 1 : 0;
    return REGIONE_OK;
}

extern "C" int regione_profile_read(regione_ctx* ctx, double* total_ms_host, int64_t* launches_host, int32_t n_classes) {
    if (!ctx || !total_ms_host || !launches_host || n_classes <= 0) RG_FAIL(REGIONE_ERR_INVALID_ARG, "profile_read: null argument");
    for (int i = 0; i < n_classes; ++i) { total_ms_host[i] = 0.0; launches_host[i] = 0; }
    RG_HIP(hipStreamSynchronize(ctx->stream));
    for (int s = 0; s < ctx->prof_used; ++s) {
        float ms = 0.f;
        RG_HIP(hipEventElapsedTime(&ms, ctx->prof_ev[2 * s], ctx->prof_ev[2 * s + 1]));
        const int k = ctx->prof_class[s];
        if (k >= 0 && k < n_classes) { total_ms_host[k] += ms; launches_host[k] += 1; }
    }
    ctx->prof_used = 0;
    return REGIONE_OK;
}

extern "C" int regione_layernorm(regione_ctx* ctx, const void* h, int32_t h_dtype, int32_t n, int32_t hidden,
                                 const float* shift_opt, const float* scale_opt, void* u) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "layernorm: null context");
    if (n < 0 || hidden <= 0) RG_FAIL(REGIONE_ERR_INVALID_ARG, "layernorm: n=%d hidden=%d", n, hidden);
    if (h_dtype != REGIONE_BF16 && h_dtype != REGIONE_FP32) RG_FAIL(REGIONE_ERR_INVALID_ARG, "layernorm: bad dtype %d", h_dtype);
    if (n == 0) return REGIONE_OK;
    if (!h || !u) RG_FAIL(REGIONE_ERR_INVALID_ARG, "layernorm: null tensor");
    return rg_layernorm_mod(ctx, h, h_dtype == REGIONE_FP32, n, hidden, shift_opt, scale_opt, u);
}

// Velocity head of the step, fused with what follows it in a fresh region step: v = h W^T + b in the storage type, the
// velocity cache takes v (Eq.9, fresh branch), x_e <- x_e - dt v (Eq.4), and the updated rows are written to their
// positions in the full latent (the merge).  One GEMM launch and one merge launch in bf16 contexts.
extern "C" int regione_velocity_head(regione_ctx* ctx, const void* h_rows, const void* w_head_packed, const float* b_head_opt,
                                     int32_t n, int32_t c, int32_t hidden, float dt, void* v_out_opt, void* c_a, void* x_e,
                                     void* x_full_opt, const int32_t* index_opt, int32_t dtype) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "velocity_head: null context");
    if (n < 0 || c <= 0 || hidden <= 0) RG_FAIL(REGIONE_ERR_INVALID_ARG, "velocity_head: n=%d c=%d hidden=%d", n, c, hidden);
    if (dtype != REGIONE_BF16 && dtype != REGIONE_FP32) RG_FAIL(REGIONE_ERR_INVALID_ARG, "velocity_head: bad dtype %d", dtype);
    if (n == 0) return REGIONE_OK;
    if (!h_rows || !w_head_packed || !c_a || !x_e) RG_FAIL(REGIONE_ERR_INVALID_ARG, "velocity_head: null tensor");
    if (x_full_opt && !index_opt) RG_FAIL(REGIONE_ERR_INVALID_ARG, "velocity_head: a full latent needs the index list");
    if (ctx->f32 || hidden < 128) {
        // float32 contexts (and heads too short to split): the three calls the fused path stands for; v needs a place
        void* v = v_out_opt ? v_out_opt : c_a;      // the cache receives the fresh velocity anyway
        if (int rc = regione_linear(ctx, h_rows, w_head_packed, b_head_opt, n, c, hidden, REGIONE_ACT_NONE, dtype, v)) return rc;
        if (int rc = regione_velocity_cache(ctx, 0, 1.0f, dt, v, c_a, nullptr, x_e, nullptr, n, c, dtype)) return rc;
        if (x_full_opt) return regione_scatter(ctx, x_full_opt, c, dtype, index_opt, nullptr, n, x_e);
        return REGIONE_OK;
    }
    GemmEpilogue ep = {};
    ep.bias = b_head_opt; ep.y = v_out_opt; ep.ldy = c; ep.y_f32 = dtype == REGIONE_FP32;
    ep.vel_ca = c_a; ep.vel_xe = x_e; ep.vel_xfull = x_full_opt; ep.vel_index = index_opt; ep.vel_dt = dt;
    return rg_gemm_velocity(ctx, h_rows, hidden, w_head_packed, n, c, hidden, ep);
}

extern "C" int regione_region_step(regione_ctx* ctx, const regione_region_step_args* a, int32_t* n_edited_host) {
    if (!ctx || !a || !n_edited_host) RG_FAIL(REGIONE_ERR_INVALID_ARG, "region_step: null argument");
    if (a->n_blocks < 0 || a->n_txt_fresh < 0) RG_FAIL(REGIONE_ERR_INVALID_ARG, "region_step: n_blocks=%d n_txt_fresh=%d", a->n_blocks, a->n_txt_fresh);
    if (a->h_dtype != REGIONE_BF16 && a->h_dtype != REGIONE_FP32) RG_FAIL(REGIONE_ERR_INVALID_ARG, "region_step: bad h_dtype %d", a->h_dtype);
    if (a->n_tokens > 0 && (!a->h_full || !a->h_rows || !a->h_rows_out || !a->x_e || !a->c_a || !a->x_next_full || !a->w_head_packed))
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "region_step: null tensor");
    if (a->n_blocks > 0 && (!a->blocks || !a->block_types || !a->k_caches || !a->v_caches)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "region_step: null block array");
    if (a->n_txt_fresh > 0 && !a->slots) RG_FAIL(REGIONE_ERR_INVALID_ARG, "region_step: fresh text rows need the slot list");
    const int H = ctx->dims.hidden;
    int32_t n = 0;
    if (int rc = rg_partition_early_count(ctx, a->x_t, a->v, a->x_ref, a->n_tokens, a->c, a->dtype, a->sigma_t, a->eta, a->score_opt, a->mask,
                                          a->e_index, a->u_index, a->n_edited_dev, &n)) return rc;
    *n_edited_host = n;
    if (n == 0) return REGIONE_OK;
    const size_t h_es = a->h_dtype == REGIONE_FP32 ? 4 : 2;
    const size_t txt_bytes = static_cast<size_t>(a->n_txt_fresh) * H * h_es;
    char* rows_in = static_cast<char*>(a->h_rows) + txt_bytes;          // the gathered rows follow the text rows
    if (int rc = regione_gather_pair(ctx, a->h_full, H, a->h_dtype, rows_in, a->x_t, a->c, a->dtype, a->x_e, a->e_index, a->n_edited_dev, n)) return rc;
    const int32_t* slot_index = a->e_index;
    int32_t slot_offset = a->slot_offset;
    if (a->n_txt_fresh > 0) {
        if (int rc = regione_fresh_slots(ctx, a->e_index, a->n_edited_dev, n, a->n_txt_fresh, a->slots)) return rc;
        slot_index = a->slots; slot_offset = 0;
    }
    const void* in = a->h_rows;
    for (int b = 0; b < a->n_blocks; ++b) {
        if (int rc = regione_block_forward(ctx, &a->blocks[b], a->block_types[b], in, a->h_rows_out, a->h_dtype, a->n_txt_fresh + n, a->n_txt_fresh,
                                           slot_index, slot_offset, a->k_caches[b], a->v_caches[b], a->n_all, REGIONE_FLAG_RETRIEVE)) return rc;
        in = a->h_rows_out;
    }
    const char* rows_out = static_cast<const char*>(in) + txt_bytes;
    if (int rc = regione_velocity_head(ctx, rows_out, a->w_head_packed, a->b_head_opt, n, a->c, H, a->dt, a->v_out_opt, a->c_a, a->x_e,
                                       a->x_next_full, a->e_index, a->dtype)) return rc;
    if (a->h_next_full_opt) return regione_scatter(ctx, a->h_next_full_opt, H, a->h_dtype, a->e_index, a->n_edited_dev, n, rows_out);
    return REGIONE_OK;
}

namespace {

// The second lane: its stream and events exist from the first call that wants them.
int ensure_side_lane(regione_ctx* ctx) {
    if (ctx->side_stream) return REGIONE_OK;
    RG_HIP(hipStreamCreateWithFlags(&ctx->side_stream, hipStreamNonBlocking));   // default priority
    RG_HIP(hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming));
    RG_HIP(hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming));
    return REGIONE_OK;
}
// The side lane starts after everything enqueued on the main stream so far ...
int lane_fork(regione_ctx* ctx) {
    RG_HIP(hipEventRecord(ctx->ev_fork, ctx->stream));
    RG_HIP(hipStreamWaitEvent(ctx->side_stream, ctx->ev_fork, 0));
    return REGIONE_OK;
}
// ... and the main stream goes on after everything enqueued on the side lane.
int lane_join(regione_ctx* ctx) {
    RG_HIP(hipEventRecord(ctx->ev_join, ctx->side_stream));
    RG_HIP(hipStreamWaitEvent(ctx->stream, ctx->ev_join, 0));
    return REGIONE_OK;
}
// While alive, launches through the context go to the side lane: its stream and the upper half of the K-split workspace
// (the main lane is left the lower half for the same time by LaneHalf).
struct LaneSwap {
    regione_ctx* c; hipStream_t stream; float* part; size_t bytes; bool on;
    LaneSwap(regione_ctx* ctx, bool side) : c(ctx), stream(ctx->stream), part(ctx->gemm_part), bytes(ctx->gemm_part_bytes), on(side) {
        if (!on) return;
        const size_t half = (bytes / 2) & ~static_cast<size_t>(255);
        c->stream = c->side_stream;
        c->gemm_part = reinterpret_cast<float*>(reinterpret_cast<char*>(part) + half);
        c->gemm_part_bytes = half;
    }
    ~LaneSwap() { if (on) { c->stream = stream; c->gemm_part = part; c->gemm_part_bytes = bytes; } }
};
struct LaneHalf {
    regione_ctx* c; size_t bytes; bool on;
    LaneHalf(regione_ctx* ctx, bool forked) : c(ctx), bytes(ctx->gemm_part_bytes), on(forked) { if (on) c->gemm_part_bytes = (bytes / 2) & ~static_cast<size_t>(255); }
    ~LaneHalf() { if (on) c->gemm_part_bytes = bytes; }
};

int check_stream_weights_fp8(const regione_stream_weights_fp8& w, int block_type, const char* which) {
    const bool dbl = block_type == REGIONE_BLOCK_DOUBLE;
    if (!w.w_1 || !w.w_2 || !w.s_1 || !w.s_2 || (dbl && (!w.w_qkv || !w.w_o || !w.s_qkv || !w.s_o)))
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward_fp8: null weight or scale in the %s stream", which);
    return REGIONE_OK;
}

// Codes of one projection's input rows ([max_fresh, H + M] bytes) and their row scales: allocated by the first
// 8-bit block call of a context, freed with it.
int ensure_fp8_workspace(regione_ctx* ctx) {
    if (ctx->q8) return REGIONE_OK;
    const size_t cols = static_cast<size_t>(ctx->dims.hidden) + ctx->dims.mlp;    // the joint row of a single-stream block
    const size_t rows = static_cast<size_t>(ctx->dims.max_fresh);
    if (rows == 0) return REGIONE_OK;
    RG_HIP(hipMalloc(reinterpret_cast<void**>(&ctx->q8), rows * cols));
    ctx->q8_bytes = rows * cols;
    if (hipMalloc(reinterpret_cast<void**>(&ctx->q8_scale), rows * sizeof(float)) != hipSuccess) {
        (void)hipFree(ctx->q8); ctx->q8 = nullptr;
        RG_FAIL(REGIONE_ERR_HIP, "block_forward_fp8: cannot allocate the scale workspace");
    }
    return REGIONE_OK;
}

int check_stream_weights(const regione_stream_weights& w, int block_type, const char* which) {
    if (block_type == REGIONE_BLOCK_DOUBLE) {
        if (!w.w_qkv || !w.w_o || !w.w_1 || !w.w_2) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: null weight in the %s stream", which);
    } else {
        if (!w.w_1 || !w.w_2) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: null weight in the %s stream", which);
    }
    return REGIONE_OK;
}

}  // namespace

// n_branches independent sequences (the conditional and unconditional branch of classifier-free guidance) through one
// set of weights: rows [b*n_fresh, (b+1)*n_fresh) of h and cache rows [b*n_all, (b+1)*n_all) belong to branch b; slots
// and positions are shared.  When no text row is fresh (or the block is single-stream) all branches' rows form ONE
// row group, so every projection is one GEMM over n_branches*n_fresh rows; attention runs per branch.
// w8 != null: the 8-bit form of the block's projections (regione_block_forward_fp8); `taps`
// then names the places that receive copies of the intermediates.
static int block_forward_impl(regione_ctx* ctx, const regione_block_weights* w, int32_t block_type,
                              const void* h_in, void* h_out, int32_t h_dtype, int32_t n_branches,
                              int32_t n_fresh, int32_t n_txt_fresh, const int32_t* slot_index, int32_t slot_offset,
                              void* k_cache, void* v_cache, int32_t n_all, int32_t flags,
                              const regione_block_weights_fp8* w8 = nullptr, const regione_fp8_taps* taps = nullptr) {
    if (!ctx || !w) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: null context or weights");
    if (n_branches < 1) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: %d branches", n_branches);
    if (block_type != REGIONE_BLOCK_DOUBLE && block_type != REGIONE_BLOCK_SINGLE) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: bad block type %d", block_type);
    if (h_dtype != REGIONE_BF16 && h_dtype != REGIONE_FP32) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: bad h_dtype %d", h_dtype);
    if (ctx->f32 && h_dtype != REGIONE_FP32) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: a float32 context carries a float32 residual stream");
    if (ctx->f32 && (w->rope || w->img.q_norm || w->img.k_norm || w->txt.q_norm || w->txt.k_norm))
        RG_FAIL(REGIONE_ERR_UNSUPPORTED, "block_forward: query/key normalisation and rotary embedding are bf16-context features");
    if (flags & ~(REGIONE_FLAG_STORE | REGIONE_FLAG_RETRIEVE)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: unknown flag bits %d", flags);
    if (flags == (REGIONE_FLAG_STORE | REGIONE_FLAG_RETRIEVE)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: store and retrieve together are not a mode of the algorithm");
    if (n_fresh < 0 || n_txt_fresh < 0 || n_txt_fresh > n_fresh) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: n_fresh=%d n_txt_fresh=%d", n_fresh, n_txt_fresh);
    if (static_cast<int64_t>(n_fresh) * n_branches > ctx->dims.max_fresh) RG_FAIL(REGIONE_ERR_WORKSPACE, "block_forward: %d rows in %d branch(es), context made for %d", n_fresh, n_branches, ctx->dims.max_fresh);
    if (flags) {
        if (n_all <= 0 || n_fresh > n_all) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "block_forward: n_fresh=%d n_all=%d", n_fresh, n_all);
        if (!k_cache || !v_cache) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: a flag is set but the cache is null");
        if (n_fresh > 0 && !slot_index) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: a flag is set but slot_index is null");
        if ((flags & REGIONE_FLAG_STORE) && n_fresh != n_all) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "block_forward: a storing forward carries every row (n_fresh=%d, n_all=%d)", n_fresh, n_all);
    }
    if (w->rope && w->rope_rows < (flags ? n_all : n_fresh)) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "block_forward: rotation table of %d rows for %d positions", w->rope_rows, flags ? n_all : n_fresh);
    const bool dbl = block_type == REGIONE_BLOCK_DOUBLE;
    const int n_txt = dbl ? n_txt_fresh : 0;
    int rc;
    if (w8) {
        if (n_fresh - n_txt > 0 && (rc = check_stream_weights_fp8(w8->img, block_type, "image")) != REGIONE_OK) return rc;
        if (n_txt > 0 && (rc = check_stream_weights_fp8(w8->txt, block_type, "text")) != REGIONE_OK) return rc;
    } else {
        if (n_fresh - n_txt > 0 && (rc = check_stream_weights(w->img, block_type, "image")) != REGIONE_OK) return rc;
        if (n_txt > 0 && (rc = check_stream_weights(w->txt, block_type, "text")) != REGIONE_OK) return rc;
    }
    if (n_fresh == 0) return REGIONE_OK;
    if (!h_in || !h_out) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward: null hidden state");

    const int H = ctx->dims.hidden, M = ctx->dims.mlp, heads = ctx->dims.heads, D = ctx->dims.head_dim;
    const int h_f32 = h_dtype == REGIONE_FP32;
    const size_t h_elem = h_f32 ? 4 : 2;
    const size_t es = ctx->f32 ? 4 : 2;     // bytes per element of activations and KV cache
    if (n_branches > 1 && n_txt > 0) {
        // text and image rows alternate between the branches: one pass per branch
        for (int b = 0; b < n_branches; ++b) {
            const size_t hoff = static_cast<size_t>(b) * n_fresh * H * h_elem, coff = static_cast<size_t>(b) * n_all * H * es;
            rc = block_forward_impl(ctx, w, block_type, static_cast<const char*>(h_in) + hoff, static_cast<char*>(h_out) + hoff, h_dtype, 1,
                                    n_fresh, n_txt_fresh, slot_index, slot_offset,
                                    k_cache ? static_cast<char*>(k_cache) + coff : nullptr, v_cache ? static_cast<char*>(v_cache) + coff : nullptr, n_all, flags);
            if (rc != REGIONE_OK) return rc;
        }
        return REGIONE_OK;
    }
    const int n_rows = n_fresh * n_branches;                       // rows of all branches, one group per stream
    const int period = n_branches > 1 ? n_fresh : 0;
    const int lda_attn = dbl ? H : H + M;   // single-stream: attention output and gelu(m) share rows of ctx->a
    char* kc = static_cast<char*>(k_cache);
    char* vc = static_cast<char*>(v_cache);
    // modulation vectors formed here from the step's conditioning vector (one one-vector linear layer per stream)
    regione_stream_weights sw[2] = {w->txt, w->img};
    if (w->cond) {
        if (ctx->f32) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "block_forward: forming the modulation vectors inside the call is a bf16-context feature");
        const int n_vec = dbl ? 6 : 3;
        for (int s = 0; s < 2; ++s) {
            if (!sw[s].w_mod || (s == 0 ? n_txt : n_rows - n_txt) <= 0) continue;
            float* mod = ctx->mod_ws + static_cast<size_t>(s) * 6 * H;
            if ((rc = regione_vec_linear(ctx, w->cond, REGIONE_ACT_SILU, sw[s].w_mod, sw[s].b_mod, n_vec * H, H, mod)) != REGIONE_OK) return rc;
            sw[s].shift1 = mod; sw[s].scale1 = mod + H; sw[s].gate1 = mod + 2 * H;
            if (dbl) { sw[s].shift2 = mod + 3 * H; sw[s].scale2 = mod + 4 * H; sw[s].gate2 = mod + 5 * H; }
        }
    }
    struct Rows { int r0, n; const regione_stream_weights* w; };
    const Rows groups[2] = {{0, n_txt, &sw[0]}, {n_txt, n_rows - n_txt, &sw[1]}};

    // several branches: the projection's epilogue takes one slot per row, branch b's shifted by b * n_all cache rows
    const int32_t* gemm_slots = slot_index;
    if (flags && n_branches > 1) {
        if ((rc = rg_expand_slots(ctx, slot_index, n_fresh, n_branches, n_all, ctx->slot_all)) != REGIONE_OK) return rc;
        gemm_slots = ctx->slot_all;
    }

    // Text and image rows of a double-stream block go through different weights: until the attention joins them, and
    // again after it, the two groups are independent, so the text group runs on the context's second lane and the
    // workgroups of both fill the chip together (each group alone leaves part of its last round of tiles empty).
    // (the 8-bit form keeps one lane: its groups share the workspace of the codes)
    const bool two_lanes = groups[0].n > 0 && groups[1].n > 0 && !ctx->prof_on && !w8;
    if (w8 && (rc = ensure_fp8_workspace(ctx)) != REGIONE_OK) return rc;
    // copy of an intermediate into the caller's tap (8-bit form only), rows of the group at their place
    auto tap = [&](void* dst, const void* src, size_t row0, size_t rows, size_t row_bytes) -> int {
        if (!dst) return REGIONE_OK;
        RG_HIP(hipMemcpyAsync(static_cast<char*>(dst) + row0 * row_bytes, src, rows * row_bytes, hipMemcpyDeviceToDevice, ctx->stream));
        return REGIONE_OK;
    };
    if (two_lanes && (rc = ensure_side_lane(ctx)) != REGIONE_OK) return rc;

    // ---- first half: LayerNorm + modulation, QKV (and MLP-in for single-stream) projection
    if (two_lanes && (rc = lane_fork(ctx)) != REGIONE_OK) return rc;
    for (const Rows& g : groups) {
        if (g.n <= 0) continue;
        LaneSwap swap(ctx, two_lanes && &g == &groups[0]);
        LaneHalf half(ctx, two_lanes && &g == &groups[1]);
        const char* hin = static_cast<const char*>(h_in) + static_cast<size_t>(g.r0) * H * h_elem;
        char* u = ctx->u + static_cast<size_t>(g.r0) * H * es;
        const regione_stream_weights_fp8* g8 = w8 ? (&g == &groups[0] ? &w8->txt : &w8->img) : nullptr;
        if (g8) rc = rg_layernorm_mod_fp8(ctx, hin, h_f32, g.n, H, g.w->shift1, g.w->scale1, ctx->q8, ctx->q8_scale);
        else rc = rg_layernorm_mod(ctx, hin, h_f32, g.n, H, g.w->shift1, g.w->scale1, u);
        if (rc != REGIONE_OK) return rc;
        if (g8 && taps && ((rc = tap(taps->u1_codes, ctx->q8, g.r0, g.n, H)) != REGIONE_OK || (rc = tap(taps->u1_scale, ctx->q8_scale, g.r0, g.n, 4)) != REGIONE_OK)) return rc;
        GemmEpilogue ep = {};
        ep.kind = EPI_QKV; ep.hidden = H;
        ep.q = reinterpret_cast<bf16_t*>(ctx->q + static_cast<size_t>(g.r0) * H * es); ep.ldq = H;
        if (flags) { ep.k = reinterpret_cast<bf16_t*>(kc); ep.v = reinterpret_cast<bf16_t*>(vc); ep.slot = gemm_slots + g.r0; ep.slot_offset = slot_offset; }
        else { ep.k = reinterpret_cast<bf16_t*>(ctx->kf + static_cast<size_t>(g.r0) * H * es); ep.v = reinterpret_cast<bf16_t*>(ctx->vf + static_cast<size_t>(g.r0) * H * es); ep.slot = nullptr; }
        ep.ldkv = H;
        if (g8 && dbl) {
            ep.bias = g.w->b_qkv; ep.row_scale = ctx->q8_scale; ep.col_scale = g8->s_qkv;
            rc = rg_gemm_fp8(ctx, ctx->q8, H, static_cast<const uint8_t*>(g8->w_qkv), g.n, 3 * H, H, ep);
        } else if (g8) {
            ep.bias = g.w->b_1; ep.act = REGIONE_ACT_GELU_TANH; ep.row_scale = ctx->q8_scale; ep.col_scale = g8->s_1;
            ep.y = ctx->a + static_cast<size_t>(g.r0) * lda_attn * es; ep.ldy = lda_attn; ep.y_col0 = H; ep.y_f32 = 0;
            rc = rg_gemm_fp8(ctx, ctx->q8, H, static_cast<const uint8_t*>(g8->w_1), g.n, 3 * H + M, H, ep);
        } else if (dbl) {
            ep.bias = g.w->b_qkv;
            rc = rg_gemm(ctx, u, H, g.w->w_qkv, g.n, 3 * H, H, ep);
        } else {
            ep.bias = g.w->b_1; ep.act = REGIONE_ACT_GELU_TANH;
            ep.y = ctx->a + static_cast<size_t>(g.r0) * lda_attn * es; ep.ldy = lda_attn; ep.y_col0 = H; ep.y_f32 = ctx->f32;
            rc = rg_gemm(ctx, u, H, g.w->w_1, g.n, 3 * H + M, H, ep);
        }
        if (rc != REGIONE_OK) return rc;
        // extras: normalised and rotated queries and keys, in place where the projection wrote them (bf16 contexts only)
        if (!ctx->f32) rc = rg_qk_norm_rope(ctx, ep.q, H, ep.k, H, flags ? slot_index + g.r0 : nullptr, slot_index ? slot_index + g.r0 : nullptr, g.r0, slot_offset, period, n_all, g.n, heads, D,
                             g.w->q_norm, g.w->k_norm, w->rope, w->rope_rows);
        if (rc != REGIONE_OK) return rc;
        if (g8 && taps && (rc = tap(taps->q, ep.q, g.r0, g.n, static_cast<size_t>(H) * 2)) != REGIONE_OK) return rc;
    }

    if (two_lanes && (rc = lane_join(ctx)) != REGIONE_OK) return rc;

    // ---- attention (Eq.6).  With a flag set the fresh K,V already sit in their cache slots, so the
    // key list is the whole cached sequence; without a flag it is the fresh rows only.
    for (int b = 0; b < n_branches; ++b) {
        const size_t r0 = static_cast<size_t>(b) * n_fresh * es, c0 = static_cast<size_t>(b) * n_all * H * es;
        if (flags) rc = rg_attention(ctx, ctx->q + r0 * H, H, n_fresh, nullptr, nullptr, H, 0, kc + c0, vc + c0, H, n_all, nullptr, heads, D, 0.f, ctx->a + r0 * lda_attn, lda_attn);
        else rc = rg_attention(ctx, ctx->q + r0 * H, H, n_fresh, ctx->kf + r0 * H, ctx->vf + r0 * H, H, n_fresh, nullptr, nullptr, H, 0, nullptr, heads, D, 0.f, ctx->a + r0 * lda_attn, lda_attn);
        if (rc != REGIONE_OK) return rc;
    }

    if (w8 && taps && (rc = tap(taps->attn, ctx->a, 0, n_fresh, static_cast<size_t>(lda_attn) * 2)) != REGIONE_OK) return rc;

    // ---- second half
    if (two_lanes && (rc = lane_fork(ctx)) != REGIONE_OK) return rc;
    for (const Rows& g : groups) {
        if (g.n <= 0) continue;
        LaneSwap swap(ctx, two_lanes && &g == &groups[0]);
        LaneHalf half(ctx, two_lanes && &g == &groups[1]);
        const char* hin = static_cast<const char*>(h_in) + static_cast<size_t>(g.r0) * H * h_elem;
        char* hout = static_cast<char*>(h_out) + static_cast<size_t>(g.r0) * H * h_elem;
        const char* a = ctx->a + static_cast<size_t>(g.r0) * lda_attn * es;
        GemmEpilogue ep = {};
        ep.kind = EPI_RESID;
        const regione_stream_weights_fp8* g8 = w8 ? (&g == &groups[0] ? &w8->txt : &w8->img) : nullptr;
        if (!dbl) {
            ep.bias = g.w->b_2; ep.gate = g.w->gate1;
            ep.resid = hin; ep.ldr = H; ep.resid_f32 = h_f32;
            ep.y = hout; ep.ldy = H; ep.y_f32 = h_f32;
            if (g8) {     // the joint row [attention | GELU(m)] becomes one row of codes
                ep.row_scale = ctx->q8_scale; ep.col_scale = g8->s_2;
                if ((rc = regione_quantize_rows_fp8(ctx, a, g.n, H + M, ctx->q8, ctx->q8_scale)) != REGIONE_OK) return rc;
                if (taps && ((rc = tap(taps->a_codes, ctx->q8, g.r0, g.n, static_cast<size_t>(H) + M)) != REGIONE_OK || (rc = tap(taps->a_scale, ctx->q8_scale, g.r0, g.n, 4)) != REGIONE_OK)) return rc;
                rc = rg_gemm_fp8(ctx, ctx->q8, H + M, static_cast<const uint8_t*>(g8->w_2), g.n, H, H + M, ep);
            } else {
                rc = rg_gemm(ctx, a, lda_attn, g.w->w_2, g.n, H, H + M, ep);
            }
            if (rc != REGIONE_OK) return rc;
            continue;
        }
        float* h1 = ctx->h1 + static_cast<size_t>(g.r0) * H;
        ep.bias = g.w->b_o; ep.gate = g.w->gate1;
        ep.resid = hin; ep.ldr = H; ep.resid_f32 = h_f32;
        ep.y = h1; ep.ldy = H; ep.y_f32 = 1;
        char* u = ctx->u + static_cast<size_t>(g.r0) * H * es;
        char* m = ctx->m + static_cast<size_t>(g.r0) * M * es;
        GemmEpilogue up = {};
        up.kind = EPI_PLAIN; up.bias = g.w->b_1; up.act = REGIONE_ACT_GELU_TANH; up.act_from = 0;
        up.y = m; up.ldy = M; up.y_f32 = ctx->f32;
        GemmEpilogue dn = {};
        dn.kind = EPI_RESID; dn.bias = g.w->b_2; dn.gate = g.w->gate2;
        dn.resid = h1; dn.ldr = H; dn.resid_f32 = 1;
        dn.y = hout; dn.ldy = H; dn.y_f32 = h_f32;
        if (g8) {
            // every projection's input rows become E4M3 codes with one scale per row in the shared workspace; the GEMM
            // that follows on the stream consumes them before the next stage overwrites them
            const uint8_t* q8 = ctx->q8;
            ep.row_scale = up.row_scale = dn.row_scale = ctx->q8_scale;
            ep.col_scale = g8->s_o; up.col_scale = g8->s_1; dn.col_scale = g8->s_2;
            if ((rc = regione_quantize_rows_fp8(ctx, a, g.n, H, ctx->q8, ctx->q8_scale)) != REGIONE_OK) return rc;
            if (taps && ((rc = tap(taps->a_codes, q8, g.r0, g.n, H)) != REGIONE_OK || (rc = tap(taps->a_scale, ctx->q8_scale, g.r0, g.n, 4)) != REGIONE_OK)) return rc;
            if ((rc = rg_gemm_fp8(ctx, q8, H, static_cast<const uint8_t*>(g8->w_o), g.n, H, H, ep)) != REGIONE_OK) return rc;
            if (taps && (rc = tap(taps->h1, h1, g.r0, g.n, static_cast<size_t>(H) * 4)) != REGIONE_OK) return rc;
            if ((rc = rg_layernorm_mod_fp8(ctx, h1, 1, g.n, H, g.w->shift2, g.w->scale2, ctx->q8, ctx->q8_scale)) != REGIONE_OK) return rc;
            if (taps && ((rc = tap(taps->u2_codes, q8, g.r0, g.n, H)) != REGIONE_OK || (rc = tap(taps->u2_scale, ctx->q8_scale, g.r0, g.n, 4)) != REGIONE_OK)) return rc;
            if ((rc = rg_gemm_fp8(ctx, q8, H, static_cast<const uint8_t*>(g8->w_1), g.n, M, H, up)) != REGIONE_OK) return rc;
            if (taps && (rc = tap(taps->m, m, g.r0, g.n, static_cast<size_t>(M) * 2)) != REGIONE_OK) return rc;
            if ((rc = regione_quantize_rows_fp8(ctx, m, g.n, M, ctx->q8, ctx->q8_scale)) != REGIONE_OK) return rc;
            if (taps && ((rc = tap(taps->m_codes, q8, g.r0, g.n, M)) != REGIONE_OK || (rc = tap(taps->m_scale, ctx->q8_scale, g.r0, g.n, 4)) != REGIONE_OK)) return rc;
            if ((rc = rg_gemm_fp8(ctx, q8, M, static_cast<const uint8_t*>(g8->w_2), g.n, H, M, dn)) != REGIONE_OK) return rc;
            continue;
        }
        if ((rc = rg_gemm(ctx, a, H, g.w->w_o, g.n, H, H, ep)) != REGIONE_OK) return rc;
        if ((rc = rg_layernorm_mod(ctx, h1, 1, g.n, H, g.w->shift2, g.w->scale2, u)) != REGIONE_OK) return rc;
        if ((rc = rg_gemm(ctx, u, H, g.w->w_1, g.n, M, H, up)) != REGIONE_OK) return rc;
        if ((rc = rg_gemm(ctx, m, M, g.w->w_2, g.n, H, M, dn)) != REGIONE_OK) return rc;
    }
    if (two_lanes && (rc = lane_join(ctx)) != REGIONE_OK) return rc;
    return REGIONE_OK;
}

extern "C" int regione_block_forward(regione_ctx* ctx, const regione_block_weights* w, int32_t block_type,
                                     const void* h_in, void* h_out, int32_t h_dtype,
                                     int32_t n_fresh, int32_t n_txt_fresh, const int32_t* slot_index, int32_t slot_offset,
                                     void* k_cache, void* v_cache, int32_t n_all, int32_t flags) {
    return block_forward_impl(ctx, w, block_type, h_in, h_out, h_dtype, 1, n_fresh, n_txt_fresh, slot_index, slot_offset, k_cache, v_cache, n_all, flags);
}

extern "C" int regione_block_forward_fp8(regione_ctx* ctx, const regione_block_weights* w, const regione_block_weights_fp8* w8, int32_t block_type,
                                         const void* h_in, void* h_out, int32_t h_dtype,
                                         int32_t n_fresh, int32_t n_txt_fresh, const int32_t* slot_index, int32_t slot_offset,
                                         void* k_cache, void* v_cache, int32_t n_all, int32_t flags, const regione_fp8_taps* taps_opt) {
    if (!ctx || !w8) RG_FAIL(REGIONE_ERR_INVALID_ARG, "block_forward_fp8: null context or weights");
    if (ctx->f32) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "block_forward_fp8: the 8-bit projections belong to bf16 contexts");
    if (ctx->dims.hidden > 4096 || (ctx->dims.hidden % 128) || (ctx->dims.mlp % 128))
        RG_FAIL(REGIONE_ERR_UNSUPPORTED, "block_forward_fp8: hidden=%d (at most 4096) and mlp=%d must be multiples of 128", ctx->dims.hidden, ctx->dims.mlp);
    if (block_type == REGIONE_BLOCK_SINGLE && ctx->dims.hidden + ctx->dims.mlp > 16384)
        RG_FAIL(REGIONE_ERR_UNSUPPORTED, "block_forward_fp8: a single-stream block's joint row of %d columns exceeds the row quantiser's 16384", ctx->dims.hidden + ctx->dims.mlp);
    return block_forward_impl(ctx, w, block_type, h_in, h_out, h_dtype, 1, n_fresh, n_txt_fresh, slot_index, slot_offset, k_cache, v_cache, n_all, flags,
                              w8, taps_opt);
}

extern "C" int regione_block_forward_batched(regione_ctx* ctx, const regione_block_weights* w, int32_t block_type,
                                             const void* h_in, void* h_out, int32_t h_dtype, int32_t n_branches,
                                             int32_t n_fresh, int32_t n_txt_fresh, const int32_t* slot_index, int32_t slot_offset,
                                             void* k_cache, void* v_cache, int32_t n_all, int32_t flags) {
    return block_forward_impl(ctx, w, block_type, h_in, h_out, h_dtype, n_branches, n_fresh, n_txt_fresh, slot_index, slot_offset, k_cache, v_cache, n_all, flags);
}
