// Shared declarations of the library's translation units (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdarg.h>
#include <stdio.h>
#include "regione.h"
#include "regione_bench.h"

typedef uint16_t bf16_t;  // raw bfloat16 bits in memory

struct regione_ctx {
    hipStream_t stream;
    regione_dims dims;
    int device;
    int f32;       // compute dtype of the context is float32: the activation buffers below then hold 4-byte elements
    // workspace (device)
    int32_t* part_counts;  // scratch of the partition: per-block edited counts, then one decision bit per token
    int64_t part_counts_cap;   // its size in int32 entries
    int32_t* n_edited_pinned;      // pinned host copy of the last edited-token count (host address)
    int32_t* n_edited_pinned_dev;  // the same memory as the device sees it
    int32_t count_ticket;          // last ticket handed to a partition whose count the host polls for (word 1 of the pinned memory)
    // activation buffers: elements of the compute dtype (bf16, or float32 in a float32 context); addressed in bytes
    char* u;       // [max_fresh, H]     normalised + modulated rows
    char* q;       // [max_fresh, H]
    char* kf;      // [max_fresh, H]     fresh keys when the cache is not used
    char* vf;      // [max_fresh, H]
    char* a;       // [max_fresh, H+M]   attention output (+ activated MLP part, single-stream)
    float* h1;     // [max_fresh, H]     residual stream between the two halves of a block
    char* m;       // [max_fresh, M]     activated MLP hidden rows
    float* attn_part;  // split-KV partial results
    size_t attn_part_bytes;
    int32_t* slot_all; // [max_fresh] slot list of all branches of a batched block call
    float* mod_ws;     // [2][6H] modulation vectors of the two streams when a block call forms them itself
    // workspace of the 8-bit block (allocated by its first call): codes of one projection's input rows and their scales
    uint8_t* q8; size_t q8_bytes; float* q8_scale;
    float* gemm_part;  // split-K partial sums
    size_t gemm_part_bytes;
    // second lane for independent work inside one call (text and image rows of a double-stream block use different
    // weights, so their projections do not depend on each other): a stream of the default priority and two events,
    // created on first use; while a lane swap is active, `stream` and `gemm_part` name the lane's own stream and half
    hipStream_t side_stream;
    hipEvent_t ev_fork, ev_join;
    int gemm_force_tn, gemm_force_splits;  // 0 = chosen per call
    int attn_force_splits;  // 0 = chosen per call
    // kernels that need more than 64 KiB of LDS have to be granted it once per device: one bit per kernel family and
    // instantiation that this context (one device) has already asked for
    uint32_t lds_grant_mask;
    // optional per-kernel-class timing with HIP events on the context's stream
    int prof_on;
    int prof_used;
    int prof_cap;
    hipEvent_t* prof_ev;   // 2 * prof_cap events: start/stop pairs
    int* prof_class;       // class of each pair
};

// Brackets the launches of one kernel class with an event pair when profiling is on.
struct ProfScope {
    regione_ctx* c; int slot;
    ProfScope(regione_ctx* ctx, int kernel_class) : c(ctx), slot(-1) {
        if (c && c->prof_on && c->prof_used < c->prof_cap) {
            slot = c->prof_used++;
            c->prof_class[slot] = kernel_class;
            (void)hipEventRecord(c->prof_ev[2 * slot], c->stream);
        }
    }
    ~ProfScope() { if (slot >= 0) (void)hipEventRecord(c->prof_ev[2 * slot + 1], c->stream); }
};

void regione_set_error(const char* fmt, ...);
#define RG_FAIL(code, ...) do { regione_set_error(__VA_ARGS__); return (code); } while (0)
#define RG_HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
    regione_set_error("%s failed: %s", #call, hipGetErrorString(e_)); return REGIONE_ERR_HIP; } } while (0)
#define RG_LAUNCH_CHECK() RG_HIP(hipGetLastError())

static inline bool rg_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- device helpers
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    __bf16 h = static_cast<__bf16>(f);  // round to nearest even (v_cvt_pk_bf16_f32 on gfx950)
    return __builtin_bit_cast(bf16_t, h);
}

// ---- internal launchers (each enqueues on ctx->stream and returns an error code)
enum { EPI_PLAIN = 0, EPI_QKV = 1, EPI_RESID = 2, EPI_VELOCITY = 3 };   // EPI_VELOCITY exists only as the merge step of a K-split GEMM

struct GemmEpilogue {
    int kind;            // EPI_*
    int vec_ok;          // set by rg_gemm: the wide (8 columns per lane) epilogue may be used
    const float* bias;   // [N] or null
    int act;             // REGIONE_ACT_* (applied to columns >= act_from)
    int act_from;
    // EPI_PLAIN: y[row*ldy + col] (bf16 or f32)
    void* y; int ldy; int y_f32;
    // EPI_QKV: columns [0,H) -> q[row*ldq+col]; [H,2H) -> k[slot(row)*ldkv + col-H]; [2H,3H) -> v[...];
    //          columns >= 3H -> y[row*ldy + y_col0 + col-3H] (single-stream MLP part)
    bf16_t* q; int ldq; bf16_t* k; bf16_t* v; int ldkv; const int32_t* slot; int slot_offset; int hidden; int y_col0;
    // EPI_RESID: y[row*ldy+col] = resid[row*ldr+col] + gate[col]*(acc+bias)
    const void* resid; int ldr; int resid_f32; const float* gate;
    // 8-bit GEMM only: the float32 sums are multiplied by row_scale[row] * col_scale[col] before anything else
    const float* row_scale; const float* col_scale;
    // merge_kind == EPI_VELOCITY (a plain K-split GEMM whose merge kernel finishes the step, Eq.9 fresh branch + Eq.4 + merge):
    //   v = storage-rounded(acc + bias); y (if non-null) = v; vel_ca = v; vel_xe -= vel_dt * v; vel_xfull[vel_index[row]] = vel_xe
    int merge_kind;
    void* vel_ca; void* vel_xe; void* vel_xfull; const int32_t* vel_index; float vel_dt;
};

// a, w_packed (and the epilogue's q, k, v, y, resid where they are activations) are bf16, or float32 in a float32 context
int rg_gemm(regione_ctx* ctx, const void* a, int lda, const void* w_packed, int m, int n, int k, const GemmEpilogue& ep);
// y = x W^T + b as a K-split GEMM whose merge kernel applies the velocity step described at GemmEpilogue::merge_kind (bf16 contexts)
int rg_gemm_velocity(regione_ctx* ctx, const void* a, int lda, const void* w_packed, int m, int n, int k, const GemmEpilogue& ep);
int rg_gemm_f32(regione_ctx* ctx, const float* a, int lda, const float* w, int m, int n, int k, const GemmEpilogue& ep);
// E4M3 operands (k counts 8-bit elements, a multiple of 128; lda in bytes, a multiple of 16); ep.row_scale / col_scale set
// LayerNorm + modulation with the E4M3 row quantisation of its float32 result: codes [n, hidden], one scale per row
int rg_layernorm_mod_fp8(regione_ctx* ctx, const void* h, int h_f32, int n, int hidden, const float* shift, const float* scale,
                         uint8_t* q, float* row_scale);
int rg_gemm_fp8(regione_ctx* ctx, const uint8_t* a, int lda, const uint8_t* w_packed, int m, int n, int k, const GemmEpilogue& ep);
int rg_layernorm_mod(regione_ctx* ctx, const void* h, int h_f32, int n, int hidden, const float* shift, const float* scale, void* u);   // u: compute dtype
int rg_qk_norm_rope(regione_ctx* ctx, bf16_t* q, int ldq, bf16_t* k, int ldkv, const int32_t* kv_slot,
                    const int32_t* pos_slot, int pos0, int slot_offset, int slot_period, int slot_branch_rows, int n, int heads, int d,
                    const float* q_norm, const float* k_norm, const float* table, int table_rows);
int rg_expand_slots(regione_ctx* ctx, const int32_t* slot, int n, int n_branches, int branch_rows, int32_t* out);
int rg_attention(regione_ctx* ctx, const void* q, int ldq, int n_q,
                 const void* k0, const void* v0, int ldkv0, int n0,
                 const void* k1, const void* v1, int ldkv1, int n1, const int32_t* idx1,
                 int heads, int d, float scale, void* out, int ldo);
int rg_attention_f32(regione_ctx* ctx, const float* q, int ldq, int n_q,
                     const float* k0, const float* v0, int ldkv0, int n0,
                     const float* k1, const float* v1, int ldkv1, int n1, const int32_t* idx1,
                     int heads, int d, float scale, float* out, int ldo);
int rg_pack_weight_f32(regione_ctx* ctx, const float* w, int n, int k, float* w_packed);
// regione_partition whose host count arrives through a ticketed pinned word instead of a stream synchronisation
int rg_partition_early_count(regione_ctx* ctx, const void* x_t, const void* v, const void* x_ref,
                             int64_t n_tokens, int32_t c, int32_t dtype, float sigma_t, float eta,
                             float* score_opt, uint8_t* mask, int32_t* e_index, int32_t* u_index,
                             int32_t* n_edited_dev, int32_t* n_edited_host);
// the static-scratch lookup of regione_partition_static, done ahead of time by regione_create
int rg_partition_static_warm(void);
// int32 entries of scratch memory the partition needs for max_tokens tokens
int64_t rg_partition_scratch_ints(int64_t max_tokens);
