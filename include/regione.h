/*
 * regione.h - C ABI of the RegionE region-aware denoising step for AMD MI355X (gfx950).
 *
 * The library implements the data-parallel part of one region-aware step of RegionE
 * (arXiv 2510.25590, section "Methodology" and Algorithm 1): adaptive region partition,
 * gather of the edited tokens, transformer blocks on those tokens with attention over the
 * Region-Instruction KV cache (Eq.6), the adaptive velocity decay cache (Eq.7-9) with the
 * Euler update (Eq.4), and the scatter back by spatial position.
 *
 * Conventions
 *  - Every function returns REGIONE_OK (0) or a negative error code; regione_last_error()
 *    returns a message for the last failure on the calling thread.  Nothing throws.
 *  - Pointers are DEVICE pointers unless the name ends in _host.  The caller owns every
 *    tensor (inputs, outputs, KV cache, velocity cache); the library owns only the context
 *    and the workspace inside it.  Tensors are row-major with the innermost dimension
 *    contiguous; base addresses must be 16-byte aligned.
 *  - Work is enqueued on the HIP stream given to regione_create and is asynchronous; the
 *    only call that waits for the stream is regione_partition with a non-null
 *    n_edited_host.  Calls on one context must not overlap (they share its workspace).
 *  - Token order of the cached sequence is [P (text) | X (image) | I (reference image)].
 *  - Linear weights reach the library in its PACKED bf16 layout, made once per weight by
 *    regione_pack_weight from the usual row-major [out_features, in_features] matrix;
 *    biases and modulation vectors are float32.
 *  - Empty inputs (no edited token, no cache rows) are not errors: the call does nothing
 *    or degenerates as Eq.6 does.
 */
#ifndef REGIONE_H
#define REGIONE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    REGIONE_OK = 0,
    REGIONE_ERR_INVALID_ARG = -1, /* null pointer, negative size, bad enum, both flags */
    REGIONE_ERR_BAD_SHAPE = -2,   /* sizes inconsistent with each other or with the context */
    REGIONE_ERR_UNSUPPORTED = -3, /* e.g. head dimension other than 64 or 128 */
    REGIONE_ERR_WORKSPACE = -4,   /* call needs more rows than the context was created for */
    REGIONE_ERR_HIP = -5          /* a HIP runtime call failed */
};

enum { REGIONE_BF16 = 0, REGIONE_FP32 = 1 };
enum { REGIONE_BLOCK_DOUBLE = 0, REGIONE_BLOCK_SINGLE = 1 };
/* The flag pair f = (store, retrieve) of Algorithm 1. */
enum { REGIONE_FLAG_STORE = 1, REGIONE_FLAG_RETRIEVE = 2 };
enum { REGIONE_ACT_NONE = 0, REGIONE_ACT_GELU_TANH = 1, REGIONE_ACT_SILU = 2 };

typedef struct regione_ctx regione_ctx;

/* Sizes the workspace is allocated for, and the arithmetic type of the context.
 * compute_dtype = REGIONE_BF16 (0, the default): activations, weights and the KV cache are bf16, products run on
 * the bf16 matrix-core instruction with float32 sums.
 * compute_dtype = REGIONE_FP32: every tensor that this header calls bf16 for regione_pack_weight, regione_linear,
 * regione_layernorm (its output), regione_attn_kvcache, regione_block_forward(_batched) (activations, KV cache, and
 * h_dtype must be REGIONE_FP32) is float32 instead, products run on the float32 matrix-core instruction
 * (v_mfma_f32_32x32x2_f32) and the softmax in float32: the small float32 configuration the method is first checked
 * on.  One simple tile shape, built for correctness, not speed.  The block extras (q_norm / k_norm / rope) and the
 * 8-bit projections are bf16-context features: REGIONE_ERR_UNSUPPORTED in a float32 context. */
typedef struct regione_dims {
    int32_t hidden;     /* H = heads * head_dim */
    int32_t heads;
    int32_t head_dim;   /* 64 or 128 */
    int32_t mlp;        /* MLP width M */
    int32_t max_fresh;  /* most rows one regione_block_forward call will carry */
    int32_t max_tokens; /* most tokens one regione_partition call will carry */
    int32_t compute_dtype; /* REGIONE_BF16 or REGIONE_FP32 */
} regione_dims;

/* Weights of one stream of a block (host struct of device pointers to PACKED weights).
 * Double-stream block: w_qkv [3H,H], w_o [H,H], w_1 [M,H], w_2 [H,M].
 * Single-stream block: w_1 [3H+M,H] producing [q|k|v|m], w_2 [H,H+M] applied to
 * [attention | gelu(m)]; w_qkv, w_o and the *2 modulation vectors are ignored.
 * Modulation vectors [H] may be NULL (shift = scale = 0, gate = 1).
 * q_norm / k_norm [head_dim] float32, 16-byte aligned, or NULL: when given, every head of the
 * stream's queries / keys is divided by sqrt(mean(x^2) + 1e-6) and multiplied by the vector
 * (an extra of real editing transformers; the paper keeps the DiT a black box).
 * w_mod / b_mod: NULL, or the stream's modulation layer (bf16 ROW-MAJOR [6H, H] and float32 [6H]; single-stream blocks
 * [3H, H] and [3H]); used when the block's `cond` is given, see regione_block_weights. */
typedef struct regione_stream_weights {
    const void* w_qkv; const float* b_qkv;
    const void* w_o;   const float* b_o;
    const void* w_1;   const float* b_1;
    const void* w_2;   const float* b_2;
    const float* shift1; const float* scale1; const float* gate1;
    const float* shift2; const float* scale2; const float* gate2;
    const float* q_norm; const float* k_norm;
    const void* w_mod; const float* b_mod;
} regione_stream_weights;

/* rope: NULL, or the table written by regione_rope_table for ALL rope_rows positions of the
 * cached sequence [P | X | I].  Queries and keys of fresh row i are then rotated (after the
 * normalisation) by the angles of position slot_index[i] + slot_offset (of position i when
 * slot_index is NULL): a gathered token keeps the position it has in the full sequence, and
 * keys enter the cache rotated.  Positions outside [0, rope_rows) use the nearest table row.
 * cond: NULL, or the step's conditioning vector [H] float32 on the device.  Every stream that carries rows in the call
 * and has a w_mod then gets its modulation vectors from it inside the block call, before anything else runs:
 *   [shift1 | scale1 | gate1 | shift2 | scale2 | gate2] = w_mod silu(cond) + b_mod   (regione_vec_linear, SiLU on the
 * input; single-stream blocks: the first three), into the context's workspace; the stream's six pointers are then
 * ignored.  bf16 contexts only.  (The paper keeps this layer inside its black-box DiT.) */
typedef struct regione_block_weights {
    regione_stream_weights txt; /* text rows of a double-stream block */
    regione_stream_weights img; /* image / reference rows; the only set of a single-stream block */
    const float* rope;
    int32_t rope_rows;
    const float* cond;
} regione_block_weights;

/* State of the adaptive velocity decay cache between steps (host). */
typedef struct regione_avd_state {
    int32_t valid; /* 0: the cache holds no velocity yet */
    double prod;   /* product of Eq.7 factors since the cached velocity was computed */
} regione_avd_state;

const char* regione_last_error(void);

/* Creates a context bound to `hip_stream` (a hipStream_t, NULL = default stream) on the
 * current device and allocates its workspace for `dims`.  The context is released with
 * regione_destroy, which first waits for the stream. */
int regione_create(regione_ctx** out, const regione_dims* dims, void* hip_stream);
int regione_destroy(regione_ctx* ctx);

/* Adaptive region partition (section "Adaptive Region Partition", Algorithm 1 lines of the
 * ARP comment) without the morphological clean-up: one-step estimate x0 = x_t - sigma_t*v
 * (Eq.5 with t_f = 0), cosine similarity of each token of x0 with the same token of x_ref
 * over the c channels, unedited iff score > eta, and the ascending index lists.
 *   x_t, v, x_ref : [n_tokens, c] of `dtype`.
 *   score_opt     : [n_tokens] float32 or NULL.
 *   mask          : [n_tokens] uint8, 1 = edited.
 *   e_index, u_index : [n_tokens] int32 each; the first *n_edited entries of e_index and
 *                   the first n_tokens - *n_edited entries of u_index are written.
 *   n_edited_dev  : device int32.  n_edited_host_opt: host int32 or NULL; when given the
 *                   call waits for the stream and stores the count there.
 * Arithmetic: x0 in float32 (product and difference rounded separately), the three sums in
 * float64, score = dot / max(sqrt(|x0|^2) sqrt(|ref|^2), 1e-8) rounded to float32 and
 * compared with (float)eta.  A zero vector scores 0; NaN counts as edited. */
int regione_partition(regione_ctx* ctx, const void* x_t, const void* v, const void* x_ref,
                      int64_t n_tokens, int32_t c, int32_t dtype, float sigma_t, float eta,
                      float* score_opt, uint8_t* mask, int32_t* e_index, int32_t* u_index,
                      int32_t* n_edited_dev, int32_t* n_edited_host_opt);

/* regione_partition for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Needs no context and calls no allocating routine: the per-block counts
 * and decision bits that regione_partition keeps in its context's workspace live in a static device array of the library
 * (768 KiB per GPU, held until the process ends; its address is looked up on the first call on each device, or by regione_create).
 * Same kernels, same results bit for bit.  hip_stream: a hipStream_t (NULL = default stream) on the CURRENT device;
 * the call is asynchronous and returns no host count (read n_edited_dev after the stream has caught up).
 * n_tokens > 4194304 (2^22): REGIONE_ERR_WORKSPACE.  All calls on one GPU share the one array: calls that overlap
 * in time on the same GPU (different streams or threads) race; calls on one stream are safe.  Nothing in the array
 * needs clearing between calls. */
int regione_partition_static(void* hip_stream, const void* x_t, const void* v, const void* x_ref,
                             int64_t n_tokens, int32_t c, int32_t dtype, float sigma_t, float eta,
                             float* score_opt, uint8_t* mask, int32_t* e_index, int32_t* u_index,
                             int32_t* n_edited_dev);

/* Morphological clean-up of the partition on the token grid (section "Adaptive Region
 * Partition": opening and closing make the two regions more continuous; Algorithm 1 applies
 * erosion and dilation to the map cos > eta, i.e. to the unedited region).  Opening (erosion
 * then dilation) then closing (dilation then erosion) of the UNEDITED map with the 3x3 square;
 * cells outside the grid never decide (the paper names neither element nor border: both are
 * this library's reading).  mask_in [n_images * grid_h * grid_w] uint8, 1 = edited, as written
 * by regione_partition; mask_out the cleaned mask (may alias mask_in); e_index / u_index /
 * n_edited_dev / n_edited_host_opt as in regione_partition, rebuilt from the cleaned mask.
 * grid_h * grid_w <= 16384, else REGIONE_ERR_UNSUPPORTED. */
int regione_mask_cleanup(regione_ctx* ctx, const uint8_t* mask_in, int32_t grid_h, int32_t grid_w, int32_t n_images,
                         uint8_t* mask_out, int32_t* e_index, int32_t* u_index,
                         int32_t* n_edited_dev, int32_t* n_edited_host_opt);

/* Row gather X[index] (Algorithm 1, "X^E = X[E_index]"): dst[i,:] = src[index[i],:] for
 * i < n, with n = *n_dev when n_dev is non-null (clamped to n_max) and n_max otherwise.
 * Rows have row_elems elements of `dtype`; the copy is bit-exact. src and dst must not overlap. */
int regione_gather(regione_ctx* ctx, const void* src, int32_t row_elems, int32_t dtype,
                   const int32_t* index, const int32_t* n_dev, int64_t n_max, void* dst);

/* Merge by spatial position (Algorithm 1, the line after the inner loop):
 * dst_full[index[i],:] = src[i,:] for i < n; every other row of dst_full is left untouched.
 * Indices must be distinct. */
int regione_scatter(regione_ctx* ctx, void* dst_full, int32_t row_elems, int32_t dtype,
                    const int32_t* index, const int32_t* n_dev, int64_t n_max, const void* src);

/* Attention with the Region-Instruction KV cache, Eq.6:
 *   out = softmax(q [k_fresh; k_cache']^T * scale) [v_fresh; v_cache']
 * per head, where cache' is all n_c cache rows when cache_index_opt is NULL and the
 * n_cache_index rows it lists otherwise.  bf16 tensors, float32 softmax and accumulation.
 *   q, out           : [n_q, heads, d]
 *   k_fresh, v_fresh : [n_fresh, heads, d]; may be NULL when n_fresh == 0
 *   k_cache, v_cache : [n_c, heads, d]; may be NULL when n_c == 0
 * n_c == 0 is local attention (the "w/o RIKVCache" ablation).  At least one key is needed
 * when n_q > 0.  d is 64 or 128.  scale <= 0 selects 1/sqrt(d). */
int regione_attn_kvcache(regione_ctx* ctx, const void* q, int32_t n_q,
                         const void* k_fresh, const void* v_fresh, int32_t n_fresh,
                         const void* k_cache, const void* v_cache, int32_t n_c,
                         const int32_t* cache_index_opt, int32_t n_cache_index,
                         int32_t heads, int32_t d, float scale, void* out);

/* Weight packing.  The GEMM kernels read weights in the register layout of the matrix-core
 * operand: for W [n, k] (k a multiple of 64) the packed array holds, for every block of 32
 * output features and 16 input features, 64 x 8 bf16 with entry (lane, e) =
 * W[32*block_n + lane%32][16*block_k + 8*(lane/32) + e]; blocks are ordered block_n major.
 * Rows past n are zero.  regione_packed_weight_elems gives the element count of the packed
 * array (n rounded up to 32, times k).  Packing is a one-time copy on the context's stream. */
int64_t regione_packed_weight_elems(int32_t n, int32_t k);
int regione_pack_weight(regione_ctx* ctx, const void* w /*[n,k] bf16 row-major*/, int32_t n, int32_t k, void* w_packed);

/* y = act(x W^T + b): x [m,k] bf16, W packed from [n,k], b [n] float32 or NULL, y [m,n] of
 * out_dtype.  k must be a multiple of 64.  Used for the token embedding and the velocity
 * head around the blocks, and by the block itself. */
int regione_linear(regione_ctx* ctx, const void* x, const void* w_packed, const float* b_opt,
                   int32_t m, int32_t n, int32_t k, int32_t act, int32_t out_dtype, void* y);

/* 8-bit floating point variant of the dense projections (section "Region-Aware Generation":
 * the DiT's linear layers on the edited rows).  The paper computes in the model's own
 * precision; this variant is an extension with its own accuracy, never chosen silently.
 * Format: E4M3 of the OCP 8-bit floating point specification (bias 7, largest value 448,
 * no infinities), one float32 scale per row.
 *
 * regione_quantize_rows_fp8: for every row r of x [rows, cols] (bf16, finite values)
 *   amax = max |x[r,:]|, scale[r] = amax / 448, q[r,c] = e4m3(x[r,c] * (448 / amax)),
 * both quotients and the product in float32, the product clamped to +-448 and rounded to
 * nearest, ties to even.  A row of zeros gets scale 1.  q: uint8 [rows, cols]; scale:
 * float32 [rows].  cols must be a multiple of 8 and at most 16384; x and q 16-byte aligned.
 * Serves activations (a row = a token) and weights (a row = an output feature) alike.
 *
 * regione_pack_weight_fp8: the quantised weight codes [n, k] (k a multiple of 128) in the
 * operand layout of the 8-bit matrix-core instruction: for every block of 32 output
 * features and 32 input features, 64 x 16 bytes with entry (lane, e) =
 * Wq[32*block_n + lane%32][32*block_k + 16*(lane/32) + e]; rows past n are zero.  The packed
 * array has regione_packed_weight_elems(n, k) BYTES.
 *
 * regione_linear_fp8: y[m,n] = act(x_scale[m] * w_scale[n] * sum_k xq[m,k] wq[n,k] + b[n]),
 * products exact, sums in float32.  xq uint8 [m,k] row-major, k a multiple of 128; y of
 * out_dtype (bf16 or float32).  The scales are applied to the float32 sums before the bias.
 * Accuracy of the sums: the matrix-core instruction adds its 64 products in groups of 8 that
 * are aligned to the group's largest product and cut 14 bits below it, so the result is within
 * 2^-11 * sum_k |xq wq| (times the scales) of the exact sum; without a dominant product the
 * error is orders of magnitude smaller, and always far below the format's own 2^-4. */
int regione_quantize_rows_fp8(regione_ctx* ctx, const void* x, int64_t rows, int32_t cols, void* q, float* scale);
int regione_pack_weight_fp8(regione_ctx* ctx, const void* wq /*[n,k] uint8 row-major*/, int32_t n, int32_t k, void* wq_packed);
int regione_linear_fp8(regione_ctx* ctx, const void* xq, const float* x_scale, const void* wq_packed, const float* w_scale,
                       const float* b_opt, int32_t m, int32_t n, int32_t k, int32_t act, int32_t out_dtype, void* y);

/* One transformer block on the fresh rows: one layer of Phi(tokens, C_KV, f) in
 * Algorithm 1.  The block is LayerNorm (no affine, eps 1e-6) -> modulation -> QKV linear ->
 * attention -> gated residual -> LayerNorm -> modulation -> MLP with tanh-GELU -> gated
 * residual (double-stream), or the fused single-stream form described at
 * regione_stream_weights.
 *   h_in, h_out : [n_fresh, H] of h_dtype (the residual stream; may be the same buffer).
 *   n_txt_fresh : rows [0, n_txt_fresh) use w->txt, the rest w->img (double-stream only).
 *   slot_index, slot_offset : fresh row i sits at position slot_index[i] + slot_offset of the
 *                 cached sequence (e.g. E_index and the number of text tokens); slot_index is
 *                 [n_fresh] int32 and is needed when a flag is set.
 *   k_cache, v_cache : [n_all, heads, head_dim] bf16, the layer's C_KV.
 *   flags = REGIONE_FLAG_STORE    : full forward; n_fresh must equal n_all; the fresh K,V
 *                                   are written to their cache rows.
 *   flags = REGIONE_FLAG_RETRIEVE : Eq.6; keys/values are the fresh rows plus every cache
 *                                   row that is not refreshed.  The fresh K,V overwrite
 *                                   their own slots in the cache (those slots are never
 *                                   read stale by Eq.6); all other cache rows are untouched.
 *   flags = 0                     : plain attention over the fresh rows, cache unused.
 *   both flags                    : REGIONE_ERR_INVALID_ARG. */
int regione_block_forward(regione_ctx* ctx, const regione_block_weights* w, int32_t block_type,
                          const void* h_in, void* h_out, int32_t h_dtype,
                          int32_t n_fresh, int32_t n_txt_fresh, const int32_t* slot_index, int32_t slot_offset,
                          void* k_cache, void* v_cache, int32_t n_all, int32_t flags);

/* Rotary position embedding table (an extra of real editing transformers, not described by
 * the paper): pos_ids [n, n_axes] int32 on the device, axes_dims [n_axes] on the HOST, the even
 * number of head-dimension elements each axis owns (their sum is the context's head_dim, at most
 * 8 axes).  Pair j of an axis that owns a elements turns by pos * theta^(-2j/a); the pairs of
 * the axes follow each other, and pair j of a head is elements (2j, 2j+1).
 * table [n, head_dim] float32: cos of the head_dim/2 angles, then their sin (angles in float64,
 * rounded once). */
int regione_rope_table(regione_ctx* ctx, const int32_t* pos_ids, int64_t n, int32_t n_axes,
                       const int32_t* axes_dims_host, float theta, float* table);

/* The same block for n_branches independent sequences that share weights, slot list and flags:
 * the conditional and unconditional branch of classifier-free guidance, which the paper's
 * experiments run at every step ("Experimental Settings").  h_in / h_out are
 * [n_branches, n_fresh, H], k_cache / v_cache [n_branches, n_all, heads, head_dim]; the result is
 * that of n_branches regione_block_forward calls on the slices.  When no text row is fresh (or
 * the block is single-stream) every projection runs once over all n_branches * n_fresh rows, so
 * the weights are read once and the GEMMs get twice the rows; attention runs per branch.
 * n_branches * n_fresh must fit the context's max_fresh. */
int regione_block_forward_batched(regione_ctx* ctx, const regione_block_weights* w, int32_t block_type,
                                  const void* h_in, void* h_out, int32_t h_dtype, int32_t n_branches,
                                  int32_t n_fresh, int32_t n_txt_fresh, const int32_t* slot_index, int32_t slot_offset,
                                  void* k_cache, void* v_cache, int32_t n_all, int32_t flags);

/* y = W act(x) + b for ONE vector: the shape of a block's modulation (its shift, scale and gate
 * vectors), which real editing transformers compute once per step from a conditioning embedding
 * (the paper keeps this inside its black-box DiT; the block itself takes the vectors as given).
 *   x [k] float32; pre_act REGIONE_ACT_NONE or REGIONE_ACT_SILU, applied to x;
 *   w [n, k] bf16 ROW-MAJOR (not packed), 16-byte aligned; b_opt [n] float32 or NULL; y [n] float32.
 * k: a multiple of 8, at most 16384.  Products in float32.  Bound by reading w once from HBM. */
int regione_vec_linear(regione_ctx* ctx, const float* x, int32_t pre_act, const void* w, const float* b_opt,
                       int32_t n, int32_t k, float* y);

/* Sinusoidal embedding of a scalar (host value t): out[j] = cos(t f_j), out[dim/2 + j] = sin(t f_j),
 * f_j = max_period^(-j / (dim/2)), j < dim/2; formed in float64, stored float32 on the device. */
int regione_timestep_embedding(regione_ctx* ctx, double t, int32_t dim, double max_period, float* out);

/* dst[i] = src[i] converted between the storage types (to bf16: round to nearest even).  Lets a
 * caller keep the latents of the sampling loop in float32 and feed bf16 rows to the token
 * embedding.  Same dtype on both sides is a plain copy. */
int regione_cast(regione_ctx* ctx, const void* src, int32_t src_dtype, void* dst, int32_t dst_dtype, int64_t n_elems);

/* LayerNorm over the hidden width (no affine parameters, biased variance, eps 1e-6) followed
 * by the optional modulation u = y * (1 + scale) + shift: the normalisation in front of the
 * velocity head around the blocks (the blocks apply the same operation internally).
 * h [n, hidden] of h_dtype; shift_opt / scale_opt [hidden] float32 or NULL (identity);
 * u [n, hidden] bf16. */
int regione_layernorm(regione_ctx* ctx, const void* h, int32_t h_dtype, int32_t n, int32_t hidden,
                      const float* shift_opt, const float* scale_opt, void* u);

/* Control flow of Algorithm 1 (host, pure function of its hyper-parameters).  Timestep
 * indices run i = T..1; the step at index i moves X_{t_i} to X_{t_{i-1}}.  The stabilization
 * stage is t_st full steps, the last of which stores the KV cache; forced_k[n_forced] are
 * 0-based forward step counters (k = T - i) of forced full steps inside the region-aware
 * stage; every segment of region steps is closed by one storing full step; the last
 * segment's closing step is the first of the t_sm smooth steps.  Writes the steps in the
 * order they run.  seg_next of a region step is the index `next` of its segment (the
 * unedited rows jump to t_{next+1} at the segment's first step); -1 for full steps.
 * Returns REGIONE_ERR_INVALID_ARG if the stages do not fit T or max_steps is too small. */
enum { REGIONE_STEP_FULL = 0, REGIONE_STEP_FULL_STORE = 1, REGIONE_STEP_REGION = 2 };
typedef struct regione_plan_step {
    int32_t i;         /* timestep index of the step */
    int32_t kind;      /* REGIONE_STEP_* */
    int32_t seg_first; /* 1 for the first region step of a segment, else 0 */
    int32_t seg_next;  /* region steps: `next` of the segment; full steps: -1 */
} regione_plan_step;
int regione_stage_plan_host(int32_t T, int32_t t_st, int32_t t_sm, const int32_t* forced_k, int32_t n_forced,
                            regione_plan_step* steps_out, int32_t max_steps, int32_t* n_steps_out);

/* Classifier-free guidance ("Experimental Settings": on in every experiment of the paper): the
 * velocity the sampler uses, out[i] = v_uncond[i] + scale * (v_cond[i] - v_uncond[i]), in
 * float32; the three arrays have n_elems elements of `dtype`, out may be one of the inputs. */
int regione_guidance_combine(regione_ctx* ctx, const void* v_cond, const void* v_uncond, float scale, void* out,
                             int64_t n_elems, int32_t dtype);

/* Sums behind the relative change |v_new - v_old|_2 / |v_old|_2 of two velocities:
 * out[0] = sum (v_new - v_old)^2, out[1] = sum v_old^2 (float64 on the device, fixed order).
 * NOT the paper's reuse criterion (Eq.8 depends on the schedule alone): a data-dependent trigger
 * (reuse of the decayed cached velocity while the velocity changes by less than a threshold in relative norm)
 * that the loop benchmark's workload description asks for; the sampling loop offers it beside
 * regione_velocity_decision_host.  The arrays have n_elems elements of `dtype`. */
/* out_host_opt: host double[2] or NULL; when given the call waits for the stream and copies the two sums there. */
int regione_rel_change(regione_ctx* ctx, const void* v_new, const void* v_old, int64_t n_elems, int32_t dtype, double* out,
                       double* out_host_opt);

/* Host side of that trigger (pure functions of the state, like regione_velocity_decision_host for Eq.8).  The state is
 * all zeros at the first region step of every segment.
 * regione_rel_decision_host, before a region step: *reuse = 1 and *factor = decay when the previous fresh step asked
 *   for a reuse and a cached velocity exists, else *reuse = 0, *factor = 1; the request is consumed, so two reuses
 *   never follow each other.
 * regione_rel_update_host, after a FRESH region step and before regione_velocity_cache overwrites the cache:
 *   sums_host_opt = the two sums of regione_rel_change(new velocity, cached velocity), or NULL when there is nothing to
 *   compare (no edited row).  With a cached velocity and sums, rel = sqrt(sums[0]) / sqrt(sums[1]) (infinity when the
 *   old norm is zero) and the NEXT step is asked to reuse iff rel < threshold; otherwise no reuse is asked for and rel
 *   is infinity.  Marks the cache as filled.  *rel_out_opt receives rel. */
typedef struct regione_rel_state {
    int32_t have_cache; /* the velocity cache holds a fresh velocity of this segment */
    int32_t reuse_next; /* the last fresh step changed little: the next step may reuse */
} regione_rel_state;
int regione_rel_decision_host(regione_rel_state* st, float decay, int32_t* reuse, float* factor);
int regione_rel_update_host(regione_rel_state* st, const double* sums_host_opt, float threshold, double* rel_out_opt);

/* Slot list of a region step whose text rows are fresh as well (Eq.6 as printed: the input is [X^P, X^E]):
 * slots[i] = i for i < n_txt, slots[n_txt + i] = index[i] + n_txt for i < n (n as in regione_gather): image row r sits
 * at position n_txt + r of the cached sequence.  slots: [n_txt + n_max] int32. */
int regione_fresh_slots(regione_ctx* ctx, const int32_t* index, const int32_t* n_dev, int64_t n_max, int32_t n_txt, int32_t* slots);

/* out[i] = b[i] + t * b_time[i] (float32, product and sum rounded separately): the bias of a token embedding that
 * carries the time, as the small editor around the blocks uses it (the paper keeps such details inside its DiT). */
int regione_time_bias(regione_ctx* ctx, const float* b, const float* b_time, float t, float* out, int32_t n);

/* Fitting the timestep-aware factor gamma of Eq.7 (the paper says only that it is fitted on sampled data and gives
 * no procedure; this is least squares through the origin).
 * regione_sq_norms: out[i] = sum of squares of vector i, for n_vectors contiguous vectors of
 *   vec_elems elements of `dtype` (16-byte aligned, vec_elems a multiple of 8 for bf16 / 4 for
 *   float32); out is [n_vectors] float64 on the device.  Squares and sums in float64, in a fixed
 *   order.  One call over the velocities a sampler has kept gives every |v_{t_j}|^2.
 * regione_gamma_fit_host: sq_norms_host [n_samples, n_steps+1] with entry [s][j] = |v_{t_j}|^2
 *   of sample s for j = 1..n_steps (column 0 unused), t_host as in
 *   regione_velocity_decision_host.  Writes gamma_out [n_steps+1]:
 *   gamma_j = (sum_s |v_j||v_{j+1}| / sum_s |v_{j+1}|^2) / (1 - (t_{j+1} - t_j)) for
 *   1 <= j < n_steps, and 1 at both ends. */
int regione_sq_norms(regione_ctx* ctx, const void* x, int32_t dtype, int64_t n_vectors, int64_t vec_elems, double* out);
int regione_gamma_fit_host(const double* sq_norms_host, int32_t n_samples, const float* t_host, int32_t n_steps,
                           float* gamma_out);

/* Adaptive velocity decay cache, host decision (Eq.7, Eq.8): pure function of the
 * schedule.  t_host has n_steps+1 entries with t[n_steps] = 1 and t[0] = 0; gamma_host has
 * n_steps+1 entries (gamma[j] corrects the step at index j).  For the step at index j
 * (1 <= j < n_steps) updates *st and returns *reuse (0: run the DiT and cache its velocity,
 * 1: use the cached velocity times *factor). */
int regione_velocity_decision_host(const float* t_host, const float* gamma_host, int32_t n_steps,
                                   float delta, int32_t j, regione_avd_state* st,
                                   int32_t* reuse, float* factor);

/* Adaptive velocity decay cache, device part (Eq.9) fused with the Euler update (Eq.4) on
 * the edited rows, for i < n rows of c channels (n as in regione_gather):
 *   reuse == 0: c_a = v_fresh;           v_used = v_fresh
 *   reuse != 0: c_a unchanged;           v_used = factor * c_a
 *   x_e -= dt * v_used;  v_out_opt (if non-null) = v_used.
 * All tensors [n, c] of `dtype`; float32 arithmetic. */
int regione_velocity_cache(regione_ctx* ctx, int32_t reuse, float factor, float dt,
                           const void* v_fresh_opt, void* c_a, void* v_out_opt, void* x_e,
                           const int32_t* n_dev, int64_t n_max, int32_t c, int32_t dtype);

/* regione_gather / regione_scatter for two tensors that share the index list, in one launch: the hidden rows and the
 * latent rows of the edited tokens (Algorithm 1 gathers both at the start of a region step and merges both at its end).
 * Arguments as in regione_gather / regione_scatter, once per tensor. */
int regione_gather_pair(regione_ctx* ctx, const void* src_a, int32_t row_elems_a, int32_t dtype_a, void* dst_a,
                        const void* src_b, int32_t row_elems_b, int32_t dtype_b, void* dst_b,
                        const int32_t* index, const int32_t* n_dev, int64_t n_max);
int regione_scatter_pair(regione_ctx* ctx, void* dst_full_a, int32_t row_elems_a, int32_t dtype_a, const void* src_a,
                         void* dst_full_b, int32_t row_elems_b, int32_t dtype_b, const void* src_b,
                         const int32_t* index, const int32_t* n_dev, int64_t n_max);

/* The velocity head of a fresh region step together with what Algorithm 1 does with its result, in one launch
 * instead of four: v = h_rows W^T + b (regione_linear), rounded to `dtype`; the velocity cache takes it and the edited
 * rows take their Euler step (regione_velocity_cache with reuse = 0: c_a = v, x_e -= dt * v, Eq.9 and Eq.4); and the
 * updated rows are written to x_full[index[i], :] (regione_scatter) when x_full_opt is given.  Results are those of the
 * three calls bit for bit.
 *   h_rows [n, hidden] bf16 (float32 in a float32 context), w_head_packed from [c, hidden], b_head_opt [c] float32,
 *   v_out_opt / c_a / x_e [n, c] and x_full_opt [rows, c] of `dtype`; n is a host count; hidden a multiple of 64. */
int regione_velocity_head(regione_ctx* ctx, const void* h_rows, const void* w_head_packed, const float* b_head_opt,
                          int32_t n, int32_t c, int32_t hidden, float dt, void* v_out_opt, void* c_a, void* x_e,
                          void* x_full_opt, const int32_t* index_opt, int32_t dtype);

/* The unedited rows' single jump (section "Region-Aware Generation": the unedited region is estimated in one step with
 * Eq.5 from the last full velocity), done where the merge by spatial position would put its result:
 *   x_full[index[i], :] -= dt * v_full[index[i], :]   for i < n   (n as in regione_gather),
 * product and difference rounded separately in float32, every other row untouched.  One launch in place of gathering the
 * rows of x and v, stepping them and scattering them back at the end of the segment: nothing reads the unedited rows of
 * the full latent in between.  x_full, v_full: [rows, c] of `dtype`, different tensors; indices distinct. */
int regione_euler_rows(regione_ctx* ctx, void* x_full, const void* v_full, const int32_t* index, const int32_t* n_dev,
                       int64_t n_max, int32_t c, int32_t dtype, float dt);

/* regione_block_forward with the block's dense projections in 8-bit floating point (the
 * E4M3 variant above: an extension with its own accuracy, selected only by calling this entry point).  Arguments as in
 * regione_block_forward; `w` supplies biases and modulation vectors (its bf16 weight pointers are not read), `w8` the
 * quantised weights: per stream and projection the packed codes (regione_pack_weight_fp8) and one float32 scale per
 * output feature (regione_quantize_rows_fp8 on the weight rows).  What is quantised, with one scale per row (token):
 *   - the LayerNorm + modulation results feeding the QKV and the MLP-up projection, quantised from their float32
 *     values inside the LayerNorm kernel (no bf16 rounding in between);
 *   - the attention output and the activated MLP rows (bf16 as in the bf16 block), by regione_quantize_rows_fp8's
 *     kernel.
 * Everything else — attention, K/V cache (bf16), gates, residual stream, flags, slots — is the bf16 block's.
 * The first call on a context allocates the workspace of the codes (max_fresh x (H + M) bytes and max_fresh scales),
 * which lives as long as the context.
 * A single-stream block has two projections: w_1 [3H+M, H] and w_2 [H, H+M] (w_qkv, w_o unused); the input of the
 * second is the joint row [attention | GELU(m)] of H + M columns, quantised as one row.
 * Restrictions: bf16 context, hidden <= 4096, hidden and mlp multiples of 128, hidden + mlp <= 16384 for single-stream
 * blocks; one guidance branch per call.
 * taps_opt (verification aid): when given, every non-null member receives a copy of that intermediate as the library
 * computed it, rows in the order of h_in, so that each stage can be checked against a reference fed with the
 * library's own input of that stage:
 *   u1_codes [n, H] uint8, u1_scale [n] (input of the QKV projection);   q [n, H] bf16 (its query rows);
 *   attn [n, H] bf16;   a_codes [n, H], a_scale [n] (input of the output projection);   h1 [n, H] float32;
 *   u2_codes [n, H], u2_scale [n] (input of MLP up);   m [n, M] bf16;   m_codes [n, M], m_scale [n].
 * Single-stream blocks: attn [n, H+M] (the joint row), a_codes [n, H+M], a_scale; h1, u2_*, m, m_* are not written. */
typedef struct regione_stream_weights_fp8 {
    const void* w_qkv; const float* s_qkv;   /* codes packed from [3H, H]; scales [3H] */
    const void* w_o;   const float* s_o;     /* [H, H];  [H]  */
    const void* w_1;   const float* s_1;     /* [M, H];  [M]  */
    const void* w_2;   const float* s_2;     /* [H, M];  [H]  */
} regione_stream_weights_fp8;
typedef struct regione_block_weights_fp8 { regione_stream_weights_fp8 txt, img; } regione_block_weights_fp8;
typedef struct regione_fp8_taps {
    void* u1_codes; float* u1_scale; void* q; void* attn; void* a_codes; float* a_scale; float* h1;
    void* u2_codes; float* u2_scale; void* m; void* m_codes; float* m_scale;
} regione_fp8_taps;
int regione_block_forward_fp8(regione_ctx* ctx, const regione_block_weights* w, const regione_block_weights_fp8* w8, int32_t block_type,
                              const void* h_in, void* h_out, int32_t h_dtype,
                              int32_t n_fresh, int32_t n_txt_fresh, const int32_t* slot_index, int32_t slot_offset,
                              void* k_cache, void* v_cache, int32_t n_all, int32_t flags, const regione_fp8_taps* taps_opt);

/* One region-aware step in one call: the body of Algorithm 1's region-aware stage for a stack of blocks, i.e. the
 * calls above in the order of the algorithm, queued by the library without returning to the caller in between:
 *   1. adaptive region partition (regione_partition on x_t, v, x_ref): mask, E/U index lists, count;
 *   2. gather of the edited tokens' hidden rows and latent rows (regione_gather_pair);
 *   3. every block with the retrieve flag on those rows (regione_block_forward, Eq.6), block i on k_caches[i],
 *      v_caches[i]; with n_txt_fresh > 0 the first n_txt_fresh rows of h_rows are text rows that the caller has put
 *      there, the gathered rows follow them, and `slots` receives the slot list (regione_fresh_slots);
 *   4. velocity head, velocity cache of a fresh step, Euler update and merge of the latent rows into x_next_full
 *      (regione_velocity_head; Eq.9, Eq.4);
 *   5. merge of the hidden rows into h_next_full (regione_scatter) when h_next_full_opt is given.
 * Results are those of the separate calls bit for bit.  What the single call saves is the wait between 1 and 2: the
 * count that sizes every later launch reaches the host through a pinned word that the index kernel writes first, so
 * the host queues the launches of 2-5 while the partition still runs, instead of waiting for the stream.
 *   x_t, v, x_ref, score_opt, mask, e_index, u_index, n_edited_dev: as in regione_partition (n_tokens image tokens).
 *   h_full [n_tokens, hidden] of h_dtype: hidden state of the image tokens entering the stack.
 *   h_rows, h_rows_out [n_txt_fresh + n_tokens, hidden] of h_dtype: work rows (may be the same buffer).
 *   x_e, c_a, v_out_opt [n_tokens, c] of `dtype`; x_next_full [n_tokens, c]: receives the edited rows' new latents.
 *   blocks / block_types / k_caches / v_caches: host arrays of n_blocks entries; slot_offset: slot of image token 0 in
 *   the cached sequence (the number of text tokens); slots [n_txt_fresh + n_tokens] int32, needed when n_txt_fresh > 0.
 *   *n_edited_host receives the count.  With no edited token the call ends after step 1. */
typedef struct regione_region_step_args {
    const void* x_t; const void* v; const void* x_ref;
    int64_t n_tokens; int32_t c; int32_t dtype; float sigma_t; float eta;
    float* score_opt; uint8_t* mask; int32_t* e_index; int32_t* u_index; int32_t* n_edited_dev;
    const void* h_full; int32_t h_dtype; int32_t n_txt_fresh;
    void* h_rows; void* h_rows_out; int32_t* slots;
    int32_t n_blocks; int32_t n_all; int32_t slot_offset; int32_t reserved;
    const regione_block_weights* blocks; const int32_t* block_types; void* const* k_caches; void* const* v_caches;
    const void* w_head_packed; const float* b_head_opt; float dt; int32_t reserved2;
    void* v_out_opt; void* c_a; void* x_e; void* x_next_full; void* h_next_full_opt;
} regione_region_step_args;
int regione_region_step(regione_ctx* ctx, const regione_region_step_args* args, int32_t* n_edited_host);

#ifdef __cplusplus
}
#endif
#endif /* REGIONE_H */
