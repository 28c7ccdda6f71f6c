// Adaptive region partition: one-step estimate (Eq.5 with t_f = 0), per-token cosine score
// against the reference latent, threshold, and a deterministic three-kernel compaction of the
// edited / unedited index lists (Algorithm 1, ARP lines; section "Adaptive Region Partition").
//
// Kernel 1 streams x_t, v, x_ref once (16-byte loads, a group of LPT lanes per token), reduces
// the three sums in float64 inside the lane group, writes score and mask and one edited count
// per block.  Kernel 2 (one workgroup) turns the counts into exclusive offsets; kernel 3 writes the
// index lists with a ballot/popcount rank.  No atomics, so the lists come out in ascending order.
#include "common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

template <typename T> struct Vec16;
template <> struct Vec16<bf16_t> { static constexpr int N = 8; };
template <> struct Vec16<float> { static constexpr int N = 4; };

template <typename T, int VEC>
__device__ __forceinline__ void load_chunk(const T* p, float (&out)[VEC]);

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// The three inputs are read exactly once: non-temporal loads keep them from displacing anything in the caches
// (measured on MI355X: 6.9 TB/s for a read-only stream with them against 6.1 TB/s without).
template <> __device__ __forceinline__ void load_chunk<bf16_t, 8>(const bf16_t* p, float (&out)[8]) {
    const u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    uint32_t w[4] = {r[0], r[1], r[2], r[3]};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = __uint_as_float(w[i] << 16);
        out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
template <> __device__ __forceinline__ void load_chunk<float, 4>(const float* p, float (&out)[4]) {
    const f32x4 r = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    out[0] = r[0]; out[1] = r[1]; out[2] = r[2]; out[3] = r[3];
}
template <> __device__ __forceinline__ void load_chunk<bf16_t, 1>(const bf16_t* p, float (&out)[1]) { out[0] = bf16_to_f32(*p); }
template <> __device__ __forceinline__ void load_chunk<float, 1>(const float* p, float (&out)[1]) { out[0] = *p; }

__device__ __forceinline__ double shfl_xor_f64(double x, int m) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __shfl_xor(lo, m, 64);
    hi = __shfl_xor(hi, m, 64);
    return __hiloint2double(hi, lo);
}

// One block handles tokens [blockIdx.x * tok_per_block, +tok_per_block).
template <typename T, int VEC, int LPT>
__global__ void __launch_bounds__(kThreads)
score_mask_kernel(const T* __restrict__ x_t, const T* __restrict__ v, const T* __restrict__ x_ref,
                  int64_t n_tokens, int c, int tok_per_block, float sigma, float eta,
                  float* __restrict__ score, uint8_t* __restrict__ mask, int32_t* __restrict__ counts) {
    constexpr int TOK_PER_WAVE = 64 / LPT;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPT, tok_in_wave = lane / LPT;
    const int nchunks = c / VEC;
    const int64_t block_first = static_cast<int64_t>(blockIdx.x) * tok_per_block;
    int edited_count = 0;
    // Tokens past the end re-read token 0 (valid memory) and are dropped afterwards, so the loads are branch free.
    // Two passes are handled together: all their loads are issued before the first reduction starts (four at a time
    // cost too many registers for the float64 sums and ran slower).
    constexpr int UNROLL = 2;
    constexpr int PASS_STRIDE = kWaves * TOK_PER_WAVE;
    for (int pass0 = wave * TOK_PER_WAVE; pass0 < tok_per_block; pass0 += UNROLL * PASS_STRIDE) {
        double dot[UNROLL], na[UNROLL], nb[UNROLL];
        int64_t tok[UNROLL];
        bool live[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int pass = pass0 + u * PASS_STRIDE;
            tok[u] = block_first + pass + tok_in_wave;
            live[u] = (pass + tok_in_wave) < tok_per_block && tok[u] < n_tokens;
            dot[u] = 0.0; na[u] = 0.0; nb[u] = 0.0;
        }
        for (int ch = sub; ch < nchunks; ch += LPT) {
            float a[UNROLL][VEC], b[UNROLL][VEC], r[UNROLL][VEC];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int64_t base = (live[u] ? tok[u] : 0) * c + ch * VEC;
                load_chunk<T, VEC>(x_t + base, a[u]);
                load_chunk<T, VEC>(v + base, b[u]);
                load_chunk<T, VEC>(x_ref + base, r[u]);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    const float est = __fsub_rn(a[u][i], __fmul_rn(sigma, b[u][i]));  // two roundings, never an fma
                    const double e = est, rr = r[u][i];
                    dot[u] = fma(e, rr, dot[u]);
                    na[u] = fma(e, e, na[u]);
                    nb[u] = fma(rr, rr, nb[u]);
                }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
            for (int m = 1; m < LPT; m <<= 1) {
                dot[u] += shfl_xor_f64(dot[u], m);
                na[u] += shfl_xor_f64(na[u], m);
                nb[u] += shfl_xor_f64(nb[u], m);
            }
            bool edited = false;
            if (live[u] && sub == 0) {
                const double denom = fmax(sqrt(na[u]) * sqrt(nb[u]), 1e-8);
                const float s = static_cast<float>(dot[u] / denom);
                edited = !(s > eta);
                if (score) score[tok[u]] = s;
                mask[tok[u]] = edited ? 1 : 0;
            }
            edited_count += __popcll(__ballot(edited));
        }
    }
    __shared__ int wave_counts[kWaves];
    if (lane == 0) wave_counts[wave] = edited_count;
    __syncthreads();
    if (threadIdx.x == 0) {
        int s = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += wave_counts[w];
        counts[blockIdx.x] = s;
    }
}

// Exclusive prefix sum of the per-block counts, in place, by one workgroup: thread t owns a contiguous run of
// entries.  Also writes the total.
constexpr int kScanThreads = 1024;
__global__ void __launch_bounds__(kScanThreads)
scan_counts_kernel(int32_t* __restrict__ counts, int n_blocks, int32_t* __restrict__ n_edited, int32_t* __restrict__ n_edited_pinned) {
    __shared__ int wave_sum[kScanThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int per = (n_blocks + kScanThreads - 1) / kScanThreads;
    const int first = threadIdx.x * per;
    int local = 0;
    for (int i = first; i < first + per && i < n_blocks; ++i) local += counts[i];
    // inclusive scan of `local` inside the wave, then across the waves
    int incl = local;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; ++w) { if (w < wave) before += wave_sum[w]; total += wave_sum[w]; }
    int run = before + incl - local;   // exclusive prefix of this thread's first entry
    for (int i = first; i < first + per && i < n_blocks; ++i) { const int cnt = counts[i]; counts[i] = run; run += cnt; }
    if (threadIdx.x == 0) { *n_edited = total; *n_edited_pinned = total; }
}

// SUMS = false: `offsets` holds the exclusive prefix sums of the per-block counts (scan_counts_kernel ran).
// SUMS = true (few blocks): `offsets` holds the raw counts; every block adds up the counts of the blocks before it
// itself, and the last block writes the total, which saves the scan kernel's launch.
template <bool SUMS>
__global__ void __launch_bounds__(kThreads)
write_index_kernel(const uint8_t* __restrict__ mask, const int32_t* __restrict__ offsets,
                   int64_t n_tokens, int tok_per_block,
                   int32_t* __restrict__ e_index, int32_t* __restrict__ u_index,
                   int32_t* __restrict__ n_edited, int32_t* __restrict__ n_edited_pinned) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __shared__ int wave_e[kWaves];
    int base_e;
    if (SUMS) {
        int part = 0;
        for (int b = threadIdx.x; b < static_cast<int>(blockIdx.x); b += kThreads) part += offsets[b];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) part += __shfl_xor(part, d, 64);
        if (lane == 0) wave_e[wave] = part;
        __syncthreads();
        base_e = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) base_e += wave_e[w];
        if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
            const int total = base_e + offsets[blockIdx.x];
            *n_edited = total;
            *n_edited_pinned = total;
        }
        // (the first round below starts with a barrier, so wave_e can be reused)
    } else {
        base_e = offsets[blockIdx.x];   // edited tokens in all blocks before this one
    }
    const int64_t block_first = static_cast<int64_t>(blockIdx.x) * tok_per_block;
    int64_t base_u = block_first - base_e;
    for (int off = 0; off < tok_per_block; off += kThreads) {
        const int64_t tok = block_first + off + threadIdx.x;
        const bool live = (off + static_cast<int>(threadIdx.x)) < tok_per_block && tok < n_tokens;
        const bool ed = live && mask[tok] != 0;
        const unsigned long long bal = __ballot(ed);
        const int rank_in_wave = __popcll(bal & ((1ull << lane) - 1ull));
        __syncthreads();  // wave_e of the previous round has been read
        if (lane == 0) wave_e[wave] = __popcll(bal);
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) { if (w < wave) before += wave_e[w]; total += wave_e[w]; }
        const int rank_e = before + rank_in_wave;                      // edited tokens before this one in the round
        const int pos_in_round = static_cast<int>(threadIdx.x);
        if (live) {
            if (ed) e_index[base_e + rank_e] = static_cast<int32_t>(tok);
            else u_index[base_u + (pos_in_round - rank_e)] = static_cast<int32_t>(tok);
        }
        base_e += total;
        base_u += kThreads - total;   // tail rounds past n_tokens write nothing, so over-counting there is harmless
    }
}

__global__ void set_i32_kernel(int32_t* p, int32_t* p_pinned, int32_t v) { *p = v; *p_pinned = v; }

template <typename T, int VEC>
int launch_score(hipStream_t stream, int32_t* counts, int lpt, dim3 grid, const void* x_t, const void* v, const void* x_ref, int64_t n, int c,
                 int tpb, float sigma, float eta, float* score, uint8_t* mask) {
    const T* a = static_cast<const T*>(x_t); const T* b = static_cast<const T*>(v); const T* r = static_cast<const T*>(x_ref);
#define RG_CASE(L) case L: hipLaunchKernelGGL((score_mask_kernel<T, VEC, L>), grid, dim3(kThreads), 0, stream, \
        a, b, r, n, c, tpb, sigma, eta, score, mask, counts); break;
    switch (lpt) { RG_CASE(1) RG_CASE(2) RG_CASE(4) RG_CASE(8) RG_CASE(16) RG_CASE(32) RG_CASE(64)
        default: RG_FAIL(REGIONE_ERR_INVALID_ARG, "partition: bad lane group %d", lpt); }
#undef RG_CASE
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

// ---- morphological clean-up of the partition on the token grid
// One workgroup per image.  The unedited map lives in LDS as bytes; four passes with the 3x3 square (erosion,
// dilation = opening; dilation, erosion = closing), cells outside the grid never decide.  Writes the cleaned
// edited mask.
constexpr int kMorphThreads = 1024;
constexpr int kMorphMaxCells = 128 * 128;
template <bool ERODE>
__device__ __forceinline__ void morph_pass(const uint8_t* __restrict__ in, uint8_t* __restrict__ out, int gh, int gw) {
    for (int p = threadIdx.x; p < gh * gw; p += kMorphThreads) {
        const int r = p / gw, c = p - r * gw;
        bool acc = ERODE;
        for (int dr = -1; dr <= 1; ++dr) {
            const int rr = r + dr;
            if (rr < 0 || rr >= gh) continue;
            for (int dc = -1; dc <= 1; ++dc) {
                const int cc = c + dc;
                if (cc < 0 || cc >= gw) continue;
                const bool v = in[rr * gw + cc] != 0;
                acc = ERODE ? (acc && v) : (acc || v);
            }
        }
        out[p] = acc ? 1 : 0;
    }
    __syncthreads();
}
__global__ void __launch_bounds__(kMorphThreads)
morph_open_close_kernel(const uint8_t* mask_in, uint8_t* mask_out, int gh, int gw) {   // the two may be the same buffer
    __shared__ uint8_t a[kMorphMaxCells], b[kMorphMaxCells];
    const int cells = gh * gw;
    const int64_t base = static_cast<int64_t>(blockIdx.x) * cells;
    for (int p = threadIdx.x; p < cells; p += kMorphThreads) a[p] = mask_in[base + p] ? 0 : 1;   // unedited map
    __syncthreads();
    morph_pass<true>(a, b, gh, gw);    // opening: erosion ...
    morph_pass<false>(b, a, gh, gw);   // ... then dilation
    morph_pass<false>(a, b, gh, gw);   // closing: dilation ...
    morph_pass<true>(b, a, gh, gw);    // ... then erosion
    for (int p = threadIdx.x; p < cells; p += kMorphThreads) mask_out[base + p] = a[p] ? 0 : 1;
}

// edited tokens per block of tok_per_block tokens (the layout scan_counts_kernel and write_index_kernel expect)
__global__ void __launch_bounds__(kThreads)
count_mask_kernel(const uint8_t* __restrict__ mask, int64_t n_tokens, int tok_per_block, int32_t* __restrict__ counts) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t block_first = static_cast<int64_t>(blockIdx.x) * tok_per_block;
    int cnt = 0;
    for (int off = threadIdx.x; off < tok_per_block; off += kThreads) {
        const int64_t tok = block_first + off;
        cnt += (tok < n_tokens && mask[tok] != 0) ? 1 : 0;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) cnt += __shfl_xor(cnt, d, 64);
    __shared__ int wave_counts[kWaves];
    if (lane == 0) wave_counts[wave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        int s = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += wave_counts[w];
        counts[blockIdx.x] = s;
    }
}

// Index lists from the mask and the per-block counts in `counts`: few blocks -> one launch, else scan + lists.
// n_edited_copy: a second place for the count (the context's pinned host word; n_edited_dev itself when there is none).
int launch_index_lists(hipStream_t stream, int32_t* counts, dim3 grid, const uint8_t* mask, int64_t n_tokens, int tpb,
                       int32_t* e_index, int32_t* u_index, int32_t* n_edited_dev, int32_t* n_edited_copy) {
    if (grid.x <= 1024) {
        hipLaunchKernelGGL((write_index_kernel<true>), grid, dim3(kThreads), 0, stream,
                           mask, counts, n_tokens, tpb, e_index, u_index, n_edited_dev, n_edited_copy);
        RG_LAUNCH_CHECK();
        return REGIONE_OK;
    }
    hipLaunchKernelGGL(scan_counts_kernel, dim3(1), dim3(kScanThreads), 0, stream, counts, static_cast<int>(grid.x), n_edited_dev, n_edited_copy);
    RG_LAUNCH_CHECK();
    hipLaunchKernelGGL((write_index_kernel<false>), grid, dim3(kThreads), 0, stream,
                       mask, counts, n_tokens, tpb, e_index, u_index, n_edited_dev, n_edited_copy);
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

// The launches of the partition on `stream` with the per-block counts in `counts` (room for counts_cap entries).
int partition_launches(hipStream_t stream, int32_t* counts, int64_t counts_cap, const void* x_t, const void* v, const void* x_ref,
                       int64_t n_tokens, int32_t c, int32_t dtype, float sigma_t, float eta, float* score_opt, uint8_t* mask,
                       int32_t* e_index, int32_t* u_index, int32_t* n_edited_dev, int32_t* n_edited_copy) {
    if (n_tokens == 0) {
        hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(1), 0, stream, n_edited_dev, n_edited_copy, 0);
        RG_LAUNCH_CHECK();
        return REGIONE_OK;
    }
    const int full_vec = dtype == REGIONE_BF16 ? 8 : 4;
    const int vec = (c % full_vec == 0) ? full_vec : 1;
    const int nchunks = c / vec;
    int lpt = 1;
    while (lpt * 2 <= nchunks && lpt < 64) lpt *= 2;
    const int tok_per_pass = kWaves * (64 / lpt);
    // small inputs: few passes per block so that one image still spreads over many CUs
    int passes = 1;
    while (passes < 32 && (n_tokens / (static_cast<int64_t>(tok_per_pass) * passes * 2)) >= 2048) passes *= 2;
    const int tpb = tok_per_pass * passes;
    const int64_t nblocks = (n_tokens + tpb - 1) / tpb;
    if (nblocks > counts_cap) RG_FAIL(REGIONE_ERR_WORKSPACE, "partition: %lld blocks exceed the %lld the workspace holds", (long long)nblocks, (long long)counts_cap);
    dim3 grid(static_cast<unsigned>(nblocks));
    int rc;
    if (dtype == REGIONE_BF16) {
        rc = vec == 8 ? launch_score<bf16_t, 8>(stream, counts, lpt, grid, x_t, v, x_ref, n_tokens, c, tpb, sigma_t, eta, score_opt, mask)
                      : launch_score<bf16_t, 1>(stream, counts, lpt, grid, x_t, v, x_ref, n_tokens, c, tpb, sigma_t, eta, score_opt, mask);
    } else {
        rc = vec == 4 ? launch_score<float, 4>(stream, counts, lpt, grid, x_t, v, x_ref, n_tokens, c, tpb, sigma_t, eta, score_opt, mask)
                      : launch_score<float, 1>(stream, counts, lpt, grid, x_t, v, x_ref, n_tokens, c, tpb, sigma_t, eta, score_opt, mask);
    }
    if (rc != REGIONE_OK) return rc;
    return launch_index_lists(stream, counts, grid, mask, n_tokens, tpb, e_index, u_index, n_edited_dev, n_edited_copy);
}

int check_partition_args(const char* who, const void* x_t, const void* v, const void* x_ref, int64_t n_tokens, int32_t c, int32_t dtype,
                         const uint8_t* mask, const int32_t* e_index, const int32_t* u_index, const int32_t* n_edited_dev) {
    if (n_tokens < 0 || c <= 0) RG_FAIL(REGIONE_ERR_INVALID_ARG, "%s: n_tokens=%lld c=%d", who, (long long)n_tokens, c);
    if (dtype != REGIONE_BF16 && dtype != REGIONE_FP32) RG_FAIL(REGIONE_ERR_INVALID_ARG, "%s: bad dtype %d", who, dtype);
    if (!n_edited_dev) RG_FAIL(REGIONE_ERR_INVALID_ARG, "%s: n_edited_dev is null", who);
    if (n_tokens > 0) {
        if (!x_t || !v || !x_ref || !mask || !e_index || !u_index) RG_FAIL(REGIONE_ERR_INVALID_ARG, "%s: null tensor", who);
        if (!rg_aligned16(x_t) || !rg_aligned16(v) || !rg_aligned16(x_ref)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "%s: inputs must be 16-byte aligned", who);
    }
    return REGIONE_OK;
}

}  // namespace

extern "C" int regione_partition(regione_ctx* ctx, const void* x_t, const void* v, const void* x_ref,
                                 int64_t n_tokens, int32_t c, int32_t dtype, float sigma_t, float eta,
                                 float* score_opt, uint8_t* mask, int32_t* e_index, int32_t* u_index,
                                 int32_t* n_edited_dev, int32_t* n_edited_host_opt) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "partition: null context");
    if (int rc = check_partition_args("partition", x_t, v, x_ref, n_tokens, c, dtype, mask, e_index, u_index, n_edited_dev)) return rc;
    if (n_tokens > ctx->dims.max_tokens) RG_FAIL(REGIONE_ERR_WORKSPACE, "partition: %lld tokens, context made for %d", (long long)n_tokens, ctx->dims.max_tokens);
    {
    ProfScope prof(ctx, REGIONE_PROF_PARTITION);
    if (int rc = partition_launches(ctx->stream, ctx->part_counts, ctx->part_counts_cap, x_t, v, x_ref, n_tokens, c, dtype, sigma_t, eta,
                                    score_opt, mask, e_index, u_index, n_edited_dev, ctx->n_edited_pinned_dev)) return rc;
    }
    if (n_edited_host_opt) {   // the kernels wrote the count to pinned host memory too: no copy to wait for, only the stream
        RG_HIP(hipStreamSynchronize(ctx->stream));
        *n_edited_host_opt = *static_cast<volatile int32_t*>(ctx->n_edited_pinned);
    }
    return REGIONE_OK;
}

extern "C" int regione_mask_cleanup(regione_ctx* ctx, const uint8_t* mask_in, int32_t grid_h, int32_t grid_w, int32_t n_images,
                                    uint8_t* mask_out, int32_t* e_index, int32_t* u_index,
                                    int32_t* n_edited_dev, int32_t* n_edited_host_opt) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "mask_cleanup: null context");
    if (grid_h <= 0 || grid_w <= 0 || n_images < 0) RG_FAIL(REGIONE_ERR_INVALID_ARG, "mask_cleanup: grid %d x %d, %d images", grid_h, grid_w, n_images);
    if (static_cast<int64_t>(grid_h) * grid_w > kMorphMaxCells) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "mask_cleanup: grid %d x %d exceeds %d cells per image", grid_h, grid_w, kMorphMaxCells);
    if (!n_edited_dev) RG_FAIL(REGIONE_ERR_INVALID_ARG, "mask_cleanup: n_edited_dev is null");
    const int64_t n_tokens = static_cast<int64_t>(grid_h) * grid_w * n_images;
    if (n_tokens > ctx->dims.max_tokens) RG_FAIL(REGIONE_ERR_WORKSPACE, "mask_cleanup: %lld tokens, context made for %d", (long long)n_tokens, ctx->dims.max_tokens);
    {
    ProfScope prof(ctx, REGIONE_PROF_PARTITION);
    if (n_tokens == 0) {
        hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(1), 0, ctx->stream, n_edited_dev, ctx->n_edited_pinned_dev, 0);
        RG_LAUNCH_CHECK();
    } else {
        if (!mask_in || !mask_out || !e_index || !u_index) RG_FAIL(REGIONE_ERR_INVALID_ARG, "mask_cleanup: null tensor");
        const int tpb = kThreads;
        const int64_t nblocks = (n_tokens + tpb - 1) / tpb;
        if (nblocks > ctx->part_counts_cap) RG_FAIL(REGIONE_ERR_WORKSPACE, "mask_cleanup: %lld blocks exceed the workspace", (long long)nblocks);
        hipLaunchKernelGGL(morph_open_close_kernel, dim3(static_cast<unsigned>(n_images)), dim3(kMorphThreads), 0, ctx->stream, mask_in, mask_out, grid_h, grid_w);
        RG_LAUNCH_CHECK();
        const dim3 grid(static_cast<unsigned>(nblocks));
        hipLaunchKernelGGL(count_mask_kernel, grid, dim3(kThreads), 0, ctx->stream, mask_out, n_tokens, tpb, ctx->part_counts);
        RG_LAUNCH_CHECK();
        if (int rc2 = launch_index_lists(ctx->stream, ctx->part_counts, grid, mask_out, n_tokens, tpb, e_index, u_index, n_edited_dev, ctx->n_edited_pinned_dev)) return rc2;
    }
    }
    if (n_edited_host_opt) {   // the kernels wrote the count to pinned host memory too: no copy to wait for, only the stream
        RG_HIP(hipStreamSynchronize(ctx->stream));
        *n_edited_host_opt = *static_cast<volatile int32_t*>(ctx->n_edited_pinned);
    }
    return REGIONE_OK;
}

// ---- the partition for callers that cannot allocate device memory
// Same kernels as regione_partition; the per-block counts live in a static device array instead of a context's
// workspace.  Every GPU holds its own copy of the array at its own address, looked up once per device.
#define RG_STATIC_COUNTS 65536                       /* int32 entries: 256 KiB per GPU, held until the process ends */
static __device__ __align__(256) int32_t scratch[RG_STATIC_COUNTS];

namespace {

constexpr int64_t kStaticCounts = RG_STATIC_COUNTS;
constexpr int64_t kStaticMaxTokens = int64_t{1} << 22;
constexpr int kMaxDevices = 64;

int32_t* g_scratch_ptr[kMaxDevices];                 // device address of `scratch` on each device, null until looked up

// Address of this device's copy of `scratch` (host code must never pass the array's name to a kernel: on the host it
// is a stand-in, not a device address).
int scratch_for_current_device(int32_t** out) {
    int dev = -1;
    RG_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "partition_static: device ordinal %d (at most %d devices)", dev, kMaxDevices);
    int32_t* p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        void* sym = nullptr;
        RG_HIP(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
        if (!sym) RG_FAIL(REGIONE_ERR_HIP, "partition_static: the scratch symbol has no address on device %d", dev);
        p = static_cast<int32_t*>(sym);
        __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);   // every thread looks up the same address: a race is harmless
    }
    *out = p;
    return REGIONE_OK;
}

}  // namespace

int rg_partition_static_warm(void) {
    int32_t* p = nullptr;
    return scratch_for_current_device(&p);
}

extern "C" int regione_partition_static(void* hip_stream, const void* x_t, const void* v, const void* x_ref,
                                        int64_t n_tokens, int32_t c, int32_t dtype, float sigma_t, float eta,
                                        float* score_opt, uint8_t* mask, int32_t* e_index, int32_t* u_index,
                                        int32_t* n_edited_dev) {
    if (int rc = check_partition_args("partition_static", x_t, v, x_ref, n_tokens, c, dtype, mask, e_index, u_index, n_edited_dev)) return rc;
    if (n_tokens > kStaticMaxTokens)
        RG_FAIL(REGIONE_ERR_WORKSPACE, "partition_static: %lld tokens exceed the limit of %lld of the entry point that allocates nothing",
                (long long)n_tokens, (long long)kStaticMaxTokens);
    int32_t* counts = nullptr;
    if (int rc = scratch_for_current_device(&counts)) return rc;
    // Nothing in the array has to start at zero: the score kernel writes the count of every block of this call before
    // the index kernels read them, and entries past the call's block count are never read.
    return partition_launches(static_cast<hipStream_t>(hip_stream), counts, kStaticCounts, x_t, v, x_ref, n_tokens, c, dtype, sigma_t, eta,
                              score_opt, mask, e_index, u_index, n_edited_dev, n_edited_dev);
}
