// Adaptive region partition: one-step estimate (Eq.5 with t_f = 0), per-token cosine score
// against the reference latent, threshold, and a deterministic compaction of the edited /
// unedited index lists (Algorithm 1, ARP lines; section "Adaptive Region Partition").
//
// Kernel 1 streams x_t, v, x_ref once (16-byte loads, a group of LPT lanes per token, the loads of
// the next tokens in flight while the current ones are reduced), sums in float64 inside the lane
// group, and leaves the three sums of every token of its block in LDS; one thread per token then
// forms the score and the decision.  It writes ONE BIT per token (and the score, if asked for) and
// one edited count per block: on MI355X a trickle of small writes inside a read stream costs far
// more than its bytes (measured on 8.4 M tokens: 463 us without the 5 bytes per token of score and
// byte mask, 548 us with them).  Kernel 2 (one workgroup, only for many blocks) turns the counts
// into exclusive offsets; kernel 3 expands the bits into the byte mask and writes the index lists
// with a popcount rank.  No atomics, so the lists come out in ascending order.
#include "common.h"
#include <atomic>
#include <chrono>
#include <climits>

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxBlockTokens = 1024;   // tokens per workgroup of the score kernel (LDS: three float64 sums per token)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// One chunk of VEC elements as loaded (raw) and as floats.  The three inputs are read exactly once: non-temporal loads
// keep them from displacing anything in the caches (6.9 TB/s for a read-only stream with them against 6.1 without).
template <typename T, int VEC> struct Chunk;
template <> struct Chunk<bf16_t, 8> {
    u32x4 raw;
    __device__ __forceinline__ void load(const bf16_t* p) { raw = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)); }
    __device__ __forceinline__ void unpack(float (&out)[8]) const {
#pragma unroll
        for (int i = 0; i < 4; ++i) { out[2 * i] = __uint_as_float(raw[i] << 16); out[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u); }
    }
};
template <> struct Chunk<float, 4> {
    f32x4 raw;
    __device__ __forceinline__ void load(const float* p) { raw = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p)); }
    __device__ __forceinline__ void unpack(float (&out)[4]) const { out[0] = raw[0]; out[1] = raw[1]; out[2] = raw[2]; out[3] = raw[3]; }
};
template <> struct Chunk<bf16_t, 1> {
    bf16_t raw;
    __device__ __forceinline__ void load(const bf16_t* p) { raw = *p; }
    __device__ __forceinline__ void unpack(float (&out)[1]) const { out[0] = bf16_to_f32(raw); }
};
template <> struct Chunk<float, 1> {
    float raw;
    __device__ __forceinline__ void load(const float* p) { raw = *p; }
    __device__ __forceinline__ void unpack(float (&out)[1]) const { out[0] = raw; }
};

__device__ __forceinline__ double shfl_xor_f64(double x, int m) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __shfl_xor(lo, m, 64);
    hi = __shfl_xor(hi, m, 64);
    return __hiloint2double(hi, lo);
}
// The value of another lane of the same row of 16 through the data-parallel-primitive path of the vector ALU (no trip
// through LDS as with a shuffle).  CTRL: 0xB1 = lanes xor 1, 0x4E = xor 2, 0x141 = i <-> 7 - i, 0x140 = i <-> 15 - i.
template <int CTRL> __device__ __forceinline__ double dpp_f64(double x) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xf, 0xf, true);
    hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}
// Sum over the LPT lanes of a token's group, the same in every lane of the group.  After the xor-1 and xor-2 steps the
// four lanes of a quad agree, so the mirrored lane of the other quad (then of the other half row) holds the partner's sum.
template <int LPT> __device__ __forceinline__ double group_sum(double x) {
    if (LPT >= 2) x += dpp_f64<0xB1>(x);
    if (LPT >= 4) x += dpp_f64<0x4E>(x);
    if (LPT >= 8) x += dpp_f64<0x141>(x);
    if (LPT >= 16) x += dpp_f64<0x140>(x);
    if (LPT >= 32) x += shfl_xor_f64(x, 16);
    if (LPT >= 64) x += shfl_xor_f64(x, 32);
    return x;
}

// One block handles tokens [blockIdx.x * tok_per_block, +tok_per_block); tok_per_block is a multiple of 64 and at most
// kMaxBlockTokens.  PIPE: every lane owns exactly one chunk of its token (c == VEC * LPT) and the chunks of the next
// STAGE tokens are requested before the current ones are reduced.  Otherwise a lane loops over its chunks.
// bits: one 64-bit word per 64 tokens, bit = edited; words of tokens past n_tokens are written with those bits clear.
template <typename T, int VEC, int LPT, bool PIPE>
__global__ void __launch_bounds__(kThreads)
score_bits_kernel(const T* __restrict__ x_t, const T* __restrict__ v, const T* __restrict__ x_ref,
                  int64_t n_tokens, int c, int tok_per_block, float sigma, float eta,
                  float* __restrict__ score, uint64_t* __restrict__ bits, int32_t* __restrict__ counts) {
    constexpr int TPW = 64 / LPT;                       // tokens per wave and pass
    constexpr int STAGE = 2;                            // passes whose loads travel together
    constexpr int STAGE_TOK = kWaves * TPW * STAGE;     // tokens per workgroup and stage
    __shared__ double s_sum[3][kMaxBlockTokens];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPT, tiw = lane / LPT;
    const int64_t block_first = static_cast<int64_t>(blockIdx.x) * tok_per_block;
    int64_t left = n_tokens - block_first;
    const int block_tokens = static_cast<int>(left < tok_per_block ? left : tok_per_block);
    const int n_stage = (block_tokens + STAGE_TOK - 1) / STAGE_TOK;
    auto tok_of = [&](int st, int u) { return st * STAGE_TOK + (u * kWaves + wave) * TPW + tiw; };   // token inside the block

    auto accumulate = [&](const Chunk<T, VEC>& ca, const Chunk<T, VEC>& cb, const Chunk<T, VEC>& cr, double& dot, double& na, double& nb) __attribute__((always_inline)) {
        float a[VEC], b[VEC], r[VEC];
        ca.unpack(a); cb.unpack(b); cr.unpack(r);
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            const float est = __fsub_rn(a[i], __fmul_rn(sigma, b[i]));  // two roundings, never an fma
            const double e = est, rr = r[i];
            dot = fma(e, rr, dot);
            na = fma(e, e, na);
            nb = fma(rr, rr, nb);
        }
    };
    auto finish = [&](int t, double dot, double na, double nb) __attribute__((always_inline)) {
        dot = group_sum<LPT>(dot); na = group_sum<LPT>(na); nb = group_sum<LPT>(nb);
        if (sub == 0 && t < block_tokens) { s_sum[0][t] = dot; s_sum[1][t] = na; s_sum[2][t] = nb; }
    };

    if (PIPE) {
        // tokens past the end of the block re-read its first token (valid memory) and are dropped afterwards
        Chunk<T, VEC> ra[2][STAGE], rb[2][STAGE], rr[2][STAGE];
        auto issue = [&](int st, int buf) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < STAGE; ++u) {
                const int t = tok_of(st, u);
                const int64_t base = (block_first + (t < block_tokens ? t : 0)) * c + sub * VEC;
                ra[buf][u].load(x_t + base); rb[buf][u].load(v + base); rr[buf][u].load(x_ref + base);
            }
        };
        auto reduce = [&](int st, int buf) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < STAGE; ++u) {
                double dot = 0.0, na = 0.0, nb = 0.0;
                accumulate(ra[buf][u], rb[buf][u], rr[buf][u], dot, na, nb);
                finish(tok_of(st, u), dot, na, nb);
            }
        };
        if (n_stage > 0) issue(0, 0);
        for (int st = 0; st < n_stage; st += 2) {
            if (st + 1 < n_stage) issue(st + 1, 1);
            reduce(st, 0);
            if (st + 1 < n_stage) {
                if (st + 2 < n_stage) issue(st + 2, 0);
                reduce(st + 1, 1);
            }
        }
    } else {
        const int nchunks = c / VEC;
        for (int st = 0; st < n_stage; ++st) {
            double dot[STAGE], na[STAGE], nb[STAGE];
#pragma unroll
            for (int u = 0; u < STAGE; ++u) { dot[u] = 0.0; na[u] = 0.0; nb[u] = 0.0; }
            for (int ch = sub; ch < nchunks; ch += LPT) {
                Chunk<T, VEC> ca[STAGE], cb[STAGE], cr[STAGE];
#pragma unroll
                for (int u = 0; u < STAGE; ++u) {
                    const int t = tok_of(st, u);
                    const int64_t base = (block_first + (t < block_tokens ? t : 0)) * c + ch * VEC;
                    ca[u].load(x_t + base); cb[u].load(v + base); cr[u].load(x_ref + base);
                }
#pragma unroll
                for (int u = 0; u < STAGE; ++u) accumulate(ca[u], cb[u], cr[u], dot[u], na[u], nb[u]);
            }
#pragma unroll
            for (int u = 0; u < STAGE; ++u) finish(tok_of(st, u), dot[u], na[u], nb[u]);
        }
    }
    __syncthreads();

    // one thread per token: score, decision, one bit
    int edited_count = 0;
    for (int t0 = 0; t0 < tok_per_block; t0 += kThreads) {
        const int t = t0 + threadIdx.x;
        bool edited = false;
        if (t < block_tokens) {
            const double denom = fmax(sqrt(s_sum[1][t]) * sqrt(s_sum[2][t]), 1e-8);
            const float s = static_cast<float>(s_sum[0][t] / denom);
            edited = !(s > eta);
            if (score) __builtin_nontemporal_store(s, score + block_first + t);
        }
        const unsigned long long word = __ballot(edited);
        edited_count += __popcll(word);
        if (lane == 0 && t0 + wave * 64 < block_tokens) bits[(block_first + t0) / 64 + wave] = word;
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

// The count's second destination.  With a ticket (a host waits for THIS call's count on a pinned host word without
// waiting for the stream) the ticket follows the count into the next word, behind a system-scope fence, so that a host
// that sees the ticket reads the count that belongs to it.
__device__ __forceinline__ void publish_count(int32_t* __restrict__ dst, int32_t total, int32_t ticket) {
    *dst = total;
    if (ticket) {
        __threadfence_system();
        *reinterpret_cast<volatile int32_t*>(dst + 1) = ticket;
    }
}

// Exclusive prefix sum of the per-block counts, in place, by one workgroup: thread t owns a contiguous run of
// entries.  Also writes the total.
constexpr int kScanThreads = 1024;
__global__ void __launch_bounds__(kScanThreads)
scan_counts_kernel(int32_t* __restrict__ counts, int n_blocks, int32_t* __restrict__ n_edited, int32_t* __restrict__ n_edited_pinned, int32_t ticket) {
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
    if (threadIdx.x == 0) { *n_edited = total; publish_count(n_edited_pinned, total, ticket); }
}

// SUMS = false: `offsets` holds the exclusive prefix sums of the per-block counts (scan_counts_kernel ran).
// SUMS = true (few blocks): `offsets` holds the raw counts; every block adds up the counts of the blocks before it
// itself, and the last block writes the total, which saves the scan kernel's launch.
// BITS = true: the decisions come as one bit per token (`bits`, written by score_bits_kernel) and the byte mask is
// written here; BITS = false: they are read from the byte mask.  tok_per_block is a multiple of 64.
template <bool SUMS, bool BITS>
__global__ void __launch_bounds__(kThreads)
write_index_kernel(const uint64_t* __restrict__ bits, uint8_t* __restrict__ mask, const int32_t* __restrict__ offsets,
                   int64_t n_tokens, int tok_per_block,
                   int32_t* __restrict__ e_index, int32_t* __restrict__ u_index,
                   int32_t* __restrict__ n_edited, int32_t* __restrict__ n_edited_pinned, int32_t ticket) {
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
            publish_count(n_edited_pinned, total, ticket);
        }
    } else {
        base_e = offsets[blockIdx.x];   // edited tokens in all blocks before this one
    }
    // The block's decisions as words of 64 tokens (read, or formed by ballot from the byte mask); their popcounts give
    // every word its rank offset, after which the waves write their words' tokens without meeting again.
    constexpr int kMaxWords = kMaxBlockTokens / 64;
    __shared__ unsigned long long s_words[kMaxWords];
    __shared__ int s_before[kMaxWords];
    const int64_t block_first = static_cast<int64_t>(blockIdx.x) * tok_per_block;
    int64_t left = n_tokens - block_first;
    const int block_tokens = static_cast<int>(left < tok_per_block ? left : tok_per_block);
    const int n_words = (block_tokens + 63) / 64;
    __syncthreads();   // wave_e has been read by every wave
    for (int w = wave; w < n_words; w += kWaves) {
        unsigned long long word;
        if (BITS) {
            word = bits[block_first / 64 + w];      // bits of tokens past the end are clear
        } else {
            const int64_t tok = block_first + 64 * w + lane;
            word = __ballot(tok < n_tokens && mask[tok] != 0);
        }
        if (lane == 0) s_words[w] = word;
    }
    __syncthreads();
    if (wave == 0) {
        const int cnt = lane < n_words ? __popcll(s_words[lane]) : 0;
        int incl = cnt;
#pragma unroll
        for (int d = 1; d < kMaxWords; d <<= 1) {
            const int up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        if (lane < n_words) s_before[lane] = incl - cnt;
    }
    __syncthreads();
    for (int w = wave; w < n_words; w += kWaves) {
        const unsigned long long word = s_words[w];
        const int64_t tok = block_first + 64 * w + lane;
        const bool live = tok < n_tokens;
        const bool ed = (word >> lane) & 1ull;
        const int rank = __popcll(word & ((1ull << lane) - 1ull));
        const int64_t e_at = static_cast<int64_t>(base_e) + s_before[w];          // edited tokens before this word
        const int64_t u_at = block_first + 64 * w - e_at;                          // unedited tokens before it
        if (live) {
            if (BITS) mask[tok] = ed ? 1 : 0;
            if (ed) e_index[e_at + rank] = static_cast<int32_t>(tok);
            else u_index[u_at + (lane - rank)] = static_cast<int32_t>(tok);
        }
    }
}

__global__ void set_i32_kernel(int32_t* p, int32_t* p_pinned, int32_t v, int32_t ticket) { *p = v; publish_count(p_pinned, v, ticket); }

// Scratch memory of the partition's kernels: per-block edited counts and one decision bit per token.
struct PartScratch {
    int32_t* counts; int64_t counts_cap;      // one entry per block of >= 64 tokens
    uint64_t* bits; int64_t words_cap;        // one word per 64 tokens
};
// Layout inside one int32 array that serves `max_tokens` tokens: counts, then the bit words (8-byte aligned).
__host__ inline int64_t part_scratch_counts(int64_t max_tokens) { return ((max_tokens + 63) / 64 + 8 + 1) & ~int64_t{1}; }
__host__ inline int64_t part_scratch_words(int64_t max_tokens) { return (max_tokens + 63) / 64 + 8; }
__host__ inline PartScratch part_scratch_in(int32_t* base, int64_t max_tokens) {
    PartScratch ps;
    ps.counts = base; ps.counts_cap = part_scratch_counts(max_tokens);
    ps.bits = reinterpret_cast<uint64_t*>(base + ps.counts_cap); ps.words_cap = part_scratch_words(max_tokens);
    return ps;
}

template <typename T, int VEC>
int launch_score(hipStream_t stream, const PartScratch& ps, int lpt, bool pipe, dim3 grid, const void* x_t, const void* v, const void* x_ref, int64_t n, int c,
                 int tpb, float sigma, float eta, float* score) {
    const T* a = static_cast<const T*>(x_t); const T* b = static_cast<const T*>(v); const T* r = static_cast<const T*>(x_ref);
#define RG_CASE(L) case L: \
        if (VEC > 1 && pipe) hipLaunchKernelGGL((score_bits_kernel<T, VEC, L, (VEC > 1)>), grid, dim3(kThreads), 0, stream, a, b, r, n, c, tpb, sigma, eta, score, ps.bits, ps.counts); \
        else hipLaunchKernelGGL((score_bits_kernel<T, VEC, L, false>), grid, dim3(kThreads), 0, stream, a, b, r, n, c, tpb, sigma, eta, score, ps.bits, ps.counts); \
        break;
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

// Index lists from the per-block counts in `counts` and the decisions (bits when given, else the byte mask): few blocks ->
// one launch, else scan + lists.  n_edited_copy: a second place for the count (the context's pinned host word;
// n_edited_dev itself when there is none).
int launch_index_lists(hipStream_t stream, int32_t* counts, const uint64_t* bits, dim3 grid, uint8_t* mask, int64_t n_tokens, int tpb,
                       int32_t* e_index, int32_t* u_index, int32_t* n_edited_dev, int32_t* n_edited_copy, int32_t ticket = 0) {
    const bool sums = grid.x <= 1024;
    if (!sums) {
        hipLaunchKernelGGL(scan_counts_kernel, dim3(1), dim3(kScanThreads), 0, stream, counts, static_cast<int>(grid.x), n_edited_dev, n_edited_copy, ticket);
        RG_LAUNCH_CHECK();
    }
#define RG_IDX(S, B) hipLaunchKernelGGL((write_index_kernel<S, B>), grid, dim3(kThreads), 0, stream, bits, mask, counts, n_tokens, tpb, e_index, u_index, n_edited_dev, n_edited_copy, sums ? ticket : 0)
    if (sums) { if (bits) RG_IDX(true, true); else RG_IDX(true, false); }
    else { if (bits) RG_IDX(false, true); else RG_IDX(false, false); }
#undef RG_IDX
    RG_LAUNCH_CHECK();
    return REGIONE_OK;
}

// The launches of the partition on `stream` with its scratch memory in `ps`.
int partition_launches(hipStream_t stream, const PartScratch& ps, const void* x_t, const void* v, const void* x_ref,
                       int64_t n_tokens, int32_t c, int32_t dtype, float sigma_t, float eta, float* score_opt, uint8_t* mask,
                       int32_t* e_index, int32_t* u_index, int32_t* n_edited_dev, int32_t* n_edited_copy, int32_t ticket = 0) {
    if (n_tokens == 0) {
        hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(1), 0, stream, n_edited_dev, n_edited_copy, 0, ticket);
        RG_LAUNCH_CHECK();
        return REGIONE_OK;
    }
    const int full_vec = dtype == REGIONE_BF16 ? 8 : 4;
    const int vec = (c % full_vec == 0) ? full_vec : 1;
    const int nchunks = c / vec;
    int lpt = 1;
    while (lpt * 2 <= nchunks && lpt < 64) lpt *= 2;
    const bool pipe = vec > 1 && nchunks == lpt;     // one chunk per lane: the pipelined form
    // small inputs: 64 tokens per block so that one image still spreads over many CUs
    int tpb = 64;
    while (tpb < kMaxBlockTokens && n_tokens / (static_cast<int64_t>(tpb) * 2) >= 2048) tpb *= 2;
    const int64_t nblocks = (n_tokens + tpb - 1) / tpb;
    if (nblocks > ps.counts_cap || (n_tokens + 63) / 64 > ps.words_cap)
        RG_FAIL(REGIONE_ERR_WORKSPACE, "partition: %lld tokens in %lld blocks exceed the workspace", (long long)n_tokens, (long long)nblocks);
    dim3 grid(static_cast<unsigned>(nblocks));
    int rc;
    if (dtype == REGIONE_BF16) {
        rc = vec == 8 ? launch_score<bf16_t, 8>(stream, ps, lpt, pipe, grid, x_t, v, x_ref, n_tokens, c, tpb, sigma_t, eta, score_opt)
                      : launch_score<bf16_t, 1>(stream, ps, lpt, pipe, grid, x_t, v, x_ref, n_tokens, c, tpb, sigma_t, eta, score_opt);
    } else {
        rc = vec == 4 ? launch_score<float, 4>(stream, ps, lpt, pipe, grid, x_t, v, x_ref, n_tokens, c, tpb, sigma_t, eta, score_opt)
                      : launch_score<float, 1>(stream, ps, lpt, pipe, grid, x_t, v, x_ref, n_tokens, c, tpb, sigma_t, eta, score_opt);
    }
    if (rc != REGIONE_OK) return rc;
    return launch_index_lists(stream, ps.counts, ps.bits, grid, mask, n_tokens, tpb, e_index, u_index, n_edited_dev, n_edited_copy, ticket);
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
    if (int rc = partition_launches(ctx->stream, part_scratch_in(ctx->part_counts, ctx->dims.max_tokens), x_t, v, x_ref, n_tokens, c, dtype, sigma_t, eta,
                                    score_opt, mask, e_index, u_index, n_edited_dev, ctx->n_edited_pinned_dev)) return rc;
    }
    if (n_edited_host_opt) {   // the kernels wrote the count to pinned host memory too: no copy to wait for, only the stream
        RG_HIP(hipStreamSynchronize(ctx->stream));
        *n_edited_host_opt = *static_cast<volatile int32_t*>(ctx->n_edited_pinned);
    }
    return REGIONE_OK;
}

// regione_partition for a caller inside the library that goes on launching on the same stream: the host gets the count
// as soon as the kernels have published it (a ticketed pinned host word, polled), not when the stream has drained, so
// the launches that need the count are queued while the index kernel still writes its lists.
int rg_partition_early_count(regione_ctx* ctx, const void* x_t, const void* v, const void* x_ref,
                             int64_t n_tokens, int32_t c, int32_t dtype, float sigma_t, float eta,
                             float* score_opt, uint8_t* mask, int32_t* e_index, int32_t* u_index,
                             int32_t* n_edited_dev, int32_t* n_edited_host) {
    if (!ctx || !n_edited_host) RG_FAIL(REGIONE_ERR_INVALID_ARG, "partition: null context or count");
    if (int rc = check_partition_args("partition", x_t, v, x_ref, n_tokens, c, dtype, mask, e_index, u_index, n_edited_dev)) return rc;
    if (n_tokens > ctx->dims.max_tokens) RG_FAIL(REGIONE_ERR_WORKSPACE, "partition: %lld tokens, context made for %d", (long long)n_tokens, ctx->dims.max_tokens);
    ctx->count_ticket = ctx->count_ticket == INT32_MAX ? 1 : ctx->count_ticket + 1;
    const int32_t ticket = ctx->count_ticket;
    {
    ProfScope prof(ctx, REGIONE_PROF_PARTITION);
    if (int rc = partition_launches(ctx->stream, part_scratch_in(ctx->part_counts, ctx->dims.max_tokens), x_t, v, x_ref, n_tokens, c, dtype, sigma_t, eta,
                                    score_opt, mask, e_index, u_index, n_edited_dev, ctx->n_edited_pinned_dev, ticket)) return rc;
    }
    volatile int32_t* word = ctx->n_edited_pinned;
    const auto t0 = std::chrono::steady_clock::now();
    for (;;) {
        if (word[1] == ticket) break;
        // bounded: a launch that failed on the device never publishes; after 5 ms the stream decides
        if (std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(5)) {
            RG_HIP(hipStreamSynchronize(ctx->stream));
            if (word[1] != ticket) RG_FAIL(REGIONE_ERR_HIP, "partition: the count was not published");
            break;
        }
    }
    std::atomic_thread_fence(std::memory_order_acquire);
    *n_edited_host = word[0];
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
        hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(1), 0, ctx->stream, n_edited_dev, ctx->n_edited_pinned_dev, 0, 0);
        RG_LAUNCH_CHECK();
    } else {
        if (!mask_in || !mask_out || !e_index || !u_index) RG_FAIL(REGIONE_ERR_INVALID_ARG, "mask_cleanup: null tensor");
        const int tpb = kThreads;
        const int64_t nblocks = (n_tokens + tpb - 1) / tpb;
        if (nblocks > part_scratch_counts(ctx->dims.max_tokens)) RG_FAIL(REGIONE_ERR_WORKSPACE, "mask_cleanup: %lld blocks exceed the workspace", (long long)nblocks);
        hipLaunchKernelGGL(morph_open_close_kernel, dim3(static_cast<unsigned>(n_images)), dim3(kMorphThreads), 0, ctx->stream, mask_in, mask_out, grid_h, grid_w);
        RG_LAUNCH_CHECK();
        const dim3 grid(static_cast<unsigned>(nblocks));
        hipLaunchKernelGGL(count_mask_kernel, grid, dim3(kThreads), 0, ctx->stream, mask_out, n_tokens, tpb, ctx->part_counts);
        RG_LAUNCH_CHECK();
        if (int rc2 = launch_index_lists(ctx->stream, ctx->part_counts, nullptr, grid, mask_out, n_tokens, tpb, e_index, u_index, n_edited_dev, ctx->n_edited_pinned_dev)) return rc2;
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
#define RG_STATIC_MAX_TOKENS (1 << 22)
/* int32 entries: per-block counts (one per 64 tokens) and one decision bit per token, with the padding of
   part_scratch_in: 768 KiB per GPU, held until the process ends */
#define RG_STATIC_INTS ((RG_STATIC_MAX_TOKENS / 64 + 16) + 2 * (RG_STATIC_MAX_TOKENS / 64 + 8))
static __device__ __align__(256) int32_t scratch[RG_STATIC_INTS];

namespace {

constexpr int64_t kStaticMaxTokens = RG_STATIC_MAX_TOKENS;
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

int64_t rg_partition_scratch_ints(int64_t max_tokens) { return part_scratch_counts(max_tokens) + 2 * part_scratch_words(max_tokens); }

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
    // Nothing in the array has to start at zero: the score kernel writes the count of every block and the bit word of
    // every 64 tokens of this call before the index kernels read them, and nothing past them is ever read.
    const PartScratch ps = part_scratch_in(counts, kStaticMaxTokens);
    if (ps.counts_cap + 2 * ps.words_cap > RG_STATIC_INTS) RG_FAIL(REGIONE_ERR_WORKSPACE, "partition_static: the static array is smaller than its layout");
    return partition_launches(static_cast<hipStream_t>(hip_stream), ps, x_t, v, x_ref, n_tokens, c, dtype, sigma_t, eta,
                              score_opt, mask, e_index, u_index, n_edited_dev, n_edited_dev);
}
