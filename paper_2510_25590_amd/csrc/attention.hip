// Attention with the Region-Instruction KV cache, Eq.6:
//   O = softmax(Q [K_fresh; K_cache]^T * scale) [V_fresh; V_cache]        (per head)
// Queries are the fresh (edited / text) rows only; the key list is the fresh rows followed by the
// cache rows in use, addressed as one virtual list so that a tile may straddle the two.
//
// Flash-style streaming with an online softmax.  A workgroup of 4 waves owns QB*128 query rows of
// one head; each wave owns QB blocks of 32 queries, whose Q fragments stay in registers.  Keys and
// values are staged 64 rows at a time in LDS (double buffered).  The scores are computed
// TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: a lane then holds, for ONE query
// (column lane%32), 16 of every 32 keys, so the running maximum and the rescaling factor are
// per-lane scalars, and the exponentiated scores are already in the register layout of the "B"
// operand of the second product O^T = V^T P^T.  The V^T "A" operand (8 consecutive keys per lane
// for one d) is read from the row-major V tile with ds_read_b64_tr_b16, the transposing LDS read
// of gfx950.  The k-slot of the second product pairs lane-half h, slot s of both operands, so the
// only requirement is that both sides enumerate keys identically: slot s of half h of MFMA (kb,j)
// is key kb*32 + 16*j + 8*(s/4) + 4*h + s%4, which is exactly the row order of the S^T accumulator.
#include "common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kThreads = 256;
constexpr int KT = 64;  // keys per tile

struct AttnArgs {
    const bf16_t* q; int ldq; int n_q;
    const bf16_t* k0; const bf16_t* v0; int ldkv0; int n0;       // fresh rows
    const bf16_t* k1; const bf16_t* v1; int ldkv1; int n1;       // cache rows
    const int32_t* idx1;                                        // optional row list into the cache
    int heads; float scale_log2e;
    bf16_t* out; int ldo;
    // split-KV
    int splits; int tiles_per_split; float* part;  // [splits][heads][n_q_pad][D + 2] when splits > 1
    int n_q_pad;
};

template <int D> struct Swz {
    static constexpr int CPR = D / 8;  // 16-byte chunks per row
    // K tile: spread the rows of one fragment read (same logical chunk, consecutive rows) over all banks
    __device__ static __forceinline__ int k(int row, int chunk) { return chunk ^ (row & (CPR - 1)); }
    // V tile: a transposing read touches 4 consecutive keys x 4 consecutive chunks per lane half
    __device__ static __forceinline__ int v(int row, int chunk) {
        return D == 128 ? (chunk ^ ((row & 3) << 2)) : (chunk ^ (((row >> 1) & 1) << 2));
    }
};

// Global -> register -> LDS staging of one 64-key tile.  Thread t owns 16-byte chunk t%CPR of rows t/CPR + i*(256/CPR).
template <int D>
__device__ __forceinline__ void kv_tile_load(const AttnArgs& a, int head, int key0, int n_keys,
                                             uint4 (&kr)[KT * (D / 8) / kThreads], uint4 (&vr)[KT * (D / 8) / kThreads]) {
    constexpr int CPR = D / 8;
    constexpr int PER_THREAD = KT * CPR / kThreads;
    const int r0 = threadIdx.x / CPR, c = threadIdx.x % CPR;
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
        int key = key0 + r0 + i * (kThreads / CPR);
        key = key < n_keys ? key : n_keys - 1;  // tail rows repeat a valid row; their scores are masked
        const bool fresh = key < a.n0;
        int64_t row = fresh ? key : key - a.n0;
        if (!fresh && a.idx1) row = a.idx1[row];
        const int64_t off = row * (fresh ? a.ldkv0 : a.ldkv1) + head * D + c * 8;
        const bf16_t* kb = fresh ? a.k0 : a.k1;
        const bf16_t* vb = fresh ? a.v0 : a.v1;
        kr[i] = *reinterpret_cast<const uint4*>(kb + off);
        vr[i] = *reinterpret_cast<const uint4*>(vb + off);
    }
}

template <int D>
__device__ __forceinline__ void kv_tile_store(bf16_t* k_lds, bf16_t* v_lds,
                                              const uint4 (&kr)[KT * (D / 8) / kThreads], const uint4 (&vr)[KT * (D / 8) / kThreads]) {
    constexpr int CPR = D / 8;
    constexpr int PER_THREAD = KT * CPR / kThreads;
    const int r0 = threadIdx.x / CPR, c = threadIdx.x % CPR;
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
        const int r = r0 + i * (kThreads / CPR);
        *reinterpret_cast<uint4*>(k_lds + r * D + (Swz<D>::k(r, c) << 3)) = kr[i];
        *reinterpret_cast<uint4*>(v_lds + r * D + (Swz<D>::v(r, c) << 3)) = vr[i];
    }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D, int QB>
__global__ void __launch_bounds__(kThreads)
attn_kvcache_kernel(AttnArgs a) {
    constexpr int DB = D / 32;   // 32-wide d blocks of the output
    constexpr int KK = D / 16;   // k-steps of the first product
    __shared__ __attribute__((aligned(16))) bf16_t k_lds[2][KT * D];
    __shared__ __attribute__((aligned(16))) bf16_t v_lds[2][KT * D];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int head = blockIdx.y;
    const int split = blockIdx.z;
    const int q_base = blockIdx.x * (QB * 128) + wave * (QB * 32);
    const int n_keys = a.n0 + a.n1;
    const int n_tiles = (n_keys + KT - 1) / KT;
    const int tile_begin = split * a.tiles_per_split;
    int tile_end = tile_begin + a.tiles_per_split;
    tile_end = tile_end < n_tiles ? tile_end : n_tiles;

    // Q fragments ("B" operand): lane holds query l32 of the block, d = kk*16 + 8*lh + 0..7
    bf16x8 qf[QB][KK];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int qrow = q_base + qb * 32 + l32;
        qrow = qrow < a.n_q ? qrow : a.n_q - 1;
        const bf16_t* qp = a.q + static_cast<int64_t>(qrow) * a.ldq + head * D + 8 * lh;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qf[qb][kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16);
    }

    f32x16 o[QB][DB];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[qb][db][r] = 0.f;
    }

    constexpr int LD_N = KT * (D / 8) / kThreads;
    uint4 kr[LD_N], vr[LD_N];
    if (tile_begin < tile_end) {
        kv_tile_load<D>(a, head, tile_begin * KT, n_keys, kr, vr);
        kv_tile_store<D>(k_lds[0], v_lds[0], kr, vr);
    }
    __syncthreads();

    for (int t = tile_begin; t < tile_end; ++t) {
        const int cur = (t - tile_begin) & 1;
        // the last iteration re-loads its own tile into the idle buffer: unconditional code keeps the staging registers in VGPRs
        kv_tile_load<D>(a, head, (t + 1 < tile_end ? t + 1 : t) * KT, n_keys, kr, vr);
        const bf16_t* kt = k_lds[cur];
        const bf16_t* vt = v_lds[cur];

        // ---- S^T = K Q^T for the two 32-key blocks of the tile
        f32x16 s[QB][2];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[qb][kb][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            bf16x8 kf[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const int row = kb * 32 + l32;
                kf[kb] = *reinterpret_cast<const bf16x8*>(kt + row * D + (Swz<D>::k(row, kk * 2 + lh) << 3));
            }
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
                    s[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb], qf[qb][kk], s[qb][kb], 0, 0, 0);
        }

        // ---- online softmax; accumulator r of block kb is key  t*64 + kb*32 + 8*(r/4) + 4*lh + r%4
        const bool tail = (t + 1) * KT > n_keys;
        bf16x8 pf[QB][2][2];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float mx = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float x = s[qb][kb][r] * a.scale_log2e;
                    if (tail) {
                        const int key = t * KT + kb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                        if (key >= n_keys) x = -INFINITY;
                    }
                    s[qb][kb][r] = x;
                    mx = fmaxf(mx, x);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run[qb], mx);   // finite: every tile holds at least one live key
            const float alpha = fast_exp2(m_run[qb] - m_new);
            m_run[qb] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float p = fast_exp2(s[qb][kb][8 * j + e] - m_new);
                        psum += p;
                        pf[qb][kb][j][e] = static_cast<__bf16>(p);
                    }
            l_run[qb] = l_run[qb] * alpha + psum;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[qb][db][r] *= alpha;
        }

        // ---- O^T += V^T P^T
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int key_base = kb * 32 + 16 * j + 4 * lh;      // slots 0..3: key_base + s ; slots 4..7: key_base + 8 + (s-4)
                const int src_key = key_base + ((lane & 15) >> 2);  // source row this lane addresses in the transposing read
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const int d_src = db * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);  // 4 consecutive d = 8 bytes
                    const int chunk = d_src >> 3, within = d_src & 7;
                    const bf16_t* p0 = vt + src_key * D + (Swz<D>::v(src_key, chunk) << 3) + within;
                    const bf16_t* p1 = vt + (src_key + 8) * D + (Swz<D>::v(src_key + 8, chunk) << 3) + within;
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p1));
                    const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qb][kb][j], o[qb][db], 0, 0, 0);
                }
            }

        kv_tile_store<D>(k_lds[cur ^ 1], v_lds[cur ^ 1], kr, vr);
        __syncthreads();
    }

    // ---- finish: O^T accumulator r of d-block db: d = db*32 + 8*(r/4) + 4*lh + r%4, query = l32
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int qrow = q_base + qb * 32 + l32;
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
        if (qrow >= a.n_q) continue;
        if (a.splits == 1) {
            const float inv = 1.0f / l_tot;
            bf16_t* op = a.out + static_cast<int64_t>(qrow) * a.ldo + head * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int d = db * 32 + 8 * g + 4 * lh;
                    bf16x4 pk;
#pragma unroll
                    for (int e = 0; e < 4; ++e) pk[e] = static_cast<__bf16>(o[qb][db][4 * g + e] * inv);
                    *reinterpret_cast<bf16x4*>(op + d) = pk;
                }
        } else {
            // partial result: unnormalised O, running max (log2 domain) and sum
            float* pp = a.part + ((static_cast<int64_t>(split) * a.heads + head) * a.n_q_pad + qrow) * (D + 2);
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int d = db * 32 + 8 * g + 4 * lh;
                    float4 f = make_float4(o[qb][db][4 * g], o[qb][db][4 * g + 1], o[qb][db][4 * g + 2], o[qb][db][4 * g + 3]);
                    *reinterpret_cast<float2*>(pp + d) = make_float2(f.x, f.y);
                    *reinterpret_cast<float2*>(pp + d + 2) = make_float2(f.z, f.w);
                }
            if (lh == 0) { pp[D] = m_run[qb]; pp[D + 1] = l_tot; }
        }
    }
}

// Merges the split-KV partial results: out = sum_s 2^(m_s - m) O_s / sum_s 2^(m_s - m) l_s.
template <int D>
__global__ void __launch_bounds__(kThreads)
attn_combine_kernel(const float* __restrict__ part, int splits, int heads, int n_q, int n_q_pad, bf16_t* __restrict__ out, int ldo) {
    // one thread per (query, head, 4 d's)
    constexpr int G = D / 4;
    const int64_t gid = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t total = static_cast<int64_t>(n_q) * heads * G;
    if (gid >= total) return;
    const int g = static_cast<int>(gid % G);
    const int head = static_cast<int>((gid / G) % heads);
    const int qrow = static_cast<int>(gid / (static_cast<int64_t>(G) * heads));
    float m = -INFINITY;
    for (int s = 0; s < splits; ++s) {
        const float* pp = part + ((static_cast<int64_t>(s) * heads + head) * n_q_pad + qrow) * (D + 2);
        if (pp[D + 1] > 0.f) m = fmaxf(m, pp[D]);
    }
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
    for (int s = 0; s < splits; ++s) {
        const float* pp = part + ((static_cast<int64_t>(s) * heads + head) * n_q_pad + qrow) * (D + 2);
        const float ls = pp[D + 1];
        if (!(ls > 0.f)) continue;  // a split that saw no key
        const float w = fast_exp2(pp[D] - m);
        l += w * ls;
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += w * pp[4 * g + e];
    }
    const float inv = 1.0f / l;
    bf16x4 pk;
#pragma unroll
    for (int e = 0; e < 4; ++e) pk[e] = static_cast<__bf16>(acc[e] * inv);
    *reinterpret_cast<bf16x4*>(out + static_cast<int64_t>(qrow) * ldo + head * D + 4 * g) = pk;
}

template <int D, int QB>
int launch_attention(regione_ctx* ctx, AttnArgs a) {
    const int q_tiles = (a.n_q + QB * 128 - 1) / (QB * 128);
    const int n_tiles = (a.n0 + a.n1 + KT - 1) / KT;
    // split the key range when the (query tile, head) grid would leave most CUs idle
    int splits = 1;
    const int wgs = q_tiles * a.heads;
    while (wgs * splits < 256 && splits * 2 <= n_tiles / 8 && splits < 16) splits *= 2;
    a.n_q_pad = a.n_q;
    if (splits > 1) {
        const size_t need = static_cast<size_t>(splits) * a.heads * a.n_q_pad * (D + 2) * sizeof(float);
        if (need > ctx->attn_part_bytes) splits = 1;
    }
    a.splits = splits;
    a.tiles_per_split = (n_tiles + splits - 1) / splits;
    a.part = ctx->attn_part;
    hipLaunchKernelGGL((attn_kvcache_kernel<D, QB>), dim3(q_tiles, a.heads, splits), dim3(kThreads), 0, ctx->stream, a);
    RG_LAUNCH_CHECK();
    if (splits > 1) {
        const int64_t total = static_cast<int64_t>(a.n_q) * a.heads * (D / 4);
        hipLaunchKernelGGL((attn_combine_kernel<D>), dim3(static_cast<unsigned>((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, ctx->stream,
                           a.part, splits, a.heads, a.n_q, a.n_q_pad, a.out, a.ldo);
        RG_LAUNCH_CHECK();
    }
    return REGIONE_OK;
}

}  // namespace

int rg_attention(regione_ctx* ctx, const bf16_t* q, int ldq, int n_q,
                 const bf16_t* k0, const bf16_t* v0, int ldkv0, int n0,
                 const bf16_t* k1, const bf16_t* v1, int ldkv1, int n1, const int32_t* idx1,
                 int heads, int d, float scale, bf16_t* out, int ldo) {
    if (n_q <= 0) return REGIONE_OK;
    if (n0 + n1 <= 0) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "attention: %d queries but no key", n_q);
    if (d != 64 && d != 128) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "attention: head dimension %d (64 or 128 supported)", d);
    if ((ldq & 7) || (ldo & 3) || (n0 > 0 && (ldkv0 & 7)) || (n1 > 0 && (ldkv1 & 7)))
        RG_FAIL(REGIONE_ERR_BAD_SHAPE, "attention: row strides must keep 16-byte alignment");
    ProfScope prof(ctx, REGIONE_PROF_ATTENTION);
    AttnArgs a = {};
    a.q = q; a.ldq = ldq; a.n_q = n_q;
    a.k0 = k0; a.v0 = v0; a.ldkv0 = ldkv0; a.n0 = n0;
    a.k1 = k1; a.v1 = v1; a.ldkv1 = ldkv1; a.n1 = n1; a.idx1 = idx1;
    a.heads = heads;
    a.scale_log2e = (scale > 0.f ? scale : 1.0f / sqrtf(static_cast<float>(d))) * 1.4426950408889634f;
    a.out = out; a.ldo = ldo;
    if (d == 128) return launch_attention<128, 1>(ctx, a);
    return launch_attention<64, 1>(ctx, a);
}

extern "C" int regione_attn_kvcache(regione_ctx* ctx, const void* q, int32_t n_q,
                                    const void* k_fresh, const void* v_fresh, int32_t n_fresh,
                                    const void* k_cache, const void* v_cache, int32_t n_c,
                                    const int32_t* cache_index_opt, int32_t n_cache_index,
                                    int32_t heads, int32_t d, float scale, void* out) {
    if (!ctx) RG_FAIL(REGIONE_ERR_INVALID_ARG, "attn_kvcache: null context");
    if (n_q < 0 || n_fresh < 0 || n_c < 0 || heads <= 0 || n_cache_index < 0)
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "attn_kvcache: n_q=%d n_fresh=%d n_c=%d heads=%d", n_q, n_fresh, n_c, heads);
    if (d != 64 && d != 128) RG_FAIL(REGIONE_ERR_UNSUPPORTED, "attn_kvcache: head dimension %d (64 or 128 supported)", d);
    if (n_q == 0) return REGIONE_OK;
    if (!q || !out) RG_FAIL(REGIONE_ERR_INVALID_ARG, "attn_kvcache: null q or out");
    if (n_fresh > 0 && (!k_fresh || !v_fresh)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "attn_kvcache: null fresh K/V");
    if (n_c > 0 && (!k_cache || !v_cache)) RG_FAIL(REGIONE_ERR_INVALID_ARG, "attn_kvcache: null cache");
    const int n1 = cache_index_opt ? n_cache_index : n_c;
    if (cache_index_opt && n_c == 0 && n_cache_index > 0) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "attn_kvcache: index list into an empty cache");
    if (n_fresh + n1 == 0) RG_FAIL(REGIONE_ERR_BAD_SHAPE, "attn_kvcache: %d queries but no key", n_q);
    if (!rg_aligned16(q) || !rg_aligned16(out) || !rg_aligned16(k_fresh) || !rg_aligned16(v_fresh) || !rg_aligned16(k_cache) || !rg_aligned16(v_cache))
        RG_FAIL(REGIONE_ERR_INVALID_ARG, "attn_kvcache: tensors must be 16-byte aligned");
    const int ld = heads * d;
    return rg_attention(ctx, static_cast<const bf16_t*>(q), ld, n_q,
                        static_cast<const bf16_t*>(k_fresh), static_cast<const bf16_t*>(v_fresh), ld, n_fresh,
                        static_cast<const bf16_t*>(k_cache), static_cast<const bf16_t*>(v_cache), ld, n1, cache_index_opt,
                        heads, d, scale, static_cast<bf16_t*>(out), ld);
}
