"""CPU oracle for one region-aware denoising step of RegionE.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the HIP path
must compute.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may
import it; the product (`paper_2510_25590_amd`) never does, and this file imports nothing
from the product.  Every function is written from the paper's equations with numpy in
float64 (inputs are the bf16- or fp32-stored values widened exactly), with no blocking,
fusion or reordering, so it can be checked against the paper by eye.

Citations are to the paper (arXiv 2510.25590): Eq.4 Euler sampler, Eq.5 one-step
estimate, Eq.6 attention with the Region-Instruction KV cache, Eq.7-9 adaptive velocity
decay cache, Algorithm 1 (appendix "Pseudocode of RegionE"), appendix Eq.13 (residual
cache as a decayed velocity cache).

Parity pins (tests/test_oracle_*.py): closed forms (Eq.2+Eq.5 recover X_0, appendix Eq.13
with gamma = 1), hand cases, brute force on tiny inputs, torch CPU library routines
(cosine_similarity, scaled_dot_product_attention, layer_norm, gelu; scipy.ndimage's binary
erosion and dilation for the mask clean-up; rms_norm and silu for the block extras and the
conditioning path; numpy's lstsq for the fit of Eq.7's factor) and the structural identities of
Eq.6.  Unpinned: none of the functions below; what stays unpinned is the
fidelity of the method on real model weights (PSNR/SSIM figures), which needs the models.

The transformer block is NOT described by the paper (it treats the DiT as a black box
Phi); the block here is this build's minimal MMDiT block: LayerNorm without affine
(eps 1e-6) -> optional modulation -> QKV linear -> attention -> gated residual ->
LayerNorm -> MLP with tanh-GELU -> gated residual.  Linear weights are [out, in].
Optional extras of real editing models, equally outside the paper (pinned by their
mathematics in tests/test_oracle_rope_norm.py): RMS normalisation of queries and keys
over the head dimension, and rotary position embedding whose angles belong to a token's
position in the FULL sequence, so a gathered token keeps its own; and the per-step
conditioning path that yields a block's modulation vectors (sinusoidal embedding of the
time, vector-times-matrix layers with SiLU), pinned in tests/test_oracle_modulation.py.
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64

# --------------------------------------------------------------------------- Eq.5 / ARP


def one_step_estimate_f32(x_t: np.ndarray, v: np.ndarray, dt: float) -> np.ndarray:
    """Eq.5: x_hat = x_t - v * dt, evaluated in float32 with a separately rounded product
    and difference (the precision in which the partition takes its decision)."""
    x = np.asarray(x_t, dtype=np.float32)
    vv = np.asarray(v, dtype=np.float32)
    prod = (np.float32(dt) * vv).astype(np.float32)
    return (x - prod).astype(np.float32)


def cosine_scores(a: np.ndarray, b: np.ndarray, eps: float = 1e-8) -> np.ndarray:
    """Per-token cosine similarity over the channel axis (Methodology, "Adaptive Region
    Partition"): s_n = <a_n, b_n> / max(|a_n| |b_n|, eps).  float64 sums; the score is
    rounded once to float32, the type in which it is compared and returned."""
    a = np.asarray(a, dtype=F64)
    b = np.asarray(b, dtype=F64)
    dot = np.zeros(a.shape[0], dtype=F64)
    na = np.zeros(a.shape[0], dtype=F64)
    nb = np.zeros(a.shape[0], dtype=F64)
    for c in range(a.shape[1]):  # plain left-to-right channel sum
        dot += a[:, c] * b[:, c]
        na += a[:, c] * a[:, c]
        nb += b[:, c] * b[:, c]
    denom = np.maximum(np.sqrt(na) * np.sqrt(nb), eps)
    return (dot / denom).astype(np.float32)


def threshold_mask(score: np.ndarray, eta: float) -> np.ndarray:
    """Unedited iff score > eta (strict); everything else, NaN included, is edited.
    Returns uint8 with 1 = edited."""
    unedited = np.asarray(score, dtype=np.float32) > np.float32(eta)
    return (~unedited).astype(np.uint8)


def compact(mask: np.ndarray):
    """Index lists of Algorithm 1 (E_index, U_index): ascending raster order."""
    e = [n for n in range(mask.shape[0]) if mask[n]]
    u = [n for n in range(mask.shape[0]) if not mask[n]]
    return np.asarray(e, dtype=np.int32), np.asarray(u, dtype=np.int32)


def partition(x_t, v, x_ref, sigma_t: float, eta: float):
    """Adaptive region partition without the morphological clean-up: Eq.5 with t_f = 0,
    cosine score against the reference latent, threshold, index lists."""
    xhat0 = one_step_estimate_f32(x_t, v, sigma_t)
    score = cosine_scores(xhat0, x_ref)
    mask = threshold_mask(score, eta)
    e_index, u_index = compact(mask)
    return score, mask, e_index, u_index


# --------------------------------------------------------------------------- morphological clean-up of the partition


def erode3x3(m: np.ndarray) -> np.ndarray:
    """Binary erosion of a 2-D boolean array with the 3x3 square: a cell stays set iff every
    neighbour INSIDE the grid (itself included) is set.  Cells outside the grid never decide."""
    h, w = m.shape
    out = np.zeros((h, w), dtype=bool)
    for r in range(h):
        for c in range(w):
            ok = True
            for dr in (-1, 0, 1):
                for dc in (-1, 0, 1):
                    rr, cc = r + dr, c + dc
                    if 0 <= rr < h and 0 <= cc < w and not m[rr, cc]:
                        ok = False
            out[r, c] = ok
    return out


def dilate3x3(m: np.ndarray) -> np.ndarray:
    """Binary dilation with the 3x3 square: a cell is set iff some neighbour inside the grid is set."""
    h, w = m.shape
    out = np.zeros((h, w), dtype=bool)
    for r in range(h):
        for c in range(w):
            hit = False
            for dr in (-1, 0, 1):
                for dc in (-1, 0, 1):
                    rr, cc = r + dr, c + dc
                    if 0 <= rr < h and 0 <= cc < w and m[rr, cc]:
                        hit = True
            out[r, c] = hit
    return out


def mask_cleanup(edited_mask: np.ndarray, grid_h: int, grid_w: int) -> np.ndarray:
    """Morphological opening, then closing, of the region partition (section "Adaptive Region
    Partition"; Algorithm 1 applies erosion and dilation to the map cos > eta, i.e. to the
    UNEDITED region).  Opening = erosion then dilation: unedited specks smaller than the 3x3
    element become edited.  Closing = dilation then erosion: edited holes smaller than the
    element become unedited.  Readings (the paper names neither element nor border): 3x3 square,
    cells outside the token grid never decide.  edited_mask: flat uint8/bool [grid_h*grid_w],
    1 = edited; returns the cleaned flat uint8 mask."""
    unedited = ~np.asarray(edited_mask, dtype=bool).reshape(grid_h, grid_w)
    opened = dilate3x3(erode3x3(unedited))
    closed = erode3x3(dilate3x3(opened))
    return (~closed).reshape(-1).astype(np.uint8)


# --------------------------------------------------------------------------- gather / scatter


def gather(src: np.ndarray, index: np.ndarray) -> np.ndarray:
    """X[E_index] of Algorithm 1: literal row copy."""
    out = np.empty((len(index),) + src.shape[1:], dtype=src.dtype)
    for i, n in enumerate(index):
        out[i] = src[n]
    return out


def scatter(dst_full: np.ndarray, index: np.ndarray, src: np.ndarray) -> np.ndarray:
    """Re-gather by spatial position (Algorithm 1, merge line): rows listed in `index`
    are overwritten, every other row is left as it is.  In place."""
    for i, n in enumerate(index):
        dst_full[n] = src[i]
    return dst_full


# --------------------------------------------------------------------------- block pieces


def layer_norm(h: np.ndarray, eps: float = 1e-6) -> np.ndarray:
    h = np.asarray(h, dtype=F64)
    mean = h.mean(axis=-1, keepdims=True)
    var = ((h - mean) ** 2).mean(axis=-1, keepdims=True)  # biased
    return (h - mean) / np.sqrt(var + eps)


def modulate(u: np.ndarray, shift, scale) -> np.ndarray:
    if shift is None and scale is None:
        return u
    sh = 0.0 if shift is None else np.asarray(shift, dtype=F64)
    sc = 0.0 if scale is None else np.asarray(scale, dtype=F64)
    return u * (1.0 + sc) + sh


def gelu_tanh(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=F64)
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def linear(x: np.ndarray, w: np.ndarray, b=None) -> np.ndarray:
    """y = x W^T + b with W stored [out_features, in_features]."""
    y = np.asarray(x, dtype=F64) @ np.asarray(w, dtype=F64).T
    if b is not None:
        y = y + np.asarray(b, dtype=F64)
    return y


def rms_norm(x: np.ndarray, weight=None, eps: float = 1e-6) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) over the last axis, times an optional per-element weight."""
    x = np.asarray(x, dtype=F64)
    y = x / np.sqrt((x ** 2).mean(axis=-1, keepdims=True) + eps)
    if weight is not None:
        y = y * np.asarray(weight, dtype=F64)
    return y


def rope_angles(pos_ids: np.ndarray, axes_dims, theta: float = 10000.0) -> np.ndarray:
    """Rotation angles of every token: pos_ids [n, n_axes] (integers or floats), axes_dims
    the even number of head-dimension elements given to each axis (their sum is the head
    dimension).  Pair j of an axis of dimension a turns by pos * theta^(-2j/a); the axes'
    pairs follow each other.  Returns [n, head_dim/2]."""
    pos = np.asarray(pos_ids, dtype=F64)
    out = []
    for ax, a in enumerate(axes_dims):
        if a % 2:
            raise ValueError("an axis owns whole pairs")
        j = np.arange(a // 2, dtype=F64)
        freq = theta ** (-2.0 * j / a)
        out.append(pos[:, ax:ax + 1] * freq[None, :])
    return np.concatenate(out, axis=1)


def rope_apply(x: np.ndarray, angles: np.ndarray) -> np.ndarray:
    """x [n, heads, d]; pair (x[2j], x[2j+1]) of every head is turned by angles[n, j]:
    (a, b) -> (a cos - b sin, a sin + b cos)."""
    x = np.asarray(x, dtype=F64)
    ang = np.asarray(angles, dtype=F64)
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., 0::2], x[..., 1::2]
    y = np.empty_like(x)
    y[..., 0::2] = a * c - b * s
    y[..., 1::2] = a * s + b * c
    return y


def silu(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=F64)
    return x / (1.0 + np.exp(-x))


def vec_linear(x, w, b=None, pre_act: str = "none") -> np.ndarray:
    """y = W act(x) + b for ONE vector x [k], W [n, k]: the shape of a block's modulation
    (shift, scale, gate vectors) computed from a conditioning embedding, act = SiLU there."""
    x = np.asarray(x, dtype=F64)
    if pre_act == "silu":
        x = silu(x)
    elif pre_act != "none":
        raise ValueError(pre_act)
    y = np.asarray(w, dtype=F64) @ x
    if b is not None:
        y = y + np.asarray(b, dtype=F64)
    return y


def timestep_embedding(t: float, dim: int, max_period: float = 10000.0) -> np.ndarray:
    """Sinusoidal embedding of a scalar: [cos(t f_j) for j < dim/2] then [sin(t f_j)],
    f_j = max_period^(-j / (dim/2))."""
    if dim % 2:
        raise ValueError("dim must be even")
    half = dim // 2
    f = max_period ** (-np.arange(half, dtype=F64) / half)
    return np.concatenate([np.cos(t * f), np.sin(t * f)])


def attention_kvcache(q, k_fresh, v_fresh, k_cache=None, v_cache=None, cache_index=None, scale=None):
    """Eq.6.  q, k_fresh, v_fresh: [n_q, heads, d]; caches: [n_c, heads, d].
    Keys/values = the fresh rows followed by the cache rows in use (`cache_index`, or all
    of them when it is None).  Plain softmax per head and query row, no mask."""
    q = np.asarray(q, dtype=F64)
    keys = [np.asarray(k_fresh, dtype=F64)]
    vals = [np.asarray(v_fresh, dtype=F64)]
    if k_cache is not None and len(k_cache) > 0:
        kc = np.asarray(k_cache, dtype=F64)
        vc = np.asarray(v_cache, dtype=F64)
        if cache_index is not None:
            kc = kc[np.asarray(cache_index, dtype=np.int64)]
            vc = vc[np.asarray(cache_index, dtype=np.int64)]
        keys.append(kc)
        vals.append(vc)
    k = np.concatenate(keys, axis=0)
    v = np.concatenate(vals, axis=0)
    n_q, heads, d = q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.empty((n_q, heads, d), dtype=F64)
    for h in range(heads):
        logits = (q[:, h, :] @ k[:, h, :].T) * scale
        logits = logits - logits.max(axis=1, keepdims=True)
        p = np.exp(logits)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v[:, h, :]
    return out


FLAG_STORE = 1  # f[0] of Algorithm 1
FLAG_RETRIEVE = 2  # f[1] of Algorithm 1


def _rows_by_stream(n_rows: int, n_txt_rows: int, n_streams: int):
    if n_streams == 1:
        return [slice(0, n_rows)]
    return [slice(0, n_txt_rows), slice(n_txt_rows, n_rows)]


def block_forward(streams, kind: str, h, n_txt_rows: int, slot_index, k_cache, v_cache, flags: int, heads: int,
                  return_qkv: bool = False, rope=None):
    """One transformer block Phi-layer on the fresh rows `h` [n, H] (Algorithm 1's
    Phi(tokens, C_KV, f) for one layer).

    streams: [txt_weights, img_weights] for kind == "double" (rows [0, n_txt_rows) use the
    text set, the rest the image set; one joint attention), [weights] for "single".
    slot_index[i] = position of fresh row i in the cached sequence [P | X | I].
    flags: FLAG_STORE -> plain attention over the fresh rows, then their K,V are written
    to the cache rows slot_index (cache arrays are modified in place);
    FLAG_RETRIEVE -> Eq.6 with the cache rows that are not refreshed; 0 -> plain attention.
    Extras: a stream's "q_norm" / "k_norm" [d] switch on the RMS normalisation of its queries /
    keys; `rope` [n_all, d/2] holds the angles of every position of the cached sequence and
    fresh row i takes row slot_index[i] (row i when slot_index is None).  Keys enter the cache
    normalised and rotated.
    """
    if flags == (FLAG_STORE | FLAG_RETRIEVE):
        raise ValueError("store and retrieve together are not a mode of Algorithm 1")
    h = np.asarray(h, dtype=F64)
    n, hidden = h.shape
    d = hidden // heads
    groups = _rows_by_stream(n, n_txt_rows, len(streams))
    q = np.empty((n, hidden), dtype=F64)
    k = np.empty((n, hidden), dtype=F64)
    v = np.empty((n, hidden), dtype=F64)
    m_act = [None] * len(streams)
    for s, (w, rows) in enumerate(zip(streams, groups)):
        u = modulate(layer_norm(h[rows]), w.get("shift1"), w.get("scale1"))
        if kind == "double":
            qkv = linear(u, w["w_qkv"], w["b_qkv"])
        else:
            y = linear(u, w["w_1"], w["b_1"])
            qkv = y[:, :3 * hidden]
            m_act[s] = gelu_tanh(y[:, 3 * hidden:])
        q[rows], k[rows], v[rows] = qkv[:, :hidden], qkv[:, hidden:2 * hidden], qkv[:, 2 * hidden:]
    q3, k3, v3 = (x.reshape(n, heads, d) for x in (q, k, v))
    for w, rows in zip(streams, groups):
        if w.get("q_norm") is not None:
            q3[rows] = rms_norm(q3[rows], w["q_norm"])
        if w.get("k_norm") is not None:
            k3[rows] = rms_norm(k3[rows], w["k_norm"])
    if rope is not None:
        own = np.arange(n) if slot_index is None else np.asarray(slot_index, dtype=np.int64)
        ang = np.asarray(rope, dtype=F64)[own]
        q3, k3 = rope_apply(q3, ang), rope_apply(k3, ang)
    if flags == FLAG_RETRIEVE:
        n_all = k_cache.shape[0]
        fresh = np.zeros(n_all, dtype=bool)
        fresh[np.asarray(slot_index, dtype=np.int64)] = True
        cache_index = np.nonzero(~fresh)[0]
        a = attention_kvcache(q3, k3, v3, k_cache, v_cache, cache_index)
    else:
        a = attention_kvcache(q3, k3, v3)
    if flags == FLAG_STORE:
        for i, slot in enumerate(slot_index):
            k_cache[slot] = k3[i]
            v_cache[slot] = v3[i]
    a = a.reshape(n, hidden)
    out = np.empty((n, hidden), dtype=F64)
    for s, (w, rows) in enumerate(zip(streams, groups)):
        g1 = 1.0 if w.get("gate1") is None else np.asarray(w["gate1"], dtype=F64)
        if kind == "double":
            h1 = h[rows] + g1 * linear(a[rows], w["w_o"], w["b_o"])
            u2 = modulate(layer_norm(h1), w.get("shift2"), w.get("scale2"))
            g2 = 1.0 if w.get("gate2") is None else np.asarray(w["gate2"], dtype=F64)
            out[rows] = h1 + g2 * linear(gelu_tanh(linear(u2, w["w_1"], w["b_1"])), w["w_2"], w["b_2"])
        else:
            cat = np.concatenate([a[rows], m_act[s]], axis=1)
            out[rows] = h[rows] + g1 * linear(cat, w["w_2"], w["b_2"])
    if return_qkv:
        return out, q3, k3, v3
    return out


# --------------------------------------------------------------------------- Eq.4, Eq.7-9


def euler_step(x, v, dt: float):
    """Eq.4: X_{t_{i-1}} = X_{t_i} - (t_i - t_{i-1}) v."""
    return np.asarray(x, dtype=F64) - dt * np.asarray(v, dtype=F64)


def decay_factor(t, gamma, j: int) -> float:
    """Eq.7: |v_{t_j}| / |v_{t_{j+1}}| = (1 - (t_{j+1} - t_j)) * gamma_j, with t indexed so
    that t[T] = 1 and t[0] = 0."""
    return (1.0 - (float(t[j + 1]) - float(t[j]))) * float(gamma[j])


def guidance_combine(v_cond, v_uncond, scale: float) -> np.ndarray:
    """Classifier-free guidance, which the paper's experiments keep on ("Experimental Settings"):
    the velocity used by the sampler is v_uncond + scale * (v_cond - v_uncond)."""
    v_c = np.asarray(v_cond, dtype=F64)
    v_u = np.asarray(v_uncond, dtype=F64)
    return v_u + scale * (v_c - v_u)


def fit_gamma(norms: np.ndarray, t) -> np.ndarray:
    """Timestep-aware factor of Eq.7 from sampled trajectories (the paper says only that the factor is
    fitted on sampled data, not how: here least squares through the origin).
    norms[s, j] = |v_{t_j}| of sample s for j = 1..T (column 0 is not used); t has T+1 entries.
    For j = 1..T-1 the slope c_j of |v_{t_j}| against |v_{t_{j+1}}| over the samples is
    sum_s a_s b_s / sum_s b_s^2, and gamma_j = c_j / (1 - (t_{j+1} - t_j)).  gamma_0 = gamma_T = 1
    (no ratio exists there)."""
    norms = np.asarray(norms, dtype=F64)
    T = norms.shape[1] - 1
    gamma = np.ones(T + 1, dtype=F64)
    for j in range(1, T):
        a, b = norms[:, j], norms[:, j + 1]
        gamma[j] = (a * b).sum() / (b * b).sum() / (1.0 - (float(t[j + 1]) - float(t[j])))
    return gamma


class AvdState:
    """State of the adaptive velocity decay cache: whether C_A holds a velocity, and the
    product of Eq.7 factors accumulated since it was computed."""

    def __init__(self):
        self.valid = False
        self.prod = 1.0


def avd_decision(t, gamma, delta: float, j: int, st: AvdState):
    """Eq.8 / Eq.9 at timestep index j.  Returns (reuse, factor): reuse False means the DiT
    runs and its velocity becomes the new cache; True means v = C_A * factor.  The product
    runs over the steps after the cached one up to and including j (the reading under which
    gamma = 1 gives appendix Eq.13)."""
    prod = st.prod * decay_factor(t, gamma, j)
    criterion = 1.0 - prod
    if (not st.valid) or criterion > delta:
        st.valid = True
        st.prod = 1.0
        return False, 1.0
    st.prod = prod
    return True, prod


def velocity_cache_apply(reuse: bool, factor: float, dt: float, v_fresh, c_a, x_e):
    """Eq.9 then Eq.4 on the edited rows.  Returns (v_used, c_a_new, x_e_new)."""
    if reuse:
        v_used = np.asarray(c_a, dtype=F64) * factor
        c_new = np.asarray(c_a, dtype=F64)
    else:
        v_used = np.asarray(v_fresh, dtype=F64)
        c_new = v_used.copy()
    return v_used, c_new, euler_step(x_e, v_used, dt)


# --------------------------------------------------------------------------- Algorithm 1


def relative_change(v_new, v_old) -> float:
    """|v_new - v_old|_2 / |v_old|_2 over all elements: the data-dependent reuse trigger that the
    loop benchmark's workload description asks for ("reusing v with decay 0.9 when relative
    velocity change < 0.05").  NOT part of the paper, whose criterion (Eq.8) depends on the
    schedule alone."""
    a = np.asarray(v_new, dtype=F64)
    b = np.asarray(v_old, dtype=F64)
    den = float(np.sqrt((b ** 2).sum()))
    return float(np.sqrt(((a - b) ** 2).sum())) / den if den > 0.0 else math.inf


def stage_plan(T: int, t_st: int, t_sm: int, forced_k):
    """Control flow of Algorithm 1 as a list of (i, kind) for timestep indices i = T..1
    (the step at index i moves X_{t_i} to X_{t_{i-1}}), kind in {"full", "full_store",
    "region"}, plus the segment list.  forced_k are 0-based forward step counters
    (k = T - i).  Readings: the stabilization stage is t_st steps and stores at its last;
    each segment [prev, next] runs region steps at i = prev..next+2 and one storing full
    step at i = next+1; the last segment's closing full step is the first smooth step and
    the remaining t_sm - 1 smooth steps are plain full steps."""
    forced_i = sorted((T - k for k in forced_k), reverse=True)
    tf_list = [T - t_st] + [i - 1 for i in forced_i] + [t_sm - 1]
    plan = []
    for i in range(T, T - t_st, -1):
        plan.append((i, "full_store" if i == T - t_st + 1 else "full"))
    segments = []
    for s in range(len(tf_list) - 1):
        prev, nxt = tf_list[s], tf_list[s + 1]
        segments.append((prev, nxt))
        for j in range(prev, nxt + 1, -1):
            plan.append((j, "region"))
        plan.append((nxt + 1, "full_store"))
    for i in range(t_sm - 1, 0, -1):
        plan.append((i, "full"))
    return plan, segments


def regione_loop(phi, x_T, x_ref, t, gamma, T, t_st, t_sm, forced_k, eta, delta, grid=None, rel_trigger=None,
                 forced_reuse=None):
    """Algorithm 1 on latents [N, C].  `phi(x_rows, row_index, i, mode)` returns the velocity
    for the rows given (mode "full", "full_store" or "region"; row_index None = all rows).
    Returns (x_0, log) where log lists (i, what) with what in {"full", "full_store",
    "region_fresh", "region_reuse"} and, once, ("partition", n_E).  grid = (rows, columns) of
    the token grid applies the morphological clean-up to the partition; None leaves it as thresholded.

    rel_trigger = (threshold, decay) replaces the paper's schedule criterion (Eq.8) by the
    data-dependent one of the loop benchmark's workload description (see relative_change): after a
    fresh region step whose velocity differs from the segment's previous fresh velocity by less than
    `threshold` (relative), the NEXT region step reuses decay * C_A; never two reuses in a row; a
    segment starts with two fresh steps.  The log then also holds ("rel", i, value) entries.
    forced_reuse: {i: bool} overrides the decision of step i (a flipped decision changes the whole
    trajectory, so parity runs force one side's decisions on the other)."""
    plan, segments = stage_plan(T, t_st, t_sm, forced_k)
    x = np.asarray(x_T, dtype=F64).copy()
    log = []
    v_last_full = None
    seg_start = {prev: nxt for prev, nxt in segments}
    e_index = u_index = None
    x_e = None
    st = AvdState()
    c_a = None
    pos = 0
    while pos < len(plan):
        i, kind = plan[pos]
        if kind in ("full", "full_store"):
            v = phi(x, None, i, kind)
            x = euler_step(x, v, t[i] - t[i - 1])
            v_last_full = v
            log.append((i, kind))
            pos += 1
            continue
        # first region step of a segment
        prev = i
        nxt = seg_start[prev]
        if e_index is None:
            _, mask, e_index, u_index = partition(x.astype(np.float32), v_last_full.astype(np.float32), x_ref, t[prev], eta)
            if grid is not None:
                e_index, u_index = compact(mask_cleanup(mask, grid[0], grid[1]))
            log.append(("partition", int(len(e_index))))
        x_e = gather(x, e_index)
        x_u = gather(x, u_index)
        v_u = gather(v_last_full, u_index)
        x_u = euler_step(x_u, v_u, t[prev] - t[nxt + 1])  # Eq.5: one jump for the unedited rows
        st = AvdState()
        c_a = None
        reuse_next = False
        for j in range(prev, nxt + 1, -1):
            if rel_trigger is None:
                reuse, factor = avd_decision(t, gamma, delta, j, st)
            else:
                reuse, factor = (reuse_next and c_a is not None), rel_trigger[1]
                if forced_reuse is not None and j in forced_reuse:
                    reuse = bool(forced_reuse[j]) and c_a is not None
                reuse_next = False
            v_fresh = None if reuse else phi(x_e, e_index, j, "region")
            if rel_trigger is not None and not reuse and c_a is not None:
                rel = relative_change(v_fresh, c_a)
                log.append(("rel", j, rel))
                reuse_next = rel < rel_trigger[0]
            _, c_a, x_e = velocity_cache_apply(reuse, factor if reuse else 1.0, t[j] - t[j - 1], v_fresh, c_a, x_e)
            log.append((j, "region_reuse" if reuse else "region_fresh"))
            pos += 1
        scatter(x, e_index, x_e)
        scatter(x, u_index, x_u)
    return x, log
