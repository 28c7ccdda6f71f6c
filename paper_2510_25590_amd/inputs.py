"""Seeded synthetic input generators shared by the tests, the benchmark and the smoke check.

This module holds none of the method's arithmetic: it only draws random numbers, builds
masks that say which tokens *should* come out edited, and rounds arrays to bfloat16.  Both
the CPU oracle and the HIP path are fed from here; neither of them is imported here.

Workloads follow the paper's setting (Preliminary, "Instruction-Based Editing Model"): a
sequence of text tokens, noisy image tokens and reference-image ("instruction") tokens,
with image and reference counts equal and much larger than the text count.  The paper's
benchmarks (GEdit-Bench, KontextBench) and model weights are not available, so seeded
random latents, hidden states and N(0, 0.02) weights of the same shapes stand in for them.
"""
from __future__ import annotations

import numpy as np

# ----------------------------------------------------------------------------- bf16 helpers


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 array of bfloat16 bit patterns (round to nearest even)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    with np.errstate(over="ignore"):
        r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)   # finite inputs never wrap; NaN payloads are not produced here
    return r.astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> float32 array (exact widening)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round a float array to the nearest bfloat16 value, returned as float32."""
    return from_bf16_bits(to_bf16_bits(x))


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        return bf16_round(x)
    if dtype == "f32":
        return x
    raise ValueError(f"dtype must be 'bf16' or 'f32', got {dtype!r}")


# ----------------------------------------------------------------------------- masks


def rect_mask(rng: np.random.Generator, grid_h: int, grid_w: int, rect_h: int, rect_w: int) -> np.ndarray:
    """Boolean [grid_h*grid_w] raster mask with one rect_h x rect_w rectangle at a uniform position."""
    top = int(rng.integers(0, grid_h - rect_h + 1))
    left = int(rng.integers(0, grid_w - rect_w + 1))
    m = np.zeros((grid_h, grid_w), dtype=bool)
    m[top:top + rect_h, left:left + rect_w] = True
    return m.reshape(-1)


def rect_mask_fraction(rng: np.random.Generator, grid_h: int, grid_w: int, n_target: int) -> np.ndarray:
    """One axis-aligned rectangle whose area is as close to n_target tokens as an integer rectangle gets."""
    lo = max(1, int(np.ceil(n_target / grid_w)))
    hi = min(grid_h, max(lo, int(np.sqrt(n_target) * 1.6)))
    best = None
    for _ in range(64):
        h = int(rng.integers(lo, hi + 1))
        w = int(round(n_target / h))
        if 1 <= w <= grid_w and (best is None or abs(h * w - n_target) < abs(best[0] * best[1] - n_target)):
            best = (h, w)
            if abs(h * w - n_target) <= 4:
                break
    return rect_mask(rng, grid_h, grid_w, best[0], best[1])


def blob_mask(rng: np.random.Generator, grid_h: int, grid_w: int, n_edited: int) -> np.ndarray:
    """Irregular mask: union of 1-8 Gaussian bumps, thresholded so exactly n_edited tokens are set."""
    n = grid_h * grid_w
    if n_edited <= 0:
        return np.zeros(n, dtype=bool)
    if n_edited >= n:
        return np.ones(n, dtype=bool)
    k = int(rng.integers(1, 9))
    yy, xx = np.meshgrid(np.arange(grid_h), np.arange(grid_w), indexing="ij")
    field = np.zeros((grid_h, grid_w), dtype=np.float64)
    for _ in range(k):
        cy, cx = rng.uniform(0, grid_h), rng.uniform(0, grid_w)
        s = rng.uniform(2.0, 12.0)
        field = np.maximum(field, np.exp(-((yy - cy) ** 2 + (xx - cx) ** 2) / (2 * s * s)))
    order = np.argsort(-field.reshape(-1), kind="stable")
    m = np.zeros(n, dtype=bool)
    m[order[:n_edited]] = True
    return m


# ----------------------------------------------------------------------------- latents


def latents_for_mask(rng: np.random.Generator, want_edited: np.ndarray, c: int, sigma: float, dtype: str = "bf16"):
    """Noisy latent x_t, previous velocity v and reference latent x_ref ([N, c] each) such that a
    one-step estimate lands on the reference for tokens outside `want_edited` and far from it inside.

    x0 = ref outside the mask, ref + N(0,1) inside; x_t = (1-sigma) x0 + sigma eps;
    v = eps - x0 + N(0, 0.02).  Only draws and affine mixing of the draws happen here.
    """
    n = want_edited.shape[0]
    ref = rng.standard_normal((n, c)).astype(np.float32)
    x0 = ref.copy()
    x0[want_edited] += rng.standard_normal((int(want_edited.sum()), c)).astype(np.float32)
    eps = rng.standard_normal((n, c)).astype(np.float32)
    x_t = (1.0 - sigma) * x0 + sigma * eps
    v = eps - x0 + 0.02 * rng.standard_normal((n, c)).astype(np.float32)
    return _store(x_t, dtype), _store(v, dtype), _store(ref, dtype)


# ----------------------------------------------------------------------------- model tensors

_MOD_NAMES = ("shift1", "scale1", "gate1", "shift2", "scale2", "gate2")


def stream_weights(rng: np.random.Generator, hidden: int, mlp: int, kind: str, dtype: str = "bf16", std: float = 0.02):
    """Weights of one stream of a block.  Linear weights are [out_features, in_features].

    kind == "double": w_qkv [3H,H], w_o [H,H], w_1 [M,H], w_2 [H,M] (+ biases).
    kind == "single": w_1 [3H+M,H] producing [q|k|v|m], w_2 [H,H+M] applied to [attn | act(m)].
    Modulation vectors (float32, never rounded): shift/scale small, gate near one.
    """
    def w(o, i):
        a = rng.standard_normal((o, i), dtype=np.float32)
        a *= np.float32(std)
        return _store(a, dtype)

    def b(o):
        return (std * rng.standard_normal(o)).astype(np.float32)

    p = {}
    if kind == "double":
        p["w_qkv"], p["b_qkv"] = w(3 * hidden, hidden), b(3 * hidden)
        p["w_o"], p["b_o"] = w(hidden, hidden), b(hidden)
        p["w_1"], p["b_1"] = w(mlp, hidden), b(mlp)
        p["w_2"], p["b_2"] = w(hidden, mlp), b(hidden)
    elif kind == "single":
        p["w_1"], p["b_1"] = w(3 * hidden + mlp, hidden), b(3 * hidden + mlp)
        p["w_2"], p["b_2"] = w(hidden, hidden + mlp), b(hidden)
    else:
        raise ValueError(kind)
    for name in _MOD_NAMES:
        if kind == "single" and name.endswith("2"):
            continue
        if name.startswith("gate"):
            p[name] = (1.0 + 0.1 * rng.standard_normal(hidden)).astype(np.float32)
        else:
            p[name] = (0.1 * rng.standard_normal(hidden)).astype(np.float32)
    return p


def hidden_states(rng: np.random.Generator, n: int, hidden: int, dtype: str = "bf16") -> np.ndarray:
    return _store(rng.standard_normal((n, hidden), dtype=np.float32), dtype)


def workload_seed(config: int, trial: int = 0) -> int:
    return 1000 * config + trial


# ----------------------------------------------------------------------------- a whole synthetic editor (sampling loop)


def model_weights(rng: np.random.Generator, hidden: int, mlp: int, channels: int, n_double: int, n_single: int, n_txt: int,
                  std: float = 0.02):
    """Random weights of a small MMDiT-shaped editor for the sampling loop (Algorithm 1): token embedding
    Linear(channels -> hidden) whose bias carries the timestep (b + t * b_time), n_double double-stream and
    n_single single-stream blocks, LayerNorm + Linear(hidden -> channels) velocity head, and the text tokens'
    hidden states (the encoded instruction, fixed over the loop).  bf16-representable float32 arrays."""
    embed = {"w": bf16_round((std * 4.0 * rng.standard_normal((hidden, channels))).astype(np.float32)),
             "b": (0.1 * rng.standard_normal(hidden)).astype(np.float32),
             "b_time": (0.5 * rng.standard_normal(hidden)).astype(np.float32)}
    blocks = [("double", [stream_weights(rng, hidden, mlp, "double", "bf16", std) for _ in range(2)]) for _ in range(n_double)]
    blocks += [("single", [stream_weights(rng, hidden, mlp, "single", "bf16", std)]) for _ in range(n_single)]
    head = {"w": bf16_round((std * rng.standard_normal((channels, hidden))).astype(np.float32)),
            "b": (std * rng.standard_normal(channels)).astype(np.float32)}
    h_txt = hidden_states(rng, n_txt, hidden)
    return {"embed": embed, "blocks": blocks, "head": head, "h_txt": h_txt}


def add_block_extras(rng: np.random.Generator, weights: dict, head_dim: int, grid: int, n_txt: int):
    """Switches on the block extras of a model made by model_weights: query/key normalisation vectors for every
    stream, and the positions of the sequence [text | image | reference] on three axes (text (0,0,0), image (0,y,x),
    reference (1,y,x)) with the axes' shares of the head dimension (1/8, 7/16, 7/16).  Drawn after everything else, so
    the other arrays are those of the plain model."""
    for _, streams in weights["blocks"]:
        for w in streams:
            w["q_norm"] = (1.0 + 0.1 * rng.standard_normal(head_dim)).astype(np.float32)
            w["k_norm"] = (1.0 + 0.1 * rng.standard_normal(head_dim)).astype(np.float32)
    yy, xx = np.meshgrid(np.arange(grid), np.arange(grid), indexing="ij")
    pos = [np.zeros((n_txt, 3), dtype=np.int32)]
    pos += [np.stack([np.full(grid * grid, img), yy.ravel(), xx.ravel()], axis=1).astype(np.int32) for img in (0, 1)]
    weights["positions"] = np.concatenate(pos, axis=0)
    weights["rope_axes"] = (head_dim // 8, 7 * head_dim // 16, 7 * head_dim // 16)
    return weights


def loop_latents(rng: np.random.Generator, want_edited: np.ndarray, channels: int, noise: float = 0.1):
    """Start of a sampling loop whose partition is decided by construction: reference latents ~ N(0,1); the
    starting latents equal the reference plus a little noise on the rows that should stay unedited and are
    independent N(0,1) rows where the edit is.  float32."""
    n = want_edited.shape[0]
    x_ref = rng.standard_normal((n, channels)).astype(np.float32)
    x_T = (x_ref + noise * rng.standard_normal((n, channels))).astype(np.float32)
    fresh = rng.standard_normal((n, channels)).astype(np.float32)
    x_T[want_edited] = fresh[want_edited]
    return x_T, x_ref
