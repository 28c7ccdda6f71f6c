"""The region-aware step of Algorithm 1's inner loop, composed from the oracle's functions.

TEST INFRASTRUCTURE ONLY (see regione_oracle.py).  Takes plain numpy arrays and numbers;
imports nothing from the product.

Pins (tests/test_oracle_compositions.py, tests/test_oracle_block.py): with a cache stored from the step's own
hidden state the region step equals the full forward restricted to the edited rows, in both readings of which
rows are fresh; the merge leaves unedited rows bit-identical; velocity head, Eq.9 and Eq.4 written out by hand;
cached rows come from the right streams; build_cache equals the cache a storing forward writes.
"""
from __future__ import annotations

import numpy as np

from . import regione_oracle as orc


def build_cache(streams, kind, h_store, n_txt, heads):
    """K,V of every row of the sequence [P | X | I] from the hidden state of the last full
    forward (Methodology, "Stabilization Stage": the cache is saved at a complete step).
    Only the key/value projection of the first half of the block is evaluated."""
    n_all, hidden = h_store.shape
    d = hidden // heads
    kc = np.empty((n_all, heads, d)); vc = np.empty_like(kc)
    groups = [(slice(0, n_txt), streams[0]), (slice(n_txt, n_all), streams[-1])] if kind == "double" else [(slice(0, n_all), streams[0])]
    for sl, w in groups:
        u = orc.modulate(orc.layer_norm(h_store[sl]), w.get("shift1"), w.get("scale1"))
        if kind == "double":
            kv = orc.linear(u, w["w_qkv"][hidden:], w["b_qkv"][hidden:])
        else:
            kv = orc.linear(u, w["w_1"][hidden:3 * hidden], w["b_1"][hidden:3 * hidden])
        kc[sl] = kv[:, :hidden].reshape(-1, heads, d)
        vc[sl] = kv[:, hidden:].reshape(-1, heads, d)
    return kc, vc


def region_step(x_t, v_prev, x_ref, h_now, streams, kind, w_head, b_head, k_cache, v_cache,
                n_txt, heads, sigma, eta, dt, h_txt=None):
    """partition -> gather -> block with the retrieve flag (Eq.6) -> velocity head -> velocity cache
    (fresh step, Eq.9) + Euler (Eq.4) -> scatter.  Returns a dict of every intermediate.
    With h_txt [n_txt, H] the block's input is [X^P, X^E] as in Algorithm 1: the text rows are
    fresh too (recomputed, their keys and values replace the cached ones)."""
    score, mask, e_index, u_index = orc.partition(x_t, v_prev, x_ref, sigma, eta)
    h_e = orc.gather(np.asarray(h_now, dtype=np.float64), e_index)
    x_e = orc.gather(np.asarray(x_t, dtype=np.float64), e_index)
    slots = n_txt + e_index.astype(np.int64)
    if h_txt is None:
        h_e_out = orc.block_forward(streams, kind, h_e, 0, slots, k_cache, v_cache, orc.FLAG_RETRIEVE, heads)
    else:
        rows = np.concatenate([np.asarray(h_txt, dtype=np.float64), h_e], axis=0)
        out = orc.block_forward(streams, kind, rows, n_txt, np.concatenate([np.arange(n_txt), slots]), k_cache, v_cache,
                                orc.FLAG_RETRIEVE, heads)
        h_e_out = out[n_txt:]
    v_e = orc.linear(h_e_out, w_head, b_head)
    v_used, c_a, x_e_new = orc.velocity_cache_apply(False, 1.0, dt, v_e, None, x_e)
    x_next = orc.scatter(np.asarray(x_t, dtype=np.float64).copy(), e_index, x_e_new)
    h_next = orc.scatter(np.asarray(h_now, dtype=np.float64).copy(), e_index, h_e_out)
    return dict(score=score, mask=mask, e_index=e_index, u_index=u_index, h_e_out=h_e_out, v_e=v_e, c_a=c_a,
                x_next=x_next, h_next=h_next)
