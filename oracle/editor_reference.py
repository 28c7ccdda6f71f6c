"""A small MMDiT-shaped editor for the sampling loop of Algorithm 1, composed from the oracle's functions.

TEST INFRASTRUCTURE ONLY (see regione_oracle.py).  Plain numpy in float64; imports nothing from the
product.  The model: token embedding Linear(C -> H) whose bias carries the timestep (b + t * b_time),
double-stream then single-stream blocks over the sequence [text | image | reference], LayerNorm and a
Linear(H -> C) velocity head on the image rows.  The full forward runs every row (and, in a storing
step, fills one K,V cache per block); the region forward runs the edited rows only and attends to the
cached rows of all others (Eq.6).  With a second set of text rows and a guidance scale both forwards run
once per branch (each branch has its own caches) and return the guided velocity.

Pins (tests/test_oracle_compositions.py): embedding and head written out by hand; the full forward equals the
block chain over [text | image | reference]; a region forward over every token, or over a subset, with a
same-step cache equals the full forward (restricted); the guided velocity is the combination of two
single-branch editors, each branch with caches of its own.
"""
from __future__ import annotations

import numpy as np

from . import regione_oracle as orc


class EditorReference:
    def __init__(self, weights: dict, heads: int, n_img: int, x_ref, t, h_txt_uncond=None, guidance: float = 1.0):
        self.w = weights
        self.heads = heads
        self.n_img = n_img
        self.h_txt = np.asarray(weights["h_txt"], dtype=np.float64)
        self.n_txt = self.h_txt.shape[0]
        self.guidance = guidance
        self.uncond = None
        if h_txt_uncond is not None:   # the unconditional branch: same weights, other text rows, caches of its own
            w2 = dict(weights)
            w2["h_txt"] = h_txt_uncond
            self.uncond = EditorReference(w2, heads, n_img, x_ref, t)
        self.n_all = self.n_txt + 2 * n_img
        self.hidden = self.h_txt.shape[1]
        self.x_ref = np.asarray(x_ref, dtype=np.float64)
        self.t = t
        d = self.hidden // heads
        self.caches = [(np.zeros((self.n_all, heads, d)), np.zeros((self.n_all, heads, d))) for _ in weights["blocks"]]
        # block extras: rotary angles of every position of the sequence (streams may carry q_norm / k_norm as well)
        self.rope = orc.rope_angles(weights["positions"], weights["rope_axes"]) if "positions" in weights else None
        self.calls = []

    def _embed(self, rows, t):
        e = self.w["embed"]
        return orc.linear(rows, e["w"], np.asarray(e["b"], dtype=np.float64) + t * np.asarray(e["b_time"], dtype=np.float64))

    def _head(self, h):
        return orc.linear(orc.layer_norm(h), self.w["head"]["w"], self.w["head"]["b"])

    def phi(self, x_rows, row_index, i, mode):
        """Signature of regione_oracle.regione_loop's velocity callback."""
        if self.uncond is not None:
            v_c = self._phi_branch(x_rows, row_index, i, mode)
            return orc.guidance_combine(v_c, self.uncond._phi_branch(x_rows, row_index, i, mode), self.guidance)
        return self._phi_branch(x_rows, row_index, i, mode)

    def _phi_branch(self, x_rows, row_index, i, mode):
        t = float(self.t[i])
        self.calls.append((i, mode, None if row_index is None else len(row_index)))
        if mode in ("full", "full_store"):
            h = np.concatenate([self.h_txt, self._embed(np.asarray(x_rows, dtype=np.float64), t), self._embed(self.x_ref, t)], axis=0)
            slots = np.arange(self.n_all)
            flags = orc.FLAG_STORE if mode == "full_store" else 0
            for (kind, streams), (kc, vc) in zip(self.w["blocks"], self.caches):
                h = orc.block_forward(streams, kind, h, self.n_txt, slots, kc, vc, flags, self.heads, rope=self.rope)
            return self._head(h[self.n_txt:self.n_txt + self.n_img])
        if mode != "region":
            raise ValueError(mode)
        if len(row_index) == 0:
            return np.zeros((0, np.asarray(x_rows).shape[1]))
        h = self._embed(np.asarray(x_rows, dtype=np.float64), t)
        slots = self.n_txt + np.asarray(row_index, dtype=np.int64)
        for (kind, streams), (kc, vc) in zip(self.w["blocks"], self.caches):
            h = orc.block_forward(streams, kind, h, 0, slots, kc, vc, orc.FLAG_RETRIEVE, self.heads, rope=self.rope)
        return self._head(h)
