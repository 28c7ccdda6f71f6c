"""One region-aware denoising step as a sequence of C-ABI calls (marshalling only).

`RegionStepWorkload` holds the device tensors of one synthetic workload (latents, hidden
states, one block's weights, the layer's KV cache) and `step()` issues the hot path of the
method's region-aware generation stage (Algorithm 1, inner loop) through the binding:

  regione_partition -> regione_gather_pair (hidden rows, latent rows) -> regione_block_forward
  with the retrieve flag (Eq.6) -> regione_velocity_head (velocity head, velocity cache of Eq.9,
  Euler update of Eq.4, merge of the latent rows) -> regione_scatter (hidden rows)

No arithmetic of the method happens here; torch is used for device memory only.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import binding as rg
from . import inputs


@dataclass
class StepConfig:
    name: str
    hidden: int = 3072
    heads: int = 24
    head_dim: int = 128
    mlp: int = 12288
    grid: int = 64            # image tokens = grid * grid, same number of reference tokens
    n_txt: int = 512
    channels: int = 64        # latent channels per token
    n_edited: int = 819       # 20 % of 4096
    mask: str = "rect"        # "rect" | "blob"
    kind: str = "double"      # block type
    sigma: float = 0.7
    eta: float = 0.9
    dt: float = 1.0 / 28.0
    seed: int = 2000
    text_fresh: bool = False  # region step input [X^P, X^E] as in Algorithm 1 (text rows recomputed), not X^E alone with the text in the cache
    extras: bool = False      # query/key RMS normalisation and rotary embedding (positions: text (0,0,0), image (0,y,x), reference (1,y,x))
    dtype: str = "bf16"       # "bf16" | "f32": storage and arithmetic type of the whole step (a float32 context for "f32")


CONFIG_TINY = StepConfig(name="tiny float32: hidden 256, 4x64 heads, MLP 1024, 16x16 image + 256 reference + 32 text tokens, 6x6 rectangle edited",
                         hidden=256, heads=4, head_dim=64, mlp=1024, grid=16, n_txt=32, n_edited=36, seed=1000, dtype="f32")
CONFIG_TINY_BF16 = StepConfig(name="tiny bf16: the same shapes through the bf16 kernels",
                              hidden=256, heads=4, head_dim=64, mlp=1024, grid=16, n_txt=32, n_edited=36, seed=1000)
CONFIG_BLOCK = StepConfig(name="one double-stream block: hidden 3072, 24x128 heads, MLP 12288, 4096 image + 4096 reference + 512 text tokens, "
                               "one rectangle of 20 % edited, KV cache pre-filled")


def host_inputs(cfg: StepConfig):
    """Seeded host arrays of the workload (float32 values; exactly representable in bf16 unless cfg.dtype is "f32")."""
    rng = np.random.default_rng(cfg.seed)
    n_img = cfg.grid * cfg.grid
    if cfg.mask == "rect":
        side = int(round(np.sqrt(cfg.n_edited)))
        if side * side == cfg.n_edited and side <= cfg.grid:
            want = inputs.rect_mask(rng, cfg.grid, cfg.grid, side, side)
        else:
            want = inputs.rect_mask_fraction(rng, cfg.grid, cfg.grid, cfg.n_edited)
    else:
        want = inputs.blob_mask(rng, cfg.grid, cfg.grid, cfg.n_edited)
    store = inputs.bf16_round if cfg.dtype == "bf16" else (lambda a: np.asarray(a, dtype=np.float32))
    x_t, v_prev, x_ref = inputs.latents_for_mask(rng, want, cfg.channels, cfg.sigma, cfg.dtype)
    n_all = cfg.n_txt + 2 * n_img
    h_store = inputs.hidden_states(rng, n_all, cfg.hidden, cfg.dtype)          # hidden state the cache was stored from
    h_now = store((h_store[cfg.n_txt:cfg.n_txt + n_img] + 0.05 * rng.standard_normal((n_img, cfg.hidden))).astype(np.float32))
    n_streams = 2 if cfg.kind == "double" else 1
    streams = [inputs.stream_weights(rng, cfg.hidden, cfg.mlp, cfg.kind, cfg.dtype) for _ in range(n_streams)]
    w_head = store((0.02 * rng.standard_normal((cfg.channels, cfg.hidden))).astype(np.float32))
    b_head = (0.02 * rng.standard_normal(cfg.channels)).astype(np.float32)
    if cfg.extras:   # drawn last, so the other arrays are those of the plain workload
        for w in streams:
            w["q_norm"] = (1.0 + 0.1 * rng.standard_normal(cfg.head_dim)).astype(np.float32)
            w["k_norm"] = (1.0 + 0.1 * rng.standard_normal(cfg.head_dim)).astype(np.float32)
    return dict(want=want, x_t=x_t, v_prev=v_prev, x_ref=x_ref, h_store=h_store, h_now=h_now, streams=streams,
                w_head=w_head, b_head=b_head)


class RegionStepWorkload:
    def __init__(self, cfg: StepConfig, host=None):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.host = host if host is not None else host_inputs(cfg)
        hst = self.host
        n_img = cfg.grid * cfg.grid
        self.n_img, self.n_all = n_img, cfg.n_txt + 2 * n_img
        self.dt = rg.FP32 if cfg.dtype == "f32" else rg.BF16          # dtype enum of every tensor of the step
        self.ctx = rg.Context(cfg.hidden, cfg.heads, cfg.head_dim, cfg.mlp, self.n_all, n_img, compute_dtype=self.dt)
        tdt = self.ctx.torch_dtype
        bf = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(tdt).cuda()   # the step's storage type
        f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
        self.x_t, self.v_prev, self.x_ref = bf(hst["x_t"]), bf(hst["v_prev"]), bf(hst["x_ref"])
        self.h_now = bf(hst["h_now"])
        self._keep = []
        self.weights = rg.BlockWeights()
        for name, w in zip(("txt", "img") if cfg.kind == "double" else ("img",), hst["streams"]):
            t = {k: (rg.pack_weight(self.ctx, bf(a)) if k.startswith("w_") else f32(a)) for k, a in w.items()}
            self._keep.append(t)
            setattr(self.weights, name, rg.make_stream_weights(t))
        if cfg.extras:
            d = cfg.head_dim
            axes = [d // 8, 7 * d // 16, 7 * d // 16]
            yy, xx = np.meshgrid(np.arange(cfg.grid), np.arange(cfg.grid), indexing="ij")
            pos = [np.zeros((cfg.n_txt, 3), dtype=np.int32)]
            pos += [np.stack([np.full(n_img, img), yy.ravel(), xx.ravel()], axis=1).astype(np.int32) for img in (0, 1)]
            self.rope_table = torch.empty((self.n_all, d), dtype=torch.float32, device="cuda")
            rg.regione_rope_table(self.ctx, torch.from_numpy(np.concatenate(pos, axis=0)).cuda(), self.n_all, axes, 10000.0, self.rope_table)
            self.weights.rope, self.weights.rope_rows = self.rope_table.data_ptr(), self.n_all
        self.block_type = rg.BLOCK_DOUBLE if cfg.kind == "double" else rg.BLOCK_SINGLE
        self.w_head, self.b_head = rg.pack_weight(self.ctx, bf(hst["w_head"])), f32(hst["b_head"])
        dev = "cuda"
        self.k_cache = torch.zeros((self.n_all, cfg.heads, cfg.head_dim), dtype=tdt, device=dev)
        self.v_cache = torch.zeros_like(self.k_cache)
        self.score = torch.empty(n_img, dtype=torch.float32, device=dev)
        self.mask = torch.empty(n_img, dtype=torch.uint8, device=dev)
        self.e_index = torch.empty(n_img, dtype=torch.int32, device=dev)
        self.u_index = torch.empty(n_img, dtype=torch.int32, device=dev)
        self.n_dev = torch.zeros(1, dtype=torch.int32, device=dev)
        # fresh rows of the block: [text rows (only with text_fresh) | edited rows]
        self.n_txt_fresh = cfg.n_txt if cfg.text_fresh else 0
        self.h_fresh = torch.empty((self.n_txt_fresh + n_img, cfg.hidden), dtype=tdt, device=dev)
        self.h_fresh_out = torch.empty_like(self.h_fresh)
        self.h_e, self.h_e_out = self.h_fresh[self.n_txt_fresh:], self.h_fresh_out[self.n_txt_fresh:]
        if cfg.text_fresh:
            self.h_fresh[:cfg.n_txt].copy_(bf(hst["h_store"][:cfg.n_txt]))
            self.slots = torch.empty(cfg.n_txt + n_img, dtype=torch.int32, device=dev)   # positions of the fresh rows in [P | X | I]
            self.slots[:cfg.n_txt].copy_(torch.arange(cfg.n_txt, dtype=torch.int32, device=dev))
        self.x_e = torch.empty((n_img, cfg.channels), dtype=tdt, device=dev)
        self.v_e = torch.empty_like(self.x_e)
        self.c_a = torch.zeros_like(self.x_e)
        self.x_next = self.x_t.clone()       # unedited rows keep their value; edited rows are scattered in
        self.h_next = self.h_now.clone()
        self.n_edited = -1
        self._args = None
        self._fill_cache(bf(hst["h_store"]))

    def _fill_cache(self, h_store):
        """The last full forward before the region-aware stage: stores K,V of every row (Algorithm 1, store flag)."""
        torch = self.torch
        slots = torch.arange(self.n_all, dtype=torch.int32, device="cuda")
        out = torch.empty_like(h_store)
        rg.regione_block_forward(self.ctx, self.weights, self.block_type, h_store, out, self.dt, self.n_all, self.cfg.n_txt,
                                 slots, 0, self.k_cache, self.v_cache, self.n_all, rg.FLAG_STORE)
        torch.cuda.synchronize()

    def step(self):
        """One region-aware step as ONE library call (regione_region_step)."""
        cfg = self.cfg
        if self._args is None:
            self._args = rg.make_region_step_args(
                x_t=self.x_t, v=self.v_prev, x_ref=self.x_ref, n_tokens=self.n_img, c=cfg.channels, dtype=self.dt, sigma_t=cfg.sigma, eta=cfg.eta,
                score=self.score, mask=self.mask, e_index=self.e_index, u_index=self.u_index, n_edited_dev=self.n_dev,
                h_full=self.h_now, h_dtype=self.dt, n_txt_fresh=self.n_txt_fresh, h_rows=self.h_fresh, h_rows_out=self.h_fresh_out,
                slots=self.slots if cfg.text_fresh else None, blocks=[self.weights], block_types=[self.block_type],
                k_caches=[self.k_cache], v_caches=[self.v_cache], n_all=self.n_all, slot_offset=cfg.n_txt,
                w_head=self.w_head, b_head=self.b_head, dt=cfg.dt, v_out=self.v_e, c_a=self.c_a, x_e=self.x_e,
                x_next_full=self.x_next, h_next_full=self.h_next)
        n = rg.regione_region_step(self.ctx, self._args)
        self.n_edited = n
        return n

    def step_separate(self):
        """The same step call by call (what regione_region_step stands for); the host waits for the stream after the
        partition to learn the count."""
        cfg, ctx = self.cfg, self.ctx
        n = rg.regione_partition(ctx, self.x_t, self.v_prev, self.x_ref, self.n_img, cfg.channels, self.dt, cfg.sigma, cfg.eta,
                                 self.score, self.mask, self.e_index, self.u_index, self.n_dev)
        self.n_edited = n
        rg.regione_gather_pair(ctx, self.h_now, cfg.hidden, self.dt, self.h_e, self.x_t, cfg.channels, self.dt, self.x_e, self.e_index, self.n_dev, n)
        if cfg.text_fresh:
            rg.regione_fresh_slots(ctx, self.e_index, self.n_dev, n, cfg.n_txt, self.slots)
            rg.regione_block_forward(ctx, self.weights, self.block_type, self.h_fresh, self.h_fresh_out, self.dt, cfg.n_txt + n, cfg.n_txt,
                                     self.slots, 0, self.k_cache, self.v_cache, self.n_all, rg.FLAG_RETRIEVE)
        else:
            rg.regione_block_forward(ctx, self.weights, self.block_type, self.h_e, self.h_e_out, self.dt, n, 0,
                                     self.e_index, cfg.n_txt, self.k_cache, self.v_cache, self.n_all, rg.FLAG_RETRIEVE)
        # velocity head, velocity cache (fresh step, Eq.9), Euler update (Eq.4) and the merge of the latent rows: one fused call
        rg.regione_velocity_head(ctx, self.h_e_out, self.w_head, self.b_head, n, cfg.channels, cfg.hidden, cfg.dt, self.v_e, self.c_a, self.x_e,
                                 self.x_next, self.e_index, self.dt)
        rg.regione_scatter(ctx, self.h_next, cfg.hidden, self.dt, self.e_index, self.n_dev, n, self.h_e_out)
        return n

    def flops(self, n: int):
        """Algorithmic FLOPs of one step for n edited tokens: dense projections and attention (Eq.6), nothing else."""
        cfg = self.cfg
        H, M = cfg.hidden, cfg.mlp
        gemm = 2.0 * n * H * (3 * H + H + 2 * M) + 2.0 * n * H * cfg.channels
        attn = 4.0 * n * self.n_all * H
        return gemm, attn

    def close(self):
        self.ctx.close()
