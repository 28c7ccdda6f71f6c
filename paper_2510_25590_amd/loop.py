"""The sampling loop of the method (Algorithm 1) as a sequence of C-ABI calls (marshalling only).

`EditorModel` keeps a small MMDiT-shaped editor on the device (embedding, double- and single-stream
blocks with one KV cache per block, velocity head) and runs its two forwards through the library:
the full forward over [text | image | reference] rows, which can store every block's K,V
(Algorithm 1, stabilization stage and forced steps), and the region forward over the edited rows
only, which attends to the cached rows (Eq.6).  With a second set of text rows and a guidance scale the
model carries both guidance branches through every block in one batched call (own caches per branch)
and returns the guided velocity.  `run_loop` walks the plan that
`regione_stage_plan_host` returns: full steps, the partition after the stabilization stage, the
one-step jump of the unedited rows (Eq.5), region steps under the adaptive velocity decay cache
(Eq.7-9) and the merges.  Latents, velocities and the velocity cache are float32; rows enter the
embedding as bf16.  No arithmetic of the method happens here; torch is used for device memory only.
"""
from __future__ import annotations

import numpy as np

from . import binding as rg


class EditorModel:
    def __init__(self, weights: dict, hidden: int, heads: int, head_dim: int, mlp: int, channels: int, n_img: int,
                 h_txt_uncond=None, guidance: float = 1.0):
        """weights: host arrays as made by inputs.model_weights (embed, blocks, head, h_txt).  h_txt_uncond: text rows of
        the unconditional branch; with them every forward runs both branches and returns
        v_uncond + guidance * (v_cond - v_uncond)."""
        import torch
        bf = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).cuda()
        f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
        self._setup(hidden, heads, head_dim, mlp, channels, n_img, weights["h_txt"].shape[0], 1 if h_txt_uncond is None else 2, guidance)
        self.w_embed = rg.pack_weight(self.ctx, bf(weights["embed"]["w"]))
        self.b_embed, self.b_time = f32(weights["embed"]["b"]), f32(weights["embed"]["b_time"])
        self.w_head, self.b_head = rg.pack_weight(self.ctx, bf(weights["head"]["w"])), f32(weights["head"]["b"])
        self.h_txt = [bf(weights["h_txt"])] + ([] if h_txt_uncond is None else [bf(h_txt_uncond)])
        if "positions" in weights:   # block extras: rotary table of the whole sequence, shared by all blocks
            self.rope_table = torch.empty((self.n_all, head_dim), dtype=torch.float32, device="cuda")
            rg.regione_rope_table(self.ctx, torch.from_numpy(np.ascontiguousarray(weights["positions"], dtype=np.int32)).cuda(), self.n_all,
                                  list(weights["rope_axes"]), 10000.0, self.rope_table)
        for kind, streams in weights["blocks"]:
            self._add_block(kind, [{k: (rg.pack_weight(self.ctx, bf(a)) if k.startswith("w_") else f32(a)) for k, a in w.items()}
                                   for w in streams])

    @classmethod
    def synthetic(cls, hidden: int, heads: int, head_dim: int, mlp: int, channels: int, n_img: int, n_txt: int,
                  n_double: int, n_single: int, seed: int = 0, std: float = 0.02, guidance=None):
        """The same architecture with N(0, std) weights drawn on the device (for models too large to draw on the host:
        19 double + 38 single blocks at 3072 wide are 17 GB).  For timing only: no oracle sees these weights."""
        import torch
        self = cls.__new__(cls)
        self._setup(hidden, heads, head_dim, mlp, channels, n_img, n_txt, 1 if guidance is None else 2, 1.0 if guidance is None else guidance)
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        rnd = lambda *shape, scale=std: (torch.randn(shape, device="cuda", generator=g) * scale)
        wt = lambda o, i, scale=std: rg.pack_weight(self.ctx, rnd(o, i, scale=scale).to(torch.bfloat16))
        self.w_embed = wt(hidden, channels, 4 * std)
        self.b_embed, self.b_time = rnd(hidden, scale=0.1), rnd(hidden, scale=0.5)
        # head scaled so that the velocity has the spread of the small test models (0.02 * sqrt(256) = 0.32) at any width
        self.w_head, self.b_head = wt(channels, hidden, 0.32 / float(np.sqrt(hidden))), rnd(channels)
        self.h_txt = [rnd(n_txt, hidden, scale=1.0).to(torch.bfloat16) for _ in range(self.n_branches)]

        def stream(kind):
            t = {}
            if kind == "double":
                t["w_qkv"], t["b_qkv"] = wt(3 * hidden, hidden), rnd(3 * hidden)
                t["w_o"], t["b_o"] = wt(hidden, hidden), rnd(hidden)
                t["w_1"], t["b_1"] = wt(mlp, hidden), rnd(mlp)
                t["w_2"], t["b_2"] = wt(hidden, mlp), rnd(hidden)
            else:
                t["w_1"], t["b_1"] = wt(3 * hidden + mlp, hidden), rnd(3 * hidden + mlp)
                t["w_2"], t["b_2"] = wt(hidden, hidden + mlp), rnd(hidden)
            for name in ("shift1", "scale1", "gate1") + (("shift2", "scale2", "gate2") if kind == "double" else ()):
                t[name] = 1.0 + rnd(hidden, scale=0.1) if name.startswith("gate") else rnd(hidden, scale=0.1)
            return t
        for _ in range(n_double):
            self._add_block("double", [stream("double"), stream("double")])
        for _ in range(n_single):
            self._add_block("single", [stream("single")])
        return self

    def _setup(self, hidden, heads, head_dim, mlp, channels, n_img, n_txt, n_branches=1, guidance=1.0):
        import torch
        self.torch = torch
        self.hidden, self.heads, self.head_dim, self.mlp, self.channels = hidden, heads, head_dim, mlp, channels
        self.n_img, self.n_txt = n_img, n_txt
        self.n_all = n_txt + 2 * n_img
        self.n_branches, self.guidance = n_branches, float(guidance)
        self.ctx = rg.Context(hidden, heads, head_dim, mlp, n_branches * self.n_all, n_img)
        self.blocks, self._keep = [], []
        dev = "cuda"
        self.h_a = torch.empty((n_branches, self.n_all, hidden), dtype=torch.bfloat16, device=dev)   # [branch, row, H]
        self.h_b = torch.empty_like(self.h_a)
        self.rows_bf = torch.empty((2 * n_img, channels), dtype=torch.bfloat16, device=dev)
        self.u = torch.empty((n_branches * n_img, hidden), dtype=torch.bfloat16, device=dev)
        self.v_branch = torch.empty((n_branches, n_img, channels), dtype=torch.float32, device=dev)
        self.all_slots = torch.arange(self.n_all, dtype=torch.int32, device=dev)
        self.bias_t = torch.empty(hidden, dtype=torch.float32, device=dev)

    def _add_block(self, kind: str, streams):
        """streams: one dict per stream, name -> device tensor (linear weights already packed)."""
        torch = self.torch
        bw = rg.BlockWeights()
        for name, t in zip(("txt", "img") if kind == "double" else ("img",), streams):
            self._keep.append(t)
            setattr(bw, name, rg.make_stream_weights(t))
        if getattr(self, "rope_table", None) is not None:
            bw.rope, bw.rope_rows = self.rope_table.data_ptr(), self.n_all
        kc = torch.zeros((self.n_branches, self.n_all, self.heads, self.head_dim), dtype=torch.bfloat16, device="cuda")
        self.blocks.append((rg.BLOCK_DOUBLE if kind == "double" else rg.BLOCK_SINGLE, bw, kc, torch.zeros_like(kc)))

    def _embed_bias(self, t: float):
        """Bias of the token embedding at time t, b + t * b_time, formed on the device."""
        rg.regione_time_bias(self.ctx, self.b_embed, self.b_time, float(t), self.bias_t, self.hidden)
        return self.bias_t

    def _head(self, h_rows, n, v_out):
        rg.regione_layernorm(self.ctx, h_rows, rg.BF16, n, self.hidden, None, None, self.u)
        rg.regione_linear(self.ctx, self.u, self.w_head, self.b_head, n, self.channels, self.hidden, rg.ACT_NONE, rg.FP32, v_out)

    def _guided(self, v_branches, n, v_out):
        """v_branches: [2, >= n, C] float32 (conditional, unconditional) -> the guided velocity in v_out."""
        rg.regione_guidance_combine(self.ctx, v_branches[0], v_branches[1], self.guidance, v_out, n * self.channels, rg.FP32)

    def full_forward(self, x, x_ref, t: float, store: bool, v_out):
        """Velocity of all image rows from the full sequence; with `store`, every block writes its K,V cache."""
        ctx, n_img, n_txt, B = self.ctx, self.n_img, self.n_txt, self.n_branches
        rg.regione_cast(ctx, x, rg.FP32, self.rows_bf[:n_img], rg.BF16, n_img * self.channels)
        rg.regione_cast(ctx, x_ref, rg.FP32, self.rows_bf[n_img:], rg.BF16, n_img * self.channels)
        bias = self._embed_bias(t)
        rg.regione_linear(ctx, self.rows_bf, self.w_embed, bias, 2 * n_img, self.hidden, self.channels, rg.ACT_NONE, rg.BF16,
                          self.h_a[0][n_txt:])
        for b in range(B):     # the branches differ in their text rows only
            self.h_a[b][:n_txt].copy_(self.h_txt[b])
            if b > 0:
                self.h_a[b][n_txt:].copy_(self.h_a[0][n_txt:])
        src, dst = self.h_a, self.h_b
        for block_type, bw, kc, vc in self.blocks:
            rg.regione_block_forward_batched(ctx, bw, block_type, src, dst, rg.BF16, B, self.n_all, n_txt, self.all_slots, 0, kc, vc,
                                             self.n_all, rg.FLAG_STORE if store else 0)
            src, dst = dst, src
        if B == 1:
            self._head(src[0][n_txt:n_txt + n_img], n_img, v_out)
            return
        for b in range(B):
            self._head(src[b][n_txt:n_txt + n_img], n_img, self.v_branch[b])
        self._guided(self.v_branch, n_img, v_out)

    def region_forward(self, x_e, e_index, n_e: int, t: float, v_out):
        """Velocity of the edited rows alone; keys and values of all other rows come from the caches (Eq.6)."""
        ctx, B = self.ctx, self.n_branches
        if n_e == 0:
            return
        rg.regione_cast(ctx, x_e, rg.FP32, self.rows_bf, rg.BF16, n_e * self.channels)
        bias = self._embed_bias(t)
        # rows of all branches form one [B, n_e, H] array at the start of the buffers
        src, dst = self.h_a.view(-1, self.hidden), self.h_b.view(-1, self.hidden)
        rg.regione_linear(ctx, self.rows_bf, self.w_embed, bias, n_e, self.hidden, self.channels, rg.ACT_NONE, rg.BF16, src)
        for b in range(1, B):
            src[b * n_e:(b + 1) * n_e].copy_(src[:n_e])
        for block_type, bw, kc, vc in self.blocks:
            rg.regione_block_forward_batched(ctx, bw, block_type, src, dst, rg.BF16, B, n_e, 0, e_index, self.n_txt, kc, vc, self.n_all,
                                             rg.FLAG_RETRIEVE)
            src, dst = dst, src
        if B == 1:
            self._head(src, n_e, v_out)
            return
        v = self.v_branch.view(-1, self.channels)
        self._head(src, B * n_e, v)
        self._guided((v[:n_e], v[n_e:2 * n_e]), n_e, v_out)

    def close(self):
        self.ctx.close()


def run_loop(model: EditorModel, x_T, x_ref, t, gamma, T: int, t_st: int, t_sm: int, forced_k, eta: float, delta: float, grid=None,
             rel_trigger=None, forced_reuse=None):
    """Algorithm 1.  x_T, x_ref: float32 CUDA tensors [n_img, channels]; t, gamma: host sequences of T+1 floats
    (t[T] = 1, t[0] = 0).  Returns (x_0 tensor, log) with log entries (i, what) for every step and one
    ("partition", n_edited); what is "full", "full_store", "region_fresh" or "region_reuse".  grid = (rows, columns)
    of the token grid applies the morphological clean-up to the partition.
    rel_trigger = (threshold, decay): instead of the paper's schedule criterion (Eq.8) the next region step reuses
    decay * C_A when the fresh velocity just computed differs from the previous fresh one by less than `threshold`
    (relative L2 change, `regione_rel_change`); never two reuses in a row; the log then also holds ("rel", i, value).
    forced_reuse {i: bool} overrides the decision of step i."""
    torch = model.torch
    ctx, n_img, c = model.ctx, model.n_img, model.channels
    dev = "cuda"
    x = x_T.clone()
    v = torch.zeros_like(x)                  # velocity of the last full step
    scratch = torch.empty_like(x)
    n_img_dev = torch.full((1,), n_img, dtype=torch.int32, device=dev)
    mask = torch.empty(n_img, dtype=torch.uint8, device=dev)
    e_index = torch.empty(n_img, dtype=torch.int32, device=dev)
    u_index = torch.empty(n_img, dtype=torch.int32, device=dev)
    n_e_dev = torch.zeros(1, dtype=torch.int32, device=dev)
    n_u_dev = torch.zeros(1, dtype=torch.int32, device=dev)
    x_e, v_e, c_a = torch.empty_like(x), torch.empty_like(x), torch.zeros_like(x)
    n_e = None
    log = []
    rel_sums = torch.zeros(2, dtype=torch.float64, device=dev)
    state, rel_state = rg.AvdState(), rg.RelState()
    steps = rg.regione_stage_plan_host(T, t_st, t_sm, forced_k)
    for pos, st in enumerate(steps):
        i = st.i
        if st.kind != rg.STEP_REGION:
            model.full_forward(x, x_ref, t[i], st.kind == rg.STEP_FULL_STORE, v)
            # Eq.4 on all rows: x <- x - (t_i - t_{i-1}) v   (the fresh-velocity form of the cache update, cache unused)
            rg.regione_velocity_cache(ctx, False, 1.0, float(t[i] - t[i - 1]), v, scratch, None, x, n_img_dev, n_img, c, rg.FP32)
            log.append((i, "full_store" if st.kind == rg.STEP_FULL_STORE else "full"))
            continue
        if st.seg_first:
            if n_e is None:   # adaptive region partition, once, from the last full velocity (Eq.5 + cosine + threshold)
                n_e = rg.regione_partition(ctx, x, v, x_ref, n_img, c, rg.FP32, float(t[i]), eta, None, mask, e_index, u_index, n_e_dev)
                if grid is not None:
                    n_e = rg.regione_mask_cleanup(ctx, mask, grid[0], grid[1], 1, mask, e_index, u_index, n_e_dev)
                n_u_dev.fill_(n_img - n_e)
                log.append(("partition", n_e))
            rg.regione_gather(ctx, x, c, rg.FP32, e_index, n_e_dev, n_e, x_e)
            # one jump of the unedited rows to the end of the segment with the last full velocity (Eq.5), in place: nothing
            # reads those rows of x before the merge, where the edited rows join them
            rg.regione_euler_rows(ctx, x, v, u_index, n_u_dev, n_img - n_e, c, rg.FP32, float(t[i] - t[st.seg_next + 1]))
            state, rel_state = rg.AvdState(), rg.RelState()
        if rel_trigger is None:
            reuse, factor = rg.regione_velocity_decision_host(t, gamma, T, delta, i, state)
        else:
            reuse, factor = rg.regione_rel_decision_host(rel_state, float(rel_trigger[1]))
            if forced_reuse is not None and i in forced_reuse:     # a test harness imposing another run's decisions
                reuse = bool(forced_reuse[i]) and bool(rel_state.have_cache)
                factor = float(rel_trigger[1]) if reuse else 1.0
        if not reuse:
            model.region_forward(x_e, e_index, n_e, t[i], v_e)
            if rel_trigger is not None:
                had_cache = bool(rel_state.have_cache)      # c_a still holds the previous fresh velocity
                sums = rg.regione_rel_change(ctx, v_e, c_a, n_e * c, rg.FP32, rel_sums, read_back=True) if had_cache and n_e > 0 else None
                rel = rg.regione_rel_update_host(rel_state, sums, float(rel_trigger[0]))
                if had_cache:
                    log.append(("rel", i, rel))
        rg.regione_velocity_cache(ctx, reuse, factor, float(t[i] - t[i - 1]), None if reuse else v_e, c_a, None, x_e, n_e_dev, n_e, c, rg.FP32)
        log.append((i, "region_reuse" if reuse else "region_fresh"))
        last_of_segment = pos + 1 == len(steps) or steps[pos + 1].kind != rg.STEP_REGION
        if last_of_segment:   # merge: edited and unedited rows are both at t_{next+1} now
            rg.regione_scatter(ctx, x, c, rg.FP32, e_index, n_e_dev, n_e, x_e)
    torch.cuda.synchronize()
    return x, log
