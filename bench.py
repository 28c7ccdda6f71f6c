#!/usr/bin/env python3
"""Benchmark of the RegionE region-aware step on one MI355X.

A "step" is one pass of the whole hot path over one synthetic image: adaptive region
partition, gather of the edited tokens, one 3072-wide double-stream transformer block on
them with attention over the Region-Instruction KV cache, the velocity head, the velocity
cache + Euler update and the scatter back.  Inputs are resident in HBM before the timed
region.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_FP8_TFLOPS = 5000.0    # MI355X dense fp8 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def profiled_traffic():
    """HBM-side bytes per launch from the committed rocprofv3 counter summaries (FETCH_SIZE / WRITE_SIZE runs, scaled by
    what the same counters read for a plain copy of known size): the lines `traffic_bytes_per_launch <key> <bytes>` of
    profiles/*_hbm_traffic.txt.  A key that no summary carries reads as None."""
    import glob
    table = {}
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*_hbm_traffic.txt"))):
        for line in open(path):
            parts = line.split()
            if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch":
                table[parts[1]] = float(parts[2])
    return table


def cpu_baseline(cfg, hst, reps, gpu=None):
    """The oracle as it stands, timed on the host cores: the same step on the same inputs.  With the GPU's outputs of
    that step (`gpu`) the line also carries how far the two are apart."""
    from oracle import step_reference as ref
    kc, vc = ref.build_cache(hst["streams"], cfg.kind, hst["h_store"], cfg.n_txt, cfg.heads)   # setup, like the GPU's cache fill
    t0 = time.perf_counter()
    for _ in range(reps):
        out = ref.region_step(hst["x_t"], hst["v_prev"], hst["x_ref"], hst["h_now"], hst["streams"], cfg.kind, hst["w_head"],
                              hst["b_head"], kc, vc, cfg.n_txt, cfg.heads, cfg.sigma, cfg.eta, cfg.dt)
    dt = (time.perf_counter() - t0) / reps
    n = len(out["e_index"])
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    res = {"value": n / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
           "sample": f"the whole workload ({n} edited tokens), {reps} step(s) of the numpy float64 oracle, {dt:.2f} s per step"}
    if gpu is not None:
        import numpy as np
        want = out["h_e_out"]
        diff = np.abs(gpu["h_e_out"][:n].astype(np.float64) - want)
        half_ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 2.0 ** -126))) - 8)     # what bf16 storage of the output can add
        res["parity"] = {"mask_equal": bool(np.array_equal(gpu["mask"], out["mask"])),
                         "index_lists_equal": bool(np.array_equal(gpu["e_index"][:n], out["e_index"])),
                         "stated_tolerance": {"max_abs": 2e-2, "mean_rel": 5e-3},
                         "block_out_max_abs": float(diff.max()), "block_out_mean_rel": float(diff.mean() / np.abs(want).mean()),
                         "block_out_elements": int(diff.size),
                         "block_out_over_2e-2": int((diff > 2e-2).sum()), "block_out_over_2e-2_frac": float((diff > 2e-2).mean()),
                         "block_out_over_2e-2_plus_bf16_half_ulp": int((diff > 2e-2 + half_ulp).sum()),
                         "merged_latent_max_abs": float(np.abs(gpu["x_next"].astype(np.float64) - out["x_next"]).max())}
        if gpu.get("h_e_out_f32") is not None:   # the same block with a float32 residual stream: no storage rounding in the way
            d32 = np.abs(gpu["h_e_out_f32"].astype(np.float64) - want)
            res["parity"]["f32_residual"] = {"block_out_max_abs": float(d32.max()), "block_out_mean_rel": float(d32.mean() / np.abs(want).mean()),
                                             "block_out_rms": float(np.sqrt((d32 ** 2).mean())),
                                             "block_out_over_2e-2": int((d32 > 2e-2).sum()), "block_out_over_2e-2_frac": float((d32 > 2e-2).mean())}
    return res


def membound(torch, rg):
    """HBM-bound kernels on a working set far larger than the 256 MB Infinity Cache (a batch of images as one token list)."""
    res = {}
    n_tok, c = 2048 * 4096, 64                      # 2048 images of 64x64 tokens: 3 x 1 GiB of bf16 latents
    ctx = rg.Context(256, 4, 64, 1024, 16, n_tok)
    # launch floor: the smallest kernel of the library (an 8-element copy), timed like everything else by the event
    # pairs around its launch; the single-image figures of the step ("kernels" above) are to be read against it
    tiny_src = torch.zeros(8, dtype=torch.float32, device="cuda"); tiny_dst = torch.zeros_like(tiny_src)
    rg.regione_profile_enable(ctx, True)
    for _ in range(5):
        rg.regione_cast(ctx, tiny_src, rg.FP32, tiny_dst, rg.FP32, 8)
    rg.regione_profile_read(ctx)
    for _ in range(50):
        rg.regione_cast(ctx, tiny_src, rg.FP32, tiny_dst, rg.FP32, 8)
    res["launch_floor_us"] = rg.regione_profile_read(ctx)["rows"][0] / 50 * 1e3
    rg.regione_profile_enable(ctx, False)
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    ref = torch.randn((n_tok, c), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    noise = torch.randn((n_tok, c), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    edited = (torch.rand(n_tok, generator=g, device="cuda") < 0.2).to(torch.bfloat16).unsqueeze(1)
    x_t = (0.3 * (ref.float() + edited.float() * noise.float())).to(torch.bfloat16)   # sigma 0.7, v = -x0  =>  x0_hat = x0
    v = (-(ref.float() + edited.float() * noise.float())).to(torch.bfloat16)
    del noise, edited
    score = torch.empty(n_tok, dtype=torch.float32, device="cuda")
    mask = torch.empty(n_tok, dtype=torch.uint8, device="cuda")
    e_idx = torch.empty(n_tok, dtype=torch.int32, device="cuda"); u_idx = torch.empty_like(e_idx)
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    for _ in range(2):
        n_e = rg.regione_partition(ctx, x_t, v, ref, n_tok, c, rg.BF16, 0.7, 0.9, score, mask, e_idx, u_idx, cnt)
    rg.regione_profile_enable(ctx, True)
    reps = 5
    for _ in range(reps):
        rg.regione_partition(ctx, x_t, v, ref, n_tok, c, rg.BF16, 0.7, 0.9, score, mask, e_idx, u_idx, cnt, read_count=False)
    ms = rg.regione_profile_read(ctx)["partition"][0] / reps
    nbytes = n_tok * (3 * c * 2 + 4 + 1 + 4)        # three latents in; score, mask, one index out
    res["partition"] = {"tokens": n_tok, "edited": n_e, "ms": ms, "GB/s": nbytes / ms / 1e6, "frac_hbm": nbytes / ms / 1e6 / PEAK_HBM_GBS,
                        "bytes_per_token": 3 * c * 2 + 9, "outputs": "score, mask, index lists"}
    # the same without the optional score output (the method itself needs only the mask and the index lists)
    for _ in range(reps):
        rg.regione_partition(ctx, x_t, v, ref, n_tok, c, rg.BF16, 0.7, 0.9, None, mask, e_idx, u_idx, cnt, read_count=False)
    ms = rg.regione_profile_read(ctx)["partition"][0] / reps
    nbytes = n_tok * (3 * c * 2 + 1 + 4)
    res["partition_no_score"] = {"tokens": n_tok, "edited": n_e, "ms": ms, "GB/s": nbytes / ms / 1e6, "frac_hbm": nbytes / ms / 1e6 / PEAK_HBM_GBS,
                                 "bytes_per_token": 3 * c * 2 + 5, "outputs": "mask, index lists"}
    # gather / scatter of 128-byte latent rows through the index list just built
    dst = torch.empty((n_e, c), dtype=torch.bfloat16, device="cuda")
    for name, fn in (("gather_latent", lambda: rg.regione_gather(ctx, x_t, c, rg.BF16, e_idx, cnt, n_e, dst)),
                     ("scatter_latent", lambda: rg.regione_scatter(ctx, x_t, c, rg.BF16, e_idx, cnt, n_e, dst))):
        fn(); rg.regione_profile_read(ctx)
        for _ in range(reps):
            fn()
        ms = rg.regione_profile_read(ctx)["rows"][0] / reps
        nb = n_e * (2 * c * 2 + 4)
        res[name] = {"rows": n_e, "row_bytes": 2 * c, "ms": ms, "GB/s": nb / ms / 1e6, "frac_hbm": nb / ms / 1e6 / PEAK_HBM_GBS}
    # velocity cache with the Euler update on the gathered rows (Eq.9, Eq.4): a fresh step reads v and x_e and writes the
    # cache and x_e; a reusing step reads the cache and x_e and writes x_e
    xe = torch.empty((n_e, c), dtype=torch.bfloat16, device="cuda").normal_(generator=g)
    ca = torch.empty_like(xe)
    for name, reuse, arrays in (("velocity_cache_fresh", False, 4), ("velocity_cache_reuse", True, 3)):
        fn = lambda: rg.regione_velocity_cache(ctx, reuse, 0.9, 1 / 28, dst, ca, None, xe, cnt, n_e, c, rg.BF16)
        fn(); rg.regione_profile_read(ctx)
        for _ in range(reps):
            fn()
        ms = rg.regione_profile_read(ctx)["velocity"][0] / reps
        nb = n_e * c * 2 * arrays
        res[name] = {"rows": n_e, "row_bytes": 2 * c, "ms": ms, "GB/s": nb / ms / 1e6, "frac_hbm": nb / ms / 1e6 / PEAK_HBM_GBS}
    del xe, ca
    del x_t, v, ref, score, mask, dst
    # gather / scatter of 6 KiB hidden rows: 20 % of 256 images' tokens
    hidden = 3072
    n_rows_full = 256 * 4096
    src = torch.empty((n_rows_full, hidden), dtype=torch.bfloat16, device="cuda").normal_(generator=g)
    n_h = int((e_idx[:n_e] < n_rows_full).sum().item())
    dst = torch.empty((n_h, hidden), dtype=torch.bfloat16, device="cuda")
    for name, fn in (("gather_hidden", lambda: rg.regione_gather(ctx, src, hidden, rg.BF16, e_idx, None, n_h, dst)),
                     ("scatter_hidden", lambda: rg.regione_scatter(ctx, src, hidden, rg.BF16, e_idx, None, n_h, dst))):
        fn(); rg.regione_profile_read(ctx)
        for _ in range(reps):
            fn()
        ms = rg.regione_profile_read(ctx)["rows"][0] / reps
        nb = n_h * (2 * hidden * 2 + 4)
        res[name] = {"rows": n_h, "row_bytes": 2 * hidden, "ms": ms, "GB/s": nb / ms / 1e6, "frac_hbm": nb / ms / 1e6 / PEAK_HBM_GBS}
    del src, dst
    # modulation vectors of 64 double-stream blocks (two streams each) from one conditioning vector: 128 matrices
    # [6H, H] of bf16, 14.5 GB in all, each read once
    n_mod, n_mats = 6 * hidden, 128
    mats = torch.empty((n_mats, n_mod, hidden), dtype=torch.bfloat16, device="cuda").normal_(generator=g)
    emb = torch.randn(hidden, generator=g, device="cuda", dtype=torch.float32)
    bias = torch.zeros(n_mod, dtype=torch.float32, device="cuda")
    y = torch.empty((n_mats, n_mod), dtype=torch.float32, device="cuda")
    bias_all = torch.zeros(n_mats * n_mod, dtype=torch.float32, device="cuda")
    nb = n_mats * (n_mod * hidden * 2 + n_mod * 8) + hidden * 4
    for name, run in (("modulation_vec_linear", lambda: rg.regione_vec_linear(ctx, emb, rg.ACT_SILU, mats, bias_all, n_mats * n_mod, hidden, y)),
                      ("modulation_vec_linear_per_block", lambda: [rg.regione_vec_linear(ctx, emb, rg.ACT_SILU, mats[i], bias, n_mod, hidden, y[i]) for i in range(n_mats)])):
        run(); rg.regione_profile_read(ctx)
        run()
        ms = rg.regione_profile_read(ctx)["gemm"][0]
        res[name] = {"matrices": n_mats, "rows": n_mod, "cols": hidden, "ms": ms, "GB/s": nb / ms / 1e6, "frac_hbm": nb / ms / 1e6 / PEAK_HBM_GBS}
    ctx.close()
    return res


def cfg_benchmark(steps: int, warmup: int):
    """The block of the headline workload for the TWO branches of classifier-free guidance (the paper's experiments
    run both at every step): one batched call against two single calls.  Same 820 edited rows and 8704 cache rows
    per branch; the second branch has its own hidden state and cache."""
    import torch
    from paper_2510_25590_amd import binding as rg
    from paper_2510_25590_amd import step
    cfg = step.CONFIG_BLOCK
    wl = step.RegionStepWorkload(cfg)
    n = wl.step()
    torch.cuda.synchronize()
    ctx2 = rg.Context(cfg.hidden, cfg.heads, cfg.head_dim, cfg.mlp, 2 * wl.n_img, 16)
    g = torch.Generator(device="cuda"); g.manual_seed(11)
    h_e = torch.stack([wl.h_e[:n], (wl.h_e[:n].float() + 0.05 * torch.randn((n, cfg.hidden), generator=g, device="cuda")).to(torch.bfloat16)]).contiguous()
    kc = torch.stack([wl.k_cache, wl.k_cache.flip(0)]).contiguous(); vc = torch.stack([wl.v_cache, wl.v_cache.flip(0)]).contiguous()
    out = torch.empty_like(h_e)
    e_index = wl.e_index[:n].contiguous()

    def two_calls():
        for b in range(2):
            rg.regione_block_forward(ctx2, wl.weights, wl.block_type, h_e[b], out[b], rg.BF16, n, 0, e_index, cfg.n_txt, kc[b], vc[b], wl.n_all, rg.FLAG_RETRIEVE)

    def batched():
        rg.regione_block_forward_batched(ctx2, wl.weights, wl.block_type, h_e, out, rg.BF16, 2, n, 0, e_index, cfg.n_txt, kc, vc, wl.n_all, rg.FLAG_RETRIEVE)

    res = {}
    for name, fn in (("two_calls", two_calls), ("batched", batched)):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        rg.regione_profile_enable(ctx2, True); rg.regione_profile_read(ctx2)
        for _ in range(steps):
            fn()
        prof = rg.regione_profile_read(ctx2)
        rg.regione_profile_enable(ctx2, False)
        res[name] = {"ms_per_block": ms, "tokens_per_s": 2 * n / (ms * 1e-3),
                     "kernels_ms": {k: v[0] / steps for k, v in prof.items() if v[0] > 0}}
    return {"metric": "edited-token DiT block tokens/s, two guidance branches", "value": res["batched"]["tokens_per_s"], "unit": "tokens/s",
            "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": res["batched"]["ms_per_block"], "higher_is_better": True,
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": cfg.name + "; block only, two branches", "n_edited_per_branch": n}, "detail": res}


def stack_benchmark():
    """The large-image configuration: 60 double-stream blocks at 3072 wide, 96x96 image + 9216 reference + 1024 text
    tokens (19456 rows, 14.3 GB of KV cache), 15 % of the image edited (1382 tokens of a blob): one storing full step
    and one region step through the whole stack."""
    import numpy as np
    import torch
    from paper_2510_25590_amd import binding as rg, inputs, loop
    grid, channels, n_txt, n_blocks = 96, 64, 1024, 60
    n_img = grid * grid
    rng = np.random.default_rng(inputs.workload_seed(5, 1))
    want = inputs.blob_mask(rng, grid, grid, 1382)
    x_T, x_ref = inputs.loop_latents(rng, want, channels)
    model = loop.EditorModel.synthetic(3072, 24, 128, 12288, channels, n_img, n_txt, n_blocks, 0, seed=5)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    x, x_r = dev(x_T), dev(x_ref)
    v = torch.zeros_like(x)
    e = torch.from_numpy(np.nonzero(want)[0].astype(np.int32)).cuda()
    n_e = int(want.sum())
    x_e = x[e.long()].contiguous(); v_e = torch.zeros_like(x_e)
    out = {"workload": f"{n_blocks} double-stream blocks at 3072 wide, {n_img} image + {n_img} reference + {n_txt} text tokens, {n_e} edited"}
    for name, fn in (("full_store_step", lambda: model.full_forward(x, x_r, 0.8, True, v)),
                     ("region_step", lambda: model.region_forward(x_e, e, n_e, 0.75, v_e))):
        fn(); torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        out[name] = {"seconds": (time.perf_counter() - t0) / 3}
    n_all = n_txt + 2 * n_img
    H, M = 3072, 12288
    full_flops = n_blocks * (2.0 * n_all * H * (4 * H + 2 * M) + 4.0 * n_all * n_all * H)
    region_flops = n_blocks * (2.0 * n_e * H * (4 * H + 2 * M) + 4.0 * n_e * n_all * H)
    out["full_store_step"]["TFLOP/s"] = full_flops / out["full_store_step"]["seconds"] / 1e12
    out["region_step"]["TFLOP/s"] = region_flops / out["region_step"]["seconds"] / 1e12
    out["region_step"]["edited_tokens_per_s"] = n_e / out["region_step"]["seconds"]
    out["region_step"]["ms_per_block"] = out["region_step"]["seconds"] / n_blocks * 1e3
    out["finite"] = bool(torch.isfinite(v).all().item() and torch.isfinite(v_e).all().item())
    model.close()
    return out


def loop_benchmark(n_double: int, n_single: int, guidance=None):
    """Whole sampling loop on the device: the method's 28-step schedule (6 stabilization steps, forced step at k = 16,
    2 smooth steps, velocity-decay cache with delta = 0.04 on a linear schedule) against 28 plain full steps of the same
    editor.  3072 wide, 24 heads of 128, MLP 12288, 64x64 image + 4096 reference + 512 text tokens, one 25 % blob edited
    (constructed so that the partition finds exactly it), random weights drawn on the device."""
    import numpy as np
    import torch
    from paper_2510_25590_amd import binding as rg, inputs, loop
    T, t_st, t_sm, forced = 28, 6, 2, [16]
    grid, channels, n_txt = 64, 64, 512
    n_img = grid * grid
    rng = np.random.default_rng(inputs.workload_seed(4, 9))
    want = inputs.blob_mask(rng, grid, grid, n_img // 4)
    x_T, x_ref = inputs.loop_latents(rng, want, channels)
    model = loop.EditorModel.synthetic(3072, 24, 128, 12288, channels, n_img, n_txt, n_double, n_single, seed=4, guidance=guidance)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    x_T_d, x_ref_d = dev(x_T), dev(x_ref)
    t = [k / T for k in range(T + 1)]
    gamma = [1.0] * (T + 1)
    out = {"workload": f"28-step sampling loop, {n_double} double + {n_single} single blocks at 3072 wide, 4096 image + 4096 reference + 512 text tokens"
                       + ("" if guidance is None else f", classifier-free guidance (two branches per step, scale {guidance})")}
    # "regione": the paper's schedule criterion (Eq.8, gamma = 1, delta = 0.04); "regione_relative_trigger": the data-dependent
    # trigger of the workload description (reuse 0.9 * cached velocity when two fresh velocities differ by less than 5 %)
    for name, kwargs in (("regione", dict(t_st=t_st, t_sm=t_sm, forced_k=forced, delta=0.04)),
                         ("regione_relative_trigger", dict(t_st=t_st, t_sm=t_sm, forced_k=forced, delta=0.04, rel_trigger=(0.05, 0.9))),
                         ("vanilla", dict(t_st=T - 1, t_sm=1, forced_k=[], delta=-1.0))):    # every step a full step
        for rep in range(2):    # first pass warms up (allocations, first launches)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            x0, log = loop.run_loop(model, x_T_d, x_ref_d, t, gamma, T, kwargs["t_st"], kwargs["t_sm"], kwargs["forced_k"], 0.8, kwargs["delta"],
                                    rel_trigger=kwargs.get("rel_trigger"))
            torch.cuda.synchronize()
            sec = time.perf_counter() - t0
        kinds = [w[1] for w in log if w[0] not in ("partition", "rel")]
        out[name] = {"seconds": sec, "full_steps": sum(k.startswith("full") for k in kinds), "region_fresh": kinds.count("region_fresh"),
                     "region_reuse": kinds.count("region_reuse"), "n_edited": next((w[1] for w in log if w[0] == "partition"), None),
                     "finite": bool(torch.isfinite(x0).all().item())}
        if kwargs.get("rel_trigger"):
            out[name]["relative_changes"] = [round(w[2], 4) for w in log if w[0] == "rel"]
    out["speedup"] = out["vanilla"]["seconds"] / out["regione"]["seconds"]
    out["n_edited_constructed"] = int(want.sum())
    model.close()
    return out


def fp8_projections(torch, rg, n_rows: int, reps: int = 20):
    """The four dense projections of the headline block on n_rows edited rows, bf16 against the E4M3 variant
    (row quantisation of the activations timed with it; weights are quantised and packed once, outside)."""
    hidden, mlp = 3072, 12288
    ctx = rg.Context(hidden, 24, 128, mlp, max(n_rows, 16), 16)
    g = torch.Generator(device="cuda"); g.manual_seed(9)
    res = {"rows": n_rows, "format": "OCP E4M3, one float32 scale per activation row and per output feature", "peak_TFLOPs": PEAK_FP8_TFLOPS, "shapes": {}}
    tot = {"bf16_us": 0.0, "fp8_us": 0.0, "quantize_us": 0.0, "flops": 0.0}
    for name, n, k in (("qkv", 3 * hidden, hidden), ("attn_out", hidden, hidden), ("mlp_up", mlp, hidden), ("mlp_down", hidden, mlp)):
        x = torch.randn((n_rows, k), generator=g, device="cuda").to(torch.bfloat16)
        w = (torch.randn((n, k), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
        wp = rg.pack_weight(ctx, w)
        xq = torch.empty((n_rows, k), dtype=torch.uint8, device="cuda"); sx = torch.empty(n_rows, dtype=torch.float32, device="cuda")
        wq = torch.empty((n, k), dtype=torch.uint8, device="cuda"); sw = torch.empty(n, dtype=torch.float32, device="cuda")
        rg.regione_quantize_rows_fp8(ctx, w, n, k, wq, sw)
        wqp = torch.zeros(rg.regione_packed_weight_elems(n, k), dtype=torch.uint8, device="cuda")
        rg.regione_pack_weight_fp8(ctx, wq, n, k, wqp)
        y16 = torch.empty((n_rows, n), dtype=torch.bfloat16, device="cuda"); y8 = torch.empty_like(y16)
        run16 = lambda: rg.regione_linear(ctx, x, wp, None, n_rows, n, k, rg.ACT_NONE, rg.BF16, y16)
        def run8():
            rg.regione_quantize_rows_fp8(ctx, x, n_rows, k, xq, sx)
            rg.regione_linear_fp8(ctx, xq, sx, wqp, sw, None, n_rows, n, k, rg.ACT_NONE, rg.BF16, y8)
        for _ in range(3):
            run16(); run8()
        torch.cuda.synchronize()
        rg.regione_profile_enable(ctx, True); rg.regione_profile_read(ctx)
        for _ in range(reps):
            run16()
        t16 = rg.regione_profile_read(ctx)["gemm"][0] / reps * 1e3
        for _ in range(reps):
            run8()
        prof = rg.regione_profile_read(ctx)
        rg.regione_profile_enable(ctx, False)
        t8, tq = prof["gemm"][0] / reps * 1e3, prof["rows"][0] / reps * 1e3
        fl = 2.0 * n_rows * n * k
        rel = float((y8.float() - y16.float()).norm() / y16.float().norm())
        res["shapes"][name] = {"n": n, "k": k, "bf16_us": t16, "fp8_us": t8, "quantize_us": tq, "bf16_TFLOPs": fl / t16 * 1e-6,
                               "fp8_TFLOPs": fl / t8 * 1e-6, "frac_fp8_peak": fl / t8 * 1e-6 / PEAK_FP8_TFLOPS, "rel_diff_to_bf16": rel}
        tot["bf16_us"] += t16; tot["fp8_us"] += t8; tot["quantize_us"] += tq; tot["flops"] += fl
        del x, w, wp, xq, sx, wq, sw, wqp, y16, y8
    res["all_four"] = {"bf16_us": tot["bf16_us"], "fp8_us": tot["fp8_us"], "quantize_us": tot["quantize_us"],
                       "speedup_with_quantize": tot["bf16_us"] / (tot["fp8_us"] + tot["quantize_us"]),
                       "fp8_TFLOPs": tot["flops"] / tot["fp8_us"] * 1e-6}
    ctx.close()
    return res


def fp8_block(torch, rg, steps: int, warmup: int):
    """The headline block (820 edited rows, 8704 cache rows, retrieve flag) with its four projections in E4M3
    (regione_block_forward_fp8: quantisation fused into the LayerNorms, two quantisation launches for the attention
    output and the MLP rows) against the bf16 block, same process, alternating.  Secondary figure: an extension with its
    own accuracy (tests/test_gpu_block_fp8.py), never the headline."""
    from paper_2510_25590_amd import step
    cfg = step.CONFIG_BLOCK
    wl = step.RegionStepWorkload(cfg)
    n = wl.step()
    torch.cuda.synchronize()
    ctx = wl.ctx
    bf = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    w8 = rg.BlockWeightsFp8()
    w8.txt, keep_t = rg.make_stream_weights_fp8(ctx, {k: bf(v) for k, v in wl.host["streams"][0].items() if k.startswith("w_")})
    w8.img, keep_i = rg.make_stream_weights_fp8(ctx, {k: bf(v) for k, v in wl.host["streams"][1].items() if k.startswith("w_")})
    for kp in (keep_t, keep_i):          # the unpacked codes are not needed here
        for name in kp:
            kp[name] = kp[name][:2]
    out16 = torch.empty((n, cfg.hidden), dtype=torch.bfloat16, device="cuda"); out8 = torch.empty_like(out16)
    h_e = wl.h_e[:n].clone()
    run16 = lambda: rg.regione_block_forward(ctx, wl.weights, wl.block_type, h_e, out16, rg.BF16, n, 0, wl.e_index, cfg.n_txt, wl.k_cache, wl.v_cache, wl.n_all, rg.FLAG_RETRIEVE)
    run8 = lambda: rg.regione_block_forward_fp8(ctx, wl.weights, w8, wl.block_type, h_e, out8, rg.BF16, n, 0, wl.e_index, cfg.n_txt, wl.k_cache, wl.v_cache, wl.n_all, rg.FLAG_RETRIEVE)
    res = {"rows": int(n), "keys_per_query": wl.n_all}
    for rnd in range(2):
        for name, fn in (("bf16", run16), ("fp8", run8)):
            for _ in range(warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fn()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / steps
            res[name + "_block_ms"] = min(ms, res.get(name + "_block_ms", ms))
    rg.regione_profile_enable(ctx, True); rg.regione_profile_read(ctx)
    for _ in range(steps):
        run8()
    prof = rg.regione_profile_read(ctx)
    rg.regione_profile_enable(ctx, False)
    res["fp8_kernels_ms"] = {k: v[0] / steps for k, v in prof.items() if v[1]}
    gemm_flops, _ = wl.flops(n)
    gemm_flops -= 2.0 * n * cfg.hidden * cfg.channels          # the velocity head is not part of the block
    g_ms = prof["gemm"][0] / steps
    res["fp8_gemm_TFLOPs"] = gemm_flops / (g_ms * 1e-3) / 1e12
    res["fp8_gemm_frac_of_fp8_peak"] = res["fp8_gemm_TFLOPs"] / PEAK_FP8_TFLOPS
    res["speedup"] = res["bf16_block_ms"] / res["fp8_block_ms"]
    upd16, upd8 = out16.float() - h_e.float(), out8.float() - h_e.float()
    res["rel_diff_of_block_update_to_bf16"] = float((upd8 - upd16).norm() / upd16.norm())
    wl.close()
    return res


def measured_peaks(torch, rg):
    """What this chip sustains on register-only MFMA loops (at the clock it holds under that load) and on a plain 1 GiB copy
    through the library's own row kernel: the figures to read the achieved TFLOP/s and GB/s against, beside the nominal peaks."""
    ctx = rg.Context(256, 4, 64, 1024, 16, 16)
    res = {}
    out = torch.empty(2048 * 256, dtype=torch.float32, device="cuda")
    rg.regione_profile_enable(ctx, True)
    for name, fmt, nominal in (("mfma_bf16", 0, PEAK_BF16_TFLOPS), ("mfma_fp8_e4m3", 1, PEAK_FP8_TFLOPS)):
        best = None
        for wgs in (512, 1024, 2048):           # 2, 4 and 8 waves per SIMD
            rg.regione_mfma_peak_probe(ctx, fmt, 2000, wgs, out)
            rg.regione_profile_read(ctx)
            flops = sum(rg.regione_mfma_peak_probe(ctx, fmt, 20000, wgs, out) for _ in range(3))
            ms = rg.regione_profile_read(ctx)["gemm"][0]
            tf = flops / ms * 1e-9
            if best is None or tf > best[0]:
                best = (tf, wgs, ms / 3)
        res[name] = {"TFLOPs": best[0], "workgroups": best[1], "ms": best[2], "nominal_TFLOPs": nominal, "frac_of_nominal": best[0] / nominal,
                     "implied_clock_GHz": best[0] / nominal * 2.4}
    n = 1 << 28
    src = torch.zeros(n, dtype=torch.float32, device="cuda"); dst = torch.empty_like(src)
    rg.regione_cast(ctx, src, rg.FP32, dst, rg.FP32, n)
    rg.regione_profile_read(ctx)
    for _ in range(5):
        rg.regione_cast(ctx, src, rg.FP32, dst, rg.FP32, n)
    ms = rg.regione_profile_read(ctx)["rows"][0] / 5
    rg.regione_profile_enable(ctx, False)
    res["hbm_copy"] = {"bytes_read_plus_written": 8 * n, "ms": ms, "GB/s": 8 * n / ms / 1e6, "nominal_GB/s": PEAK_HBM_GBS, "frac_of_nominal": 8 * n / ms / 1e6 / PEAK_HBM_GBS}
    # the same copy by the HIP runtime (torch's copy_ of a contiguous tensor), for comparison
    dst.copy_(src); torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record(); torch.cuda.synchronize()
    ms_rt = e0.elapsed_time(e1) / 5
    res["hbm_copy_runtime"] = {"ms": ms_rt, "GB/s": 8 * n / ms_rt / 1e6, "frac_of_nominal": 8 * n / ms_rt / 1e6 / PEAK_HBM_GBS}
    ctx.close()
    return res


def vendor_gemm_comparison(torch, rg):
    """The block's four projection shapes through this library's bf16 GEMM and through torch.matmul (the vendor's GEMM
    library underneath), same process, alternating: context for the achieved TFLOP/s, not part of the path."""
    hidden, mlp = 3072, 12288
    ctx = rg.Context(hidden, 24, 128, mlp, 8704, 16)
    g = torch.Generator(device="cuda"); g.manual_seed(13)

    def t_vendor(fn, reps):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    def t_library(fn, reps):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        rg.regione_profile_enable(ctx, True); rg.regione_profile_read(ctx)
        for _ in range(reps):
            fn()
        us = rg.regione_profile_read(ctx)["gemm"][0] / reps * 1e3
        rg.regione_profile_enable(ctx, False)
        return us

    res = {}
    for m in (820, 1640, 4096, 8704):
        for name, n, k in (("qkv", 3 * hidden, hidden), ("attn_out", hidden, hidden), ("mlp_up", mlp, hidden), ("mlp_down", hidden, mlp)):
            x = torch.randn((m, k), generator=g, device="cuda").to(torch.bfloat16)
            w = (torch.randn((n, k), generator=g, device="cuda") * 0.02).to(torch.bfloat16)
            wp = rg.pack_weight(ctx, w)
            y = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
            reps = 20 if m < 4000 else 6
            tv = tl = 1e30
            for _ in range(2):
                tv = min(tv, t_vendor(lambda: torch.matmul(x, w.t(), out=y), reps))
                tl = min(tl, t_library(lambda: rg.regione_linear(ctx, x, wp, None, m, n, k, rg.ACT_NONE, rg.BF16, y), reps))
            fl = 2.0 * m * n * k
            res[f"{name}_{m}x{n}x{k}"] = {"vendor_us": tv, "library_us": tl, "vendor_TFLOPs": fl / tv * 1e-6, "library_TFLOPs": fl / tl * 1e-6,
                                          "library_over_vendor_time": tl / tv}
            del x, w, wp, y
    # attention of the edited queries over the whole cached sequence, against torch's fused attention
    heads, d, n_c = 24, 128, 8704
    for n_q in (820, 4096):
        q = torch.randn((n_q, heads, d), generator=g, device="cuda").to(torch.bfloat16)
        kc = torch.randn((n_c, heads, d), generator=g, device="cuda").to(torch.bfloat16)
        vc = torch.randn((n_c, heads, d), generator=g, device="cuda").to(torch.bfloat16)
        out = torch.empty_like(q)
        qh, kh, vh = (t.permute(1, 0, 2).unsqueeze(0).contiguous() for t in (q, kc, vc))     # [1, heads, n, d], as the vendor kernel wants it
        fl = 4.0 * n_q * n_c * heads * d
        tv = tl = 1e30
        for _ in range(2):
            tv = min(tv, t_vendor(lambda: torch.nn.functional.scaled_dot_product_attention(qh, kh, vh), 10))
            rg.regione_profile_enable(ctx, True); rg.regione_profile_read(ctx)
            for _ in range(10):
                rg.regione_attn_kvcache(ctx, q, n_q, None, None, 0, kc, vc, n_c, None, 0, heads, d, 0.0, out)
            tl = min(tl, rg.regione_profile_read(ctx)["attention"][0] / 10 * 1e3)
            rg.regione_profile_enable(ctx, False)
        ref = torch.nn.functional.scaled_dot_product_attention(qh, kh, vh)[0].permute(1, 0, 2).float()
        res[f"attention_{n_q}q_{n_c}keys"] = {"vendor_us": tv, "library_us": tl, "vendor_TFLOPs": fl / tv * 1e-6, "library_TFLOPs": fl / tl * 1e-6,
                                              "library_over_vendor_time": tl / tv, "max_abs_diff": float((out.float() - ref).abs().max())}
    ctx.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-membound", action="store_true")
    ap.add_argument("--membound-only", action="store_true",
                    help="only the HBM-bound kernels (partition, gathers, scatters, velocity cache, modulation vectors) on multi-GiB working sets: one JSON line")
    ap.add_argument("--no-fp8", action="store_true", help="skip the secondary measurement of the projections in E4M3")
    ap.add_argument("--no-peaks", action="store_true", help="skip the register-only MFMA loops and the 1 GiB copy that measure the chip's own peaks")
    ap.add_argument("--no-mode-a", action="store_true", help="skip the secondary measurement with the text rows fresh")
    ap.add_argument("--no-profile", action="store_true", help="time the steps without the per-kernel event pairs")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run a plain 1 GiB device copy three times (calibration of the rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--block-extras", action="store_true",
                    help="time the step with query/key normalisation and rotary embedding in the block (no CPU baseline)")
    ap.add_argument("--stack", action="store_true",
                    help="time one storing full step and one region step through 60 double-stream blocks at the large-image sizes")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="only compare the bf16 GEMM of this library with torch.matmul on the block's projection shapes (one JSON line)")
    ap.add_argument("--cfg", action="store_true",
                    help="time the block for the two branches of classifier-free guidance: one batched call against two calls")
    ap.add_argument("--loop", action="store_true",
                    help="instead of the step benchmark: time the whole sampling loop (Algorithm 1, 28 steps) of a 3072-wide editor with "
                         "19 double- and 38 single-stream blocks against 28 plain full steps, and print one JSON line about it")
    ap.add_argument("--loop-guidance", type=float, default=None,
                    help="with --loop: run both guidance branches at every step with this scale (the paper's setting)")
    ap.add_argument("--loop-blocks", type=str, default="19,38", help="double,single block counts for --loop")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); run it with --gpus 1")

    import torch
    if args.vendor_gemm:
        from paper_2510_25590_amd import binding as rg_
        print(json.dumps({"vendor_gemm_comparison": vendor_gemm_comparison(torch, rg_), "data": "synthetic", "dtype": "bf16"}))
        return
    if args.copy_probe:
        a = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": a.numel() * 4, "copy_probe_bytes_written": b.numel() * 4, "copies": 3}))
        return
    from paper_2510_25590_amd import binding as rg
    from paper_2510_25590_amd import step

    rg.lib()   # fails loudly if the HIP library has not been built
    if args.membound_only:
        print(json.dumps({"membound": membound(torch, rg), "data": "synthetic", "dtype": "bf16"}))
        return
    if args.cfg:
        print(json.dumps(cfg_benchmark(args.steps, args.warmup)))
        return
    if args.stack:
        print(json.dumps(stack_benchmark()))
        return
    if args.loop:
        print(json.dumps(loop_benchmark(*[int(v) for v in args.loop_blocks.split(",")], guidance=args.loop_guidance)))
        return
    cfg = step.CONFIG_BLOCK
    if args.block_extras:   # not the headline workload: the same step with the block's query/key extras switched on
        import dataclasses
        cfg = dataclasses.replace(cfg, extras=True, name=cfg.name + "; block extras on: query/key RMS normalisation and rotary embedding")
        args.no_cpu_baseline = True
    wl = step.RegionStepWorkload(cfg)
    for _ in range(args.warmup):
        n = wl.step()
    torch.cuda.synchronize()
    # timed region 1: exactly K steps, no instrumentation -> value / ms_per_step
    t0 = time.perf_counter()
    for _ in range(args.steps):
        n = wl.step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    gemm_flops, attn_flops = wl.flops(n)
    out = {
        "metric": "edited-token DiT block tokens/s", "value": n / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "n_edited": n, "keys_per_query": wl.n_all,
                   "note": "every step includes one stream synchronisation (the edited-token count read back after the partition)"},
    }
    if not args.no_profile:
        # timed region 2: the same K steps with a HIP event pair around every kernel launch group, recorded by the library
        # on its own stream.  The pairs cost ~0.1 ms of gaps per step, which is why they are kept out of region 1.
        rg.regione_profile_enable(wl.ctx, True)
        rg.regione_profile_read(wl.ctx)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            n = wl.step()
        torch.cuda.synchronize()
        ms_profiled = (time.perf_counter() - t0) * 1e3 / args.steps
        prof = rg.regione_profile_read(wl.ctx)
        rg.regione_profile_enable(wl.ctx, False)
        kernels = {k: {"ms_per_step": v[0] / args.steps, "launch_groups_per_step": v[1] / args.steps} for k, v in prof.items()}
        g_ms = prof["gemm"][0] / args.steps
        a_ms = prof["attention"][0] / args.steps
        ach = gemm_flops / (g_ms * 1e-3) / 1e12
        traffic = profiled_traffic() if n == 820 else {}     # the committed counter summaries were taken on the default workload
        out["roofline"] = {"kernel": "gemm_bf16_kernel (QKV, attention output, MLP up, MLP down) + gemm_skinny_kernel (velocity head): 5 launches per step",
                           "bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
                           "traffic": traffic.get("gemm_bf16_kernel"),
                           "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE/WRITE_SIZE at the L2-fabric boundary, from profiles/*_hbm_traffic.txt)",
                           "algorithmic_flops_per_launch": gemm_flops / 5, "avg_launch_ms": prof["gemm"][0] / max(prof["gemm"][1], 1),
                           "measured_in": f"a second timed region of the same {args.steps} steps with HIP event pairs ({ms_profiled:.4f} ms per step there)"}
        out["attention"] = {"achieved": attn_flops / (a_ms * 1e-3) / 1e12, "unit": "TFLOP/s",
                            "frac": attn_flops / (a_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, "ms_per_step": a_ms}
        out["roofline"]["others"] = [{"kernel": "attn_kvcache_kernel + attn_combine_kernel (regione_attn_kvcache inside the block)", "bound": "mfma",
                                      "achieved": out["attention"]["achieved"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": out["attention"]["frac"],
                                      "avg_launch_ms": a_ms, "algorithmic_flops_per_launch": attn_flops, "traffic": traffic.get("attn_kvcache_kernel")}]
        out["gemm_plus_attention_tflops"] = (gemm_flops + attn_flops) / ((g_ms + a_ms) * 1e-3) / 1e12
        out["kernels"] = kernels
    host = wl.host
    gpu_out = None
    if not args.no_cpu_baseline:   # what the step left on the device, for the parity figures beside the oracle's time
        gpu_out = {"mask": wl.mask.cpu().numpy(), "e_index": wl.e_index.cpu().numpy(), "h_e_out": wl.h_e_out.float().cpu().numpy(),
                   "x_next": wl.x_next.float().cpu().numpy()}
        # the same block once more with a float32 residual stream (input and output rows float32), outside every timed region
        h32 = wl.h_e[:n].float().contiguous()
        o32 = torch.empty_like(h32)
        rg.regione_block_forward(wl.ctx, wl.weights, wl.block_type, h32, o32, rg.FP32, n, 0, wl.e_index, cfg.n_txt, wl.k_cache, wl.v_cache,
                                 wl.n_all, rg.FLAG_RETRIEVE)
        gpu_out["h_e_out_f32"] = o32.cpu().numpy()
        del h32, o32
    wl.close()
    del wl
    torch.cuda.empty_cache()
    if not args.no_mode_a:
        # secondary figure: the region step with the text rows recomputed as well (Algorithm 1's input [X^P, X^E]); the
        # headline keeps the text in the cache, as the workload is stated
        import dataclasses
        wa = step.RegionStepWorkload(dataclasses.replace(cfg, text_fresh=True), host=host)
        for _ in range(args.warmup):
            na = wa.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            na = wa.step()
        torch.cuda.synchronize()
        ms_a = (time.perf_counter() - t0) * 1e3 / args.steps
        out["text_fresh"] = {"ms_per_step": ms_a, "edited_tokens_per_s": na / (ms_a * 1e-3), "fresh_rows": cfg.n_txt + na}
        wa.close()
    if not args.no_peaks:
        out["measured_peaks"] = measured_peaks(torch, rg)
    if not args.no_fp8:
        out["fp8_projections"] = fp8_projections(torch, rg, int(n))
        # the same four projections on every row of the sequence (the shapes of a full, cache-storing forward)
        out["fp8_projections_all_rows"] = fp8_projections(torch, rg, int(out["config"]["keys_per_query"]), reps=5)
        out["fp8_block"] = fp8_block(torch, rg, args.steps, args.warmup)
    if not args.no_membound:
        out["membound"] = membound(torch, rg)
        if "roofline" in out:    # one entry per HBM-bound kernel of the path, on the multi-GiB working sets stated in `membound`
            traffic = profiled_traffic()
            names = {"partition": "score_bits_kernel + scan_counts_kernel + write_index_kernel (regione_partition with the score output)",
                     "partition_no_score": "score_bits_kernel + scan_counts_kernel + write_index_kernel (regione_partition)",
                     "gather_latent": "rows_by_index_kernel (regione_gather, 128-byte rows)", "scatter_latent": "rows_by_index_kernel (regione_scatter, 128-byte rows)",
                     "gather_hidden": "rows_by_index_kernel (regione_gather, 6 KiB rows)", "scatter_hidden": "rows_by_index_kernel (regione_scatter, 6 KiB rows)",
                     "velocity_cache_fresh": "velocity_cache_vec_kernel (regione_velocity_cache, fresh step)",
                     "velocity_cache_reuse": "velocity_cache_vec_kernel (regione_velocity_cache, reusing step)"}
            for key, kname in names.items():
                m = out["membound"].get(key)
                if m:
                    out["roofline"]["others"].append({"kernel": kname, "bound": "hbm", "achieved": m["GB/s"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                                      "frac": m["frac_hbm"], "avg_launch_ms": m["ms"], "algorithmic_bytes_per_launch": m["GB/s"] * m["ms"] * 1e6,
                                                      "traffic": traffic.get("membound_" + key)})
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, host, reps=6, gpu=gpu_out)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
