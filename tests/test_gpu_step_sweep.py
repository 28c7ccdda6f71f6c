"""GPU parity at the benchmark's shapes: the whole region-aware step against the oracle's step (bf16-stored and with a
float32 residual stream, all rows), the edited-fraction sweep {5, 20, 50, 100 %} with irregular masks (ragged query
counts).  The oracle evaluates sampled rows at the other sizes.  Outputs of a 3072-wide block are held to the stated
bound on all but 1e-5 of their elements (see gpu_util.assert_close); the tiny configuration runs in float32 at 1e-4."""
import numpy as np
import pytest
import torch

from oracle import regione_oracle as orc
from oracle import step_reference as ref
from paper_2510_25590_amd import binding as rg
from paper_2510_25590_amd import inputs, step
from gpu_util import dev, host, assert_close, block_to_device, TAIL_FRAC, HEAD_TAIL_FRAC, exceedances
from test_gpu_block import _oracle_region_rows, _model

pytestmark = pytest.mark.gpu


F32_TOL = dict(max_abs=1e-4, mean_rel_tol=2e-5)    # the tiny configuration in float32 (float32 context): tight bound, no allowance


def _tol(cfg):
    return F32_TOL if cfg.dtype == "f32" else dict(stored_bf16=True)


def _bits(t):
    return t.view(torch.int32) if t.dtype == torch.float32 else t.view(torch.int16)


@pytest.mark.parametrize("cfg", [step.CONFIG_TINY, step.CONFIG_TINY_BF16], ids=["float32", "bf16"])
def test_tiny_step_matches_oracle_step(cfg):
    wl = step.RegionStepWorkload(cfg)
    n = wl.step()
    torch.cuda.synchronize()
    h = wl.host
    kc, vc = ref.build_cache(h["streams"], cfg.kind, h["h_store"], cfg.n_txt, cfg.heads)
    want = ref.region_step(h["x_t"], h["v_prev"], h["x_ref"], h["h_now"], h["streams"], cfg.kind, h["w_head"], h["b_head"],
                           kc, vc, cfg.n_txt, cfg.heads, cfg.sigma, cfg.eta, cfg.dt)
    assert n == 36 == len(want["e_index"])
    assert np.array_equal(host(wl.mask).astype(np.uint8), want["mask"])
    assert np.array_equal(wl.e_index.cpu().numpy()[:n], want["e_index"])
    assert np.array_equal(wl.u_index.cpu().numpy()[:wl.n_img - n], want["u_index"])
    ma, mr = assert_close(host(wl.h_e_out)[:n], want["h_e_out"], "block output of the step", **_tol(cfg))
    print(f"tiny step ({cfg.dtype}): block output max abs {ma:.3e}, mean rel {mr:.3e}")
    assert_close(host(wl.v_e)[:n], want["v_e"], "velocity of the edited tokens", **(F32_TOL if cfg.dtype == "f32" else {}))
    assert_close(host(wl.c_a)[:n], want["c_a"], "cached velocity", **(F32_TOL if cfg.dtype == "f32" else {}))
    assert_close(host(wl.x_next), want["x_next"], "merged latent", **_tol(cfg))
    assert_close(host(wl.h_next), want["h_next"], "merged hidden state", **_tol(cfg))
    # unedited rows of the merged tensors are bit-identical to the inputs
    u = torch.from_numpy(want["u_index"].astype(np.int64)).cuda()
    assert torch.equal(_bits(wl.x_next[u]), _bits(wl.x_t[u]))
    assert torch.equal(_bits(wl.h_next[u]), _bits(wl.h_now[u]))
    wl.close()


@pytest.mark.parametrize("base", [step.CONFIG_TINY, step.CONFIG_TINY_BF16], ids=["float32", "bf16"])
def test_tiny_step_with_fresh_text_rows_matches_oracle_step(base):
    """Algorithm 1's region step input [X^P, X^E]: the text rows run through the block again with the edited rows."""
    import dataclasses
    cfg = dataclasses.replace(base, text_fresh=True)
    wl = step.RegionStepWorkload(cfg)
    n = wl.step()
    torch.cuda.synchronize()
    h = wl.host
    kc, vc = ref.build_cache(h["streams"], cfg.kind, h["h_store"], cfg.n_txt, cfg.heads)
    want = ref.region_step(h["x_t"], h["v_prev"], h["x_ref"], h["h_now"], h["streams"], cfg.kind, h["w_head"], h["b_head"],
                           kc, vc, cfg.n_txt, cfg.heads, cfg.sigma, cfg.eta, cfg.dt, h_txt=h["h_store"][:cfg.n_txt])
    plain = ref.region_step(h["x_t"], h["v_prev"], h["x_ref"], h["h_now"], h["streams"], cfg.kind, h["w_head"], h["b_head"],
                            *ref.build_cache(h["streams"], cfg.kind, h["h_store"], cfg.n_txt, cfg.heads), cfg.n_txt, cfg.heads, cfg.sigma, cfg.eta, cfg.dt)
    assert n == 36
    assert_close(host(wl.h_e_out)[:n], want["h_e_out"], "block output of the step, text rows fresh", **_tol(cfg))
    assert_close(host(wl.x_next), want["x_next"], "merged latent, text rows fresh", **_tol(cfg))
    # the text rows come from the same hidden state the cache was stored from, so both forms agree here
    assert np.allclose(want["h_e_out"], plain["h_e_out"], atol=1e-9)
    wl.close()


def test_benchmark_step_matches_oracle_step():
    """The launch configuration bench.py times (3072 wide, 820 edited tokens, 8704 keys), full oracle step."""
    cfg = step.CONFIG_BLOCK
    wl = step.RegionStepWorkload(cfg)
    n = wl.step()
    n2 = wl.step()          # a second pass over the same buffers gives the same result (the step is idempotent)
    torch.cuda.synchronize()
    h = wl.host
    kc, vc = ref.build_cache(h["streams"], cfg.kind, h["h_store"], cfg.n_txt, cfg.heads)
    want = ref.region_step(h["x_t"], h["v_prev"], h["x_ref"], h["h_now"], h["streams"], cfg.kind, h["w_head"], h["b_head"],
                           kc, vc, cfg.n_txt, cfg.heads, cfg.sigma, cfg.eta, cfg.dt)
    assert n == n2 == len(want["e_index"])
    assert np.array_equal(host(wl.mask).astype(np.uint8), want["mask"])
    assert np.array_equal(wl.e_index.cpu().numpy()[:n], want["e_index"])
    ma, mr = assert_close(host(wl.h_e_out)[:n], want["h_e_out"], "block output of the step", stored_bf16=True, tail_frac=TAIL_FRAC)
    n_out, frac, _ = exceedances(host(wl.h_e_out)[:n], want["h_e_out"], stored_bf16=True)
    print(f"benchmark step parity (bf16-stored): n_edited {n}, block output max abs {ma:.3e}, mean rel {mr:.3e}, {n_out} elements ({frac:.1e}) beyond 2e-2 + storage half-ulp")
    # the same block with a float32 residual stream (no storage rounding in the way), every row against the oracle
    h_in = torch.from_numpy(h["h_now"][want["e_index"]]).cuda()
    o32 = torch.empty_like(h_in)
    rg.regione_block_forward(wl.ctx, wl.weights, wl.block_type, h_in, o32, rg.FP32, n, 0, wl.e_index, cfg.n_txt, wl.k_cache, wl.v_cache, wl.n_all, rg.FLAG_RETRIEVE)
    ma32, mr32 = assert_close(host(o32), want["h_e_out"], "block output, float32 residual stream, all rows", tail_frac=TAIL_FRAC)
    n32, f32, _ = exceedances(host(o32), want["h_e_out"])
    print(f"benchmark step parity (float32 residual): max abs {ma32:.3e}, mean rel {mr32:.3e}, {n32} of {o32.numel()} elements ({f32:.1e}) beyond 2e-2")
    # the velocity head multiplies the (bf16-stored) block output by a 3072-long weight row: teacher-forced on the
    # library's own block output the head must be tight; against the oracle's exact chain it carries the block's error
    hv = host(wl.h_e_out)[:n]
    assert_close(host(wl.v_e)[:n], orc.linear(hv, h["w_head"], h["b_head"]), "velocity head on the library's block output", stored_bf16=True)
    assert_close(host(wl.v_e)[:n], want["v_e"], "velocity of the edited tokens (whole chain)", stored_bf16=True, tail_frac=HEAD_TAIL_FRAC)
    assert_close(host(wl.x_next), want["x_next"], "merged latent", stored_bf16=True)
    assert_close(host(wl.h_next), want["h_next"], "merged hidden state", stored_bf16=True, tail_frac=TAIL_FRAC)
    wl.close()


@pytest.mark.parametrize("n_edited", [205, 2048, 4096])
@pytest.mark.parametrize("h_dtype", ["bf16", "f32"])
def test_fraction_sweep_blob_masks(n_edited, h_dtype):
    """5 %, 50 % and 100 % of a 64x64 image edited, irregular masks through the partition kernel, double-stream block;
    the oracle evaluates sampled rows (20 % is covered by the step test above)."""
    if h_dtype == "f32" and n_edited != 2048:
        pytest.skip("one size is enough for the float32 residual stream")
    hidden, heads, d, mlp = 3072, 24, 128, 12288
    n_txt, n_img = 512, 4096
    n_all = n_txt + 2 * n_img
    streams, rng = _model(inputs.workload_seed(3, n_edited), "double", hidden, mlp)
    want_mask = inputs.blob_mask(rng, 64, 64, n_edited)
    x_t, v_prev, x_ref = inputs.latents_for_mask(rng, want_mask, 64, 0.7, "bf16")
    h_store = inputs.hidden_states(rng, n_all, hidden)
    ctx = rg.Context(hidden, heads, d, mlp, n_all, n_img)
    bw, keep = block_to_device(streams, "double", ctx)
    # partition on the device decides the rows
    e_idx = torch.empty(n_img, dtype=torch.int32, device="cuda"); u_idx = torch.empty_like(e_idx)
    mask = torch.empty(n_img, dtype=torch.uint8, device="cuda"); cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    n = rg.regione_partition(ctx, dev(x_t, "bf16"), dev(v_prev, "bf16"), dev(x_ref, "bf16"), n_img, 64, rg.BF16, 0.7, 0.9, None, mask, e_idx, u_idx, cnt)
    assert n == n_edited
    e = np.nonzero(want_mask)[0].astype(np.int32)
    assert np.array_equal(e_idx.cpu().numpy()[:n], e)
    rows = n_txt + e
    h_now = inputs.bf16_round((h_store[rows] + 0.05 * rng.standard_normal((n, hidden))).astype(np.float32))
    kc = torch.zeros((n_all, heads, d), dtype=torch.bfloat16, device="cuda"); vc = torch.zeros_like(kc)
    full = torch.empty((n_all, hidden), dtype=torch.bfloat16, device="cuda")
    rg.regione_block_forward(ctx, bw, rg.BLOCK_DOUBLE, dev(h_store, "bf16"), full, rg.BF16, n_all, n_txt,
                             torch.arange(n_all, dtype=torch.int32, device="cuda"), 0, kc, vc, n_all, rg.FLAG_STORE)
    tdt = torch.bfloat16 if h_dtype == "bf16" else torch.float32
    o = torch.empty((n, hidden), dtype=tdt, device="cuda")
    rg.regione_block_forward(ctx, bw, rg.BLOCK_DOUBLE, dev(h_now, h_dtype), o, rg.BF16 if h_dtype == "bf16" else rg.FP32, n, 0,
                             e_idx, n_txt, kc, vc, n_all, rg.FLAG_RETRIEVE)
    kc_o, vc_o = ref.build_cache(streams, "double", h_store, n_txt, heads)
    sample = np.sort(rng.choice(n, size=24, replace=False))
    sample[:2] = [0, n - 1]
    want = _oracle_region_rows(streams, "double", h_now, rows, kc_o, vc_o, heads, sample)
    ma, mr = assert_close(host(o)[sample], want, f"region forward with {n} edited tokens ({h_dtype} residual stream)", stored_bf16=(h_dtype == "bf16"),
                          tail_frac=TAIL_FRAC)   # 3072-wide block output: the bound is 5 sigma of the bf16 arithmetic error
    print(f"n_edited {n} ({h_dtype}): max abs {ma:.3e}, mean rel {mr:.3e}")
    ctx.close()


def test_large_image_region_forward_sampled():
    """The large-image configuration: 96x96 image + 9216 reference + 1024 text tokens (19456 keys), 1382 edited tokens of a
    blob, one double-stream block at 3072 wide; the oracle builds the whole cache and evaluates sampled edited rows."""
    hidden, heads, d, mlp = 3072, 24, 128, 12288
    n_txt, grid, n_edited = 1024, 96, 1382
    n_img = grid * grid
    n_all = n_txt + 2 * n_img
    streams, rng = _model(inputs.workload_seed(5, 2), "double", hidden, mlp)
    want_mask = inputs.blob_mask(rng, grid, grid, n_edited)
    e = np.nonzero(want_mask)[0].astype(np.int32)
    rows = n_txt + e
    h_store = inputs.hidden_states(rng, n_all, hidden)
    h_now = inputs.bf16_round((h_store[rows] + 0.05 * rng.standard_normal((n_edited, hidden))).astype(np.float32))
    ctx = rg.Context(hidden, heads, d, mlp, n_all, n_img)
    bw, keep = block_to_device(streams, "double", ctx)
    kc = torch.zeros((n_all, heads, d), dtype=torch.bfloat16, device="cuda"); vc = torch.zeros_like(kc)
    full = torch.empty((n_all, hidden), dtype=torch.bfloat16, device="cuda")
    rg.regione_block_forward(ctx, bw, rg.BLOCK_DOUBLE, dev(h_store, "bf16"), full, rg.BF16, n_all, n_txt,
                             torch.arange(n_all, dtype=torch.int32, device="cuda"), 0, kc, vc, n_all, rg.FLAG_STORE)
    o = torch.empty((n_edited, hidden), dtype=torch.bfloat16, device="cuda")
    rg.regione_block_forward(ctx, bw, rg.BLOCK_DOUBLE, dev(h_now, "bf16"), o, rg.BF16, n_edited, 0, torch.from_numpy(e).cuda(), n_txt,
                             kc, vc, n_all, rg.FLAG_RETRIEVE)
    kc_o, vc_o = ref.build_cache(streams, "double", h_store, n_txt, heads)
    sample = np.sort(rng.choice(n_edited, size=24, replace=False))
    sample[:2] = [0, n_edited - 1]
    want = _oracle_region_rows(streams, "double", h_now, rows, kc_o, vc_o, heads, sample)
    ma, mr = assert_close(host(o)[sample], want, "region forward at the large-image sizes (sampled rows)", stored_bf16=True, tail_frac=TAIL_FRAC)
    print(f"large image: n_edited {n_edited}, {n_all} keys: max abs {ma:.3e}, mean rel {mr:.3e}")
    ctx.close()
