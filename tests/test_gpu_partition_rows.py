"""GPU parity: adaptive region partition, gather/scatter and the velocity cache against the oracle."""
import numpy as np
import pytest
import torch

from oracle import regione_oracle as orc
from paper_2510_25590_amd import binding as rg
from paper_2510_25590_amd import inputs
from gpu_util import dev, host, assert_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = rg.Context(256, 4, 64, 1024, 64, 1 << 21)
    yield c
    c.close()


def run_partition(ctx, x_t, v, ref, sigma, eta, dtype):
    n, c = x_t.shape
    dx, dv, dr = dev(x_t, dtype), dev(v, dtype), dev(ref, dtype)
    score = torch.full((max(n, 1),), -7.0, device="cuda")
    mask = torch.full((max(n, 1),), 9, dtype=torch.uint8, device="cuda")
    e = torch.full((max(n, 1),), -1, dtype=torch.int32, device="cuda")
    u = torch.full((max(n, 1),), -1, dtype=torch.int32, device="cuda")
    cnt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    n_e = rg.regione_partition(ctx, dx, dv, dr, n, c, rg.BF16 if dtype == "bf16" else rg.FP32, sigma, eta, score, mask, e, u, cnt)
    assert n_e == int(cnt.item())
    return n_e, score.cpu().numpy()[:n], mask.cpu().numpy()[:n], e.cpu().numpy(), u.cpu().numpy()


def check_partition(ctx, x_t, v, ref, sigma, eta, dtype):
    n = x_t.shape[0]
    s_o, m_o, e_o, u_o = orc.partition(x_t, v, ref, sigma, eta)
    n_e, s, m, e, u = run_partition(ctx, x_t, v, ref, sigma, eta, dtype)
    assert n_e == len(e_o)
    assert np.array_equal(m, m_o)
    assert np.array_equal(e[:n_e], e_o) and np.array_equal(u[:n - n_e], u_o)
    assert np.all(e[n_e:] == -1) and np.all(u[n - n_e:] == -1)      # nothing written past the counts
    assert np.max(np.abs(s - s_o)) <= 2e-7 if n else True
    return n_e


def test_config1_fp32_returns_the_rectangle(ctx):
    rng = np.random.default_rng(inputs.workload_seed(1))
    want = inputs.rect_mask(rng, 16, 16, 6, 6)
    x_t, v, ref = inputs.latents_for_mask(rng, want, 64, 0.7, "f32")
    assert check_partition(ctx, x_t, v, ref, 0.7, 0.9, "f32") == 36


@pytest.mark.parametrize("n_e", [205, 819, 2048, 4096, 0])
def test_config3_bf16_blob_masks(ctx, n_e):
    rng = np.random.default_rng(inputs.workload_seed(3, n_e))
    want = inputs.blob_mask(rng, 64, 64, n_e)
    x_t, v, ref = inputs.latents_for_mask(rng, want, 64, 0.7, "bf16")
    assert check_partition(ctx, x_t, v, ref, 0.7, 0.9, "bf16") == n_e


@pytest.mark.parametrize("n", [0, 1, 31, 32, 33, 63, 64, 65, 255, 256, 257, 1000])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ragged_sizes(ctx, n, dtype):
    rng = np.random.default_rng(100 + n)
    want = rng.random(n) < 0.37
    x_t, v, ref = inputs.latents_for_mask(rng, want, 64, 0.6, dtype)
    check_partition(ctx, x_t, v, ref, 0.6, 0.9, dtype)


def test_many_blocks_take_the_scan_kernel_path():
    """More than 1024 blocks of tokens: the per-block counts go through the separate scan kernel (with fewer blocks the
    index kernel adds them up itself).  40 000 tokens of 64 channels are 1250 blocks; the clean-up at 128x128x17 cells
    is 1088 blocks."""
    n = 40000
    rng = np.random.default_rng(77)
    want = rng.random(n) < 0.2
    x_t, v, ref = inputs.latents_for_mask(rng, want, 64, 0.6, "bf16")
    big = rg.Context(256, 4, 64, 1024, 16, 128 * 128 * 17)
    assert check_partition(big, x_t, v, ref, 0.6, 0.9, "bf16") == int(want.sum())
    cells, n_images = 128 * 128, 17
    masks = [rng.random(cells) < 0.4 for _ in range(n_images)]
    want_clean = np.concatenate([orc.mask_cleanup(m.astype(np.uint8), 128, 128) for m in masks[:2]])
    d_in = torch.from_numpy(np.concatenate(masks).astype(np.uint8)).cuda()
    e = torch.empty(cells * n_images, dtype=torch.int32, device="cuda"); u = torch.empty_like(e)
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    n_e = rg.regione_mask_cleanup(big, d_in, 128, 128, n_images, d_in, e, u, cnt)
    got = d_in.cpu().numpy()
    assert np.array_equal(got[:2 * cells], want_clean)            # the oracle's loops on two of the images
    assert n_e == int(got.sum()) == int(cnt.item())
    assert np.array_equal(e.cpu().numpy()[:n_e], np.nonzero(got)[0].astype(np.int32))
    assert np.array_equal(u.cpu().numpy()[:cells * n_images - n_e], np.nonzero(got == 0)[0].astype(np.int32))
    big.close()


@pytest.mark.parametrize("c", [8, 16, 48, 128, 512, 1024, 7, 20])
def test_channel_counts(ctx, c):
    rng = np.random.default_rng(200 + c)
    want = rng.random(300) < 0.5
    for dtype in ("bf16", "f32"):
        x_t, v, ref = inputs.latents_for_mask(rng, want, c, 0.5, dtype)
        # low channel counts leave no margin around a 0.9 threshold; use the oracle's own scores to pick a safe eta
        s = orc.partition(x_t, v, ref, 0.5, 0.0)[0]
        srt = np.sort(s)
        gaps = np.diff(srt)
        k = int(np.argmax(gaps))
        eta = float((srt[k] + srt[k + 1]) / 2)
        check_partition(ctx, x_t, v, ref, 0.5, eta, dtype)


def test_wave_boundary_patterns(ctx):
    n = 640
    rng = np.random.default_rng(300)
    for pattern in ("none", "all", "lane0", "lane63", "alternate", "one_wave_full"):
        want = np.zeros(n, dtype=bool)
        if pattern == "all": want[:] = True
        if pattern == "lane0": want[::64] = True
        if pattern == "lane63": want[63::64] = True
        if pattern == "alternate": want[::2] = True
        if pattern == "one_wave_full": want[128:192] = True
        x_t, v, ref = inputs.latents_for_mask(rng, want, 64, 0.7, "bf16")
        assert check_partition(ctx, x_t, v, ref, 0.7, 0.9, "bf16") == int(want.sum())


def test_integer_inputs_decide_exactly_at_the_threshold(ctx):
    # small integers: every product and sum is exact in both implementations, so scores on the
    # threshold itself must fall on the same side (== eta -> edited)
    ref = np.array([[3, 4] + [0] * 6, [3, 4] + [0] * 6, [1, 0] + [0] * 6, [0] * 8], dtype=np.float32)
    xhat = np.array([[4, 3] + [0] * 6, [3, 4] + [0] * 6, [0, 1] + [0] * 6, [1] * 8], dtype=np.float32)
    v = np.ones_like(ref)
    x_t = xhat + 0.5 * v
    eta = float(np.float32(24.0 / 25.0))
    for dtype in ("f32", "bf16"):
        n_e, s, m, e, u = run_partition(ctx, x_t, v, ref, 0.5, eta, dtype)
        assert s[0] == np.float32(0.96) and m.tolist() == [1, 0, 1, 1]
        check_partition(ctx, x_t, v, ref, 0.5, eta, dtype)


def test_large_batch_of_images(ctx):
    # 256 images of 64x64 tokens as one token list: several passes per block and many blocks
    rng = np.random.default_rng(400)
    n = 256 * 4096
    want = rng.random(n) < 0.2
    x_t, v, ref = inputs.latents_for_mask(rng, want, 64, 0.7, "bf16")
    s_o = orc.cosine_scores(orc.one_step_estimate_f32(x_t, v, 0.7), ref)
    m_o = orc.threshold_mask(s_o, 0.9)
    assert np.array_equal(m_o.astype(bool), want)
    n_e, s, m, e, u = run_partition(ctx, x_t, v, ref, 0.7, 0.9, "bf16")
    assert n_e == int(want.sum())
    assert np.array_equal(m, m_o)
    assert np.array_equal(e[:n_e], np.nonzero(want)[0]) and np.array_equal(u[:n - n_e], np.nonzero(~want)[0])


@pytest.mark.parametrize("row_elems,dtype", [(64, "bf16"), (3072, "bf16"), (64, "f32"), (5, "bf16"), (3, "f32"), (12, "bf16")])
def test_gather_scatter_bit_exact(ctx, row_elems, dtype):
    rng = np.random.default_rng(500 + row_elems)
    n = 777
    x = inputs.bf16_round(rng.standard_normal((n, row_elems)).astype(np.float32)) if dtype == "bf16" else rng.standard_normal((n, row_elems)).astype(np.float32)
    mask = rng.random(n) < 0.3
    e_o, u_o = orc.compact(mask.astype(np.uint8))
    code = rg.BF16 if dtype == "bf16" else rg.FP32
    dx = dev(x, dtype)
    idx = torch.from_numpy(np.concatenate([e_o, -np.ones(n - len(e_o), dtype=np.int32)])).cuda()   # tail must never be read
    cnt = torch.tensor([len(e_o)], dtype=torch.int32, device="cuda")
    g = torch.zeros((n, row_elems), dtype=dx.dtype, device="cuda")
    rg.regione_gather(ctx, dx, row_elems, code, idx, cnt, n, g)
    assert np.array_equal(host(g)[:len(e_o)], orc.gather(x, e_o))
    assert np.all(host(g)[len(e_o):] == 0)
    # scatter(gather(x)) leaves the unedited rows bit-identical, edited rows take the new values
    y = dx.clone()
    new = (g.float() + 1.0).to(dx.dtype)
    rg.regione_scatter(ctx, y, row_elems, code, idx, cnt, n, new)
    want = orc.scatter(x.copy(), e_o, host(new)[:len(e_o)])
    bits = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(y.view(bits)[~torch.from_numpy(mask).cuda()], dx.view(bits)[~torch.from_numpy(mask).cuda()])
    assert np.array_equal(host(y), want)
    # host-side count (n_dev null) and identity / permutation index
    perm = torch.from_numpy(rng.permutation(n).astype(np.int32)).cuda()
    g2 = torch.empty_like(dx)
    rg.regione_gather(ctx, dx, row_elems, code, perm, None, n, g2)
    z = torch.zeros_like(dx)
    rg.regione_scatter(ctx, z, row_elems, code, perm, None, n, g2)
    assert torch.equal(z.view(bits), dx.view(bits))
    # empty list is a no-op
    zero = torch.zeros(1, dtype=torch.int32, device="cuda")
    before = y.clone()
    rg.regione_scatter(ctx, y, row_elems, code, idx, zero, n, new)
    assert torch.equal(before.view(bits), y.view(bits))


@pytest.mark.parametrize("c", [64, 20])      # 20 channels: rows that do not split into 16-byte pieces take the element-wise kernel
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_velocity_cache_matches_oracle(ctx, dtype, c):
    rng = np.random.default_rng(600)
    n = 819
    rnd = (lambda a: inputs.bf16_round(a)) if dtype == "bf16" else (lambda a: a)
    v = rnd(rng.standard_normal((n, c)).astype(np.float32))
    ca0 = rnd(rng.standard_normal((n, c)).astype(np.float32))
    x = rnd(rng.standard_normal((n, c)).astype(np.float32))
    code = rg.BF16 if dtype == "bf16" else rg.FP32
    sb = dtype == "bf16"
    tol = dict(max_abs=2e-2, stored_bf16=True) if sb else dict(max_abs=1e-6, mean_rel_tol=1e-6)
    cnt = torch.tensor([n - 19], dtype=torch.int32, device="cuda")
    live = n - 19
    # fresh step
    dca, dx, dvo = dev(ca0, dtype), dev(x, dtype), dev(np.zeros((n, c), np.float32), dtype)
    rg.regione_velocity_cache(ctx, False, 1.0, 1 / 28, dev(v, dtype), dca, dvo, dx, cnt, n, c, code)
    vu, cn, xn = orc.velocity_cache_apply(False, 1.0, 1 / 28, v[:live], ca0[:live], x[:live])
    assert np.array_equal(host(dca)[:live], v[:live]) and np.array_equal(host(dca)[live:], ca0[live:])
    assert np.array_equal(host(dvo)[:live], v[:live])
    assert_close(host(dx)[:live], xn, "x after a fresh step", **tol)
    assert np.array_equal(host(dx)[live:], x[live:])
    # reuse step
    dca, dx = dev(ca0, dtype), dev(x, dtype)
    f = float(np.float32((27 / 28) ** 2))
    rg.regione_velocity_cache(ctx, True, f, 1 / 28, None, dca, dvo, dx, cnt, n, c, code)
    vu, cn, xn = orc.velocity_cache_apply(True, f, 1 / 28, None, ca0[:live], x[:live])
    assert np.array_equal(host(dca), ca0)
    assert_close(host(dvo)[:live], vu, "reused velocity", **tol)
    assert_close(host(dx)[:live], xn, "x after a reuse step", **tol)
    with pytest.raises(rg.RegionEError):
        rg.regione_velocity_cache(ctx, False, 1.0, 0.1, None, dca, None, dx, cnt, n, c, code)


@pytest.mark.parametrize("c", [64, 20])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_euler_rows_in_place_equals_gather_step_scatter(ctx, dtype, c):
    """The unedited rows' jump (Eq.5) done in place on the full latent: the oracle's gather, Euler step and merge."""
    rng = np.random.default_rng(610 + c)
    n_rows = 4096
    rnd = (lambda a: inputs.bf16_round(a)) if dtype == "bf16" else (lambda a: a)
    x = rnd(rng.standard_normal((n_rows, c)).astype(np.float32))
    v = rnd(rng.standard_normal((n_rows, c)).astype(np.float32))
    u = np.sort(rng.choice(n_rows, size=3277, replace=False)).astype(np.int32)      # 80 % of the rows, as unedited rows are
    live = len(u) - 5
    code = rg.BF16 if dtype == "bf16" else rg.FP32
    dx = dev(x, dtype)
    cnt = torch.tensor([live], dtype=torch.int32, device="cuda")
    dt = 10.0 / 28.0
    rg.regione_euler_rows(ctx, dx, dev(v, dtype), torch.from_numpy(u).cuda(), cnt, len(u), c, code, dt)
    want = orc.scatter(x.astype(np.float64).copy(), u[:live], orc.euler_step(orc.gather(x, u[:live]), orc.gather(v, u[:live]), dt))
    got = host(dx)
    tol = dict(max_abs=2e-2, stored_bf16=True) if dtype == "bf16" else dict(max_abs=1e-6, mean_rel_tol=1e-6)
    assert_close(got[u[:live]], want[u[:live]], "rows after the jump", **tol)
    rest = np.setdiff1d(np.arange(n_rows), u[:live])
    assert np.array_equal(got[rest], x[rest])           # rows that are not listed (or lie past the count) are bit-identical
    # the same arithmetic as the velocity-cache kernel's reusing form with factor 1 on gathered rows: bit for bit
    xg, vg = dev(x[u[:live]], dtype), dev(v[u[:live]], dtype)
    rg.regione_velocity_cache(ctx, True, 1.0, dt, None, vg, None, xg, None, live, c, code)
    assert np.array_equal(host(xg), got[u[:live]])
    with pytest.raises(rg.RegionEError):
        rg.regione_euler_rows(ctx, dx, dx, torch.from_numpy(u).cuda(), cnt, len(u), c, code, dt)


@pytest.mark.parametrize("elems_a,elems_b,dt_a,dt_b", [(3072, 64, "bf16", "bf16"), (256, 64, "f32", "f32"), (3072, 64, "bf16", "f32"), (40, 20, "bf16", "bf16")])
def test_pair_gather_and_scatter_equal_the_single_calls(ctx, elems_a, elems_b, dt_a, dt_b):
    rng = np.random.default_rng(620 + elems_a)
    n_rows, n = 2000, 377
    idx = np.sort(rng.choice(n_rows, size=n, replace=False)).astype(np.int32)
    a = rng.standard_normal((n_rows, elems_a)).astype(np.float32); b = rng.standard_normal((n_rows, elems_b)).astype(np.float32)
    da, db = dev(a, dt_a), dev(b, dt_b)
    ca, cb = (rg.BF16 if dt_a == "bf16" else rg.FP32), (rg.BF16 if dt_b == "bf16" else rg.FP32)
    didx = torch.from_numpy(idx).cuda()
    cnt = torch.tensor([n - 7], dtype=torch.int32, device="cuda")
    ga, gb = torch.zeros((n, elems_a), dtype=da.dtype, device="cuda"), torch.zeros((n, elems_b), dtype=db.dtype, device="cuda")
    ga1, gb1 = torch.zeros_like(ga), torch.zeros_like(gb)
    rg.regione_gather_pair(ctx, da, elems_a, ca, ga, db, elems_b, cb, gb, didx, cnt, n)
    rg.regione_gather(ctx, da, elems_a, ca, didx, cnt, n, ga1); rg.regione_gather(ctx, db, elems_b, cb, didx, cnt, n, gb1)
    assert torch.equal(ga, ga1) and torch.equal(gb, gb1)
    assert torch.equal(ga[:n - 7], da[didx[:n - 7].long()]) and bool((ga[n - 7:] == 0).all())
    fa, fb = torch.zeros_like(da), torch.zeros_like(db)
    fa1, fb1 = torch.zeros_like(da), torch.zeros_like(db)
    rg.regione_scatter_pair(ctx, fa, elems_a, ca, ga, fb, elems_b, cb, gb, didx, cnt, n)
    rg.regione_scatter(ctx, fa1, elems_a, ca, didx, cnt, n, ga); rg.regione_scatter(ctx, fb1, elems_b, cb, didx, cnt, n, gb)
    assert torch.equal(fa, fa1) and torch.equal(fb, fb1)
    # nothing to move: not an error
    rg.regione_gather_pair(ctx, da, elems_a, ca, ga, db, elems_b, cb, gb, didx, cnt, 0)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("n", [1, 36, 820])
def test_velocity_head_equals_linear_cache_and_scatter(dtype, n):
    """The fused head of a fresh region step against the three calls it stands for (bit for bit), and against the oracle."""
    hidden, c, n_rows = 3072, 64, 4096
    rng = np.random.default_rng(630 + n)
    ctx2 = rg.Context(hidden, 24, 128, 12288, 1024, 16)
    h = inputs.bf16_round(rng.standard_normal((n, hidden)).astype(np.float32))
    w = inputs.bf16_round((0.02 * rng.standard_normal((c, hidden))).astype(np.float32))
    b = (0.02 * rng.standard_normal(c)).astype(np.float32)
    rnd = inputs.bf16_round if dtype == "bf16" else (lambda a: a)
    x_e = rnd(rng.standard_normal((n, c)).astype(np.float32)); x_full = rnd(rng.standard_normal((n_rows, c)).astype(np.float32))
    idx = np.sort(rng.choice(n_rows, size=n, replace=False)).astype(np.int32)
    code = rg.BF16 if dtype == "bf16" else rg.FP32
    wp = rg.pack_weight(ctx2, dev(w, "bf16")); db = torch.from_numpy(b).cuda(); dh = dev(h, "bf16"); didx = torch.from_numpy(idx).cuda()
    dt = 1.0 / 28.0
    # fused
    v1, ca1, xe1, xf1 = dev(np.zeros((n, c), np.float32), dtype), dev(np.ones((n, c), np.float32), dtype), dev(x_e, dtype), dev(x_full, dtype)
    rg.regione_velocity_head(ctx2, dh, wp, db, n, c, hidden, dt, v1, ca1, xe1, xf1, didx, code)
    # the three calls
    v2, ca2, xe2, xf2 = dev(np.zeros((n, c), np.float32), dtype), dev(np.ones((n, c), np.float32), dtype), dev(x_e, dtype), dev(x_full, dtype)
    rg.regione_linear(ctx2, dh, wp, db, n, c, hidden, rg.ACT_NONE, code, v2)
    rg.regione_velocity_cache(ctx2, False, 1.0, dt, v2, ca2, None, xe2, None, n, c, code)
    rg.regione_scatter(ctx2, xf2, c, code, didx, None, n, xe2)
    for name, p, q in (("v", v1, v2), ("c_a", ca1, ca2), ("x_e", xe1, xe2), ("x_full", xf1, xf2)):
        assert torch.equal(p, q), name
    # the oracle: linear, fresh cache step, Euler, merge
    v_o = orc.linear(h, w, b)
    _, ca_o, xe_o = orc.velocity_cache_apply(False, 1.0, dt, v_o, None, x_e)
    xf_o = orc.scatter(x_full.astype(np.float64).copy(), idx, xe_o)
    tol = dict(stored_bf16=True) if dtype == "bf16" else dict(max_abs=2e-3, mean_rel_tol=1e-4)   # float32 sums of exact bf16 products over 3072 terms
    assert_close(host(v1), v_o, "velocity", **tol)
    assert_close(host(xf1), xf_o, "merged latent", **tol)
    rest = np.setdiff1d(np.arange(n_rows), idx)
    assert np.array_equal(host(xf1)[rest], x_full[rest])
    # without the optional outputs
    ca3, xe3 = dev(np.ones((n, c), np.float32), dtype), dev(x_e, dtype)
    rg.regione_velocity_head(ctx2, dh, wp, db, n, c, hidden, dt, None, ca3, xe3, None, None, code)
    assert torch.equal(ca3, ca1) and torch.equal(xe3, xe1)
    # a forced plan of the general GEMM kernels takes the other road (K splits, the step in their merge kernel): same
    # three calls bit for bit there as well, and the oracle's result
    rg.regione_tune_gemm(ctx2, 1, 4)
    try:
        v4, ca4, xe4, xf4 = dev(np.zeros((n, c), np.float32), dtype), dev(np.ones((n, c), np.float32), dtype), dev(x_e, dtype), dev(x_full, dtype)
        rg.regione_velocity_head(ctx2, dh, wp, db, n, c, hidden, dt, v4, ca4, xe4, xf4, didx, code)
        v5, ca5, xe5 = dev(np.zeros((n, c), np.float32), dtype), dev(np.ones((n, c), np.float32), dtype), dev(x_e, dtype)
        rg.regione_linear(ctx2, dh, wp, db, n, c, hidden, rg.ACT_NONE, code, v5)
        rg.regione_velocity_cache(ctx2, False, 1.0, dt, v5, ca5, None, xe5, None, n, c, code)
        assert torch.equal(v4, v5) and torch.equal(ca4, ca5) and torch.equal(xe4, xe5)
        assert_close(host(xf4), xf_o, "merged latent, general kernels", **tol)
    finally:
        rg.regione_tune_gemm(ctx2, 0, 0)
    ctx2.close()


# ---------------------------------------------------------------- morphological clean-up of the partition


@pytest.mark.parametrize("gh, gw, n_images, density", [(1, 1, 1, 0.5), (1, 9, 1, 0.5), (7, 1, 2, 0.4), (16, 16, 1, 0.15), (64, 64, 1, 0.2),
                                                        (64, 64, 3, 0.6), (96, 96, 1, 0.9), (37, 53, 2, 0.3), (128, 128, 1, 0.5)])
def test_mask_cleanup_matches_oracle(gh, gw, n_images, density):
    rng = np.random.default_rng(gh * 1000 + gw * 10 + n_images)
    cells = gh * gw
    # blobs plus salt-and-pepper noise: what the clean-up is for
    masks = []
    for _ in range(n_images):
        m = inputs.blob_mask(rng, gh, gw, int(density * cells)) if min(gh, gw) >= 4 else (rng.random(cells) < density)
        flip = rng.random(cells) < 0.03
        masks.append(np.logical_xor(m, flip))
    mask = np.concatenate(masks).astype(np.uint8)
    want = np.concatenate([orc.mask_cleanup(m.astype(np.uint8), gh, gw) for m in masks])
    e_want, u_want = orc.compact(want)
    n = cells * n_images
    ctx = rg.Context(256, 4, 64, 1024, 16, n)
    d_in = torch.from_numpy(mask).cuda()
    d_out = torch.empty_like(d_in)
    e = torch.full((n,), -7, dtype=torch.int32, device="cuda"); u = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    n_e = rg.regione_mask_cleanup(ctx, d_in, gh, gw, n_images, d_out, e, u, cnt)
    assert n_e == len(e_want) == int(cnt.item())
    assert np.array_equal(d_out.cpu().numpy(), want)
    assert np.array_equal(e.cpu().numpy()[:n_e], e_want)
    assert np.array_equal(u.cpu().numpy()[:n - n_e], u_want)
    assert (e.cpu().numpy()[n_e:] == -7).all() and (u.cpu().numpy()[n - n_e:] == -7).all()   # nothing written past the lists
    # in place, and applying it twice changes nothing (opening then closing is an idempotent filter)
    n_e2 = rg.regione_mask_cleanup(ctx, d_out, gh, gw, n_images, d_out, e, u, cnt)
    assert n_e2 == n_e and np.array_equal(d_out.cpu().numpy(), want)
    ctx.close()


def test_mask_cleanup_degenerate_and_errors():
    ctx = rg.Context(256, 4, 64, 1024, 16, 128 * 128)
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    for fill in (0, 1):
        m = torch.full((64,), fill, dtype=torch.uint8, device="cuda")
        e = torch.empty(64, dtype=torch.int32, device="cuda"); u = torch.empty_like(e)
        assert rg.regione_mask_cleanup(ctx, m, 8, 8, 1, m, e, u, cnt) == 64 * fill
        assert (m.cpu().numpy() == fill).all()
    assert rg.regione_mask_cleanup(ctx, None, 8, 8, 0, None, None, None, cnt) == 0    # no image: count 0, nothing touched
    with pytest.raises(rg.RegionEError):
        rg.regione_mask_cleanup(ctx, m, 129, 128, 1, m, e, u, cnt)                    # more cells than a workgroup's LDS holds
    with pytest.raises(rg.RegionEError):
        rg.regione_mask_cleanup(ctx, m, 0, 8, 1, m, e, u, cnt)
    ctx.close()


@pytest.mark.parametrize("n", [0, 1, 7, 8, 4096 * 64, 4096 * 64 + 3, 40_000_003])
def test_cast_between_storage_types(ctx, n):
    rng = np.random.default_rng(900 + n)
    x = (rng.standard_normal(n) * 3.0).astype(np.float32)
    src = torch.from_numpy(x).cuda()
    dst = torch.full((n + 1,), 5.0, dtype=torch.bfloat16, device="cuda")
    rg.regione_cast(ctx, src, rg.FP32, dst, rg.BF16, n)
    assert float(dst[n]) == 5.0
    # round to nearest even, as torch's conversion
    assert torch.equal(dst[:n].view(torch.int16), src.to(torch.bfloat16).view(torch.int16))
    back = torch.full((n + 1,), 7.0, dtype=torch.float32, device="cuda")
    rg.regione_cast(ctx, dst, rg.BF16, back, rg.FP32, n)
    assert float(back[n]) == 7.0
    assert torch.equal(back[:n], dst[:n].float())
    same = torch.zeros(n + 1, dtype=torch.float32, device="cuda")
    rg.regione_cast(ctx, src, rg.FP32, same, rg.FP32, n)
    assert torch.equal(same[:n], src)
    if n > 8:   # tensors that are not 16-byte aligned take the element-wise kernels
        odd = torch.zeros(n + 1, dtype=torch.float32, device="cuda")
        rg.regione_cast(ctx, src[1:], rg.FP32, odd[1:], rg.FP32, n - 1)
        assert torch.equal(odd[1:n], src[1:]) and float(odd[0]) == 0.0 and float(odd[n]) == 0.0
        odd16 = torch.zeros(n + 1, dtype=torch.bfloat16, device="cuda")
        rg.regione_cast(ctx, src[1:], rg.FP32, odd16[1:], rg.BF16, n - 1)
        assert torch.equal(odd16[1:n].view(torch.int16), src[1:].to(torch.bfloat16).view(torch.int16)) and float(odd16[n]) == 0.0
    with pytest.raises(rg.RegionEError):
        rg.regione_cast(ctx, src, 9, dst, rg.BF16, n)


@pytest.mark.parametrize("h_dtype", ["bf16", "f32"])
@pytest.mark.parametrize("n,hidden,mod", [(5, 256, True), (37, 3072, True), (3, 3072, False), (9, 200, True), (2, 8192, True)])
def test_layernorm_modulation_matches_oracle(ctx, h_dtype, n, hidden, mod):
    rng = np.random.default_rng(950 + n + hidden)
    h = (rng.standard_normal((n, hidden)) * 2.0 + 0.5).astype(np.float32)
    if h_dtype == "bf16":
        h = inputs.bf16_round(h)
    shift = (0.1 * rng.standard_normal(hidden)).astype(np.float32) if mod else None
    scale = (0.1 * rng.standard_normal(hidden)).astype(np.float32) if mod else None
    want = orc.modulate(orc.layer_norm(h), shift, scale)
    dh = torch.from_numpy(h).cuda()
    if h_dtype == "bf16":
        dh = dh.to(torch.bfloat16)
    u = torch.full((n + 1, hidden), 3.0, dtype=torch.bfloat16, device="cuda")
    rg.regione_layernorm(ctx, dh, rg.BF16 if h_dtype == "bf16" else rg.FP32, n, hidden,
                         None if shift is None else torch.from_numpy(shift).cuda(), None if scale is None else torch.from_numpy(scale).cuda(), u)
    got = u.float().cpu().numpy()
    assert np.all(got[n] == 3.0)
    # float32 statistics, one rounding to bf16: half an ulp of values up to ~5
    assert np.abs(got[:n] - want).max() <= 2.0 ** -8 * np.maximum(1.0, np.abs(want)).max()
