"""GPU parity of the conditioning path (one-vector linear layer with SiLU, sinusoidal time
embedding) against the float64 oracle."""
import numpy as np
import pytest
import torch

from oracle import regione_oracle as orc
from paper_2510_25590_amd import binding as rg
from paper_2510_25590_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = rg.Context(256, 4, 64, 1024, 64, 64)
    yield c
    c.close()


@pytest.mark.parametrize("n,k", [(18432, 3072), (9216 + 3, 3072), (50, 64), (7, 8), (1, 520), (33, 16384)])
@pytest.mark.parametrize("act", ["silu", "none"])
def test_vec_linear_matches_oracle(ctx, n, k, act):
    rng = np.random.default_rng(4000 + n + k)
    x = rng.standard_normal(k).astype(np.float32)
    w = inputs.bf16_round((rng.standard_normal((n, k)) / np.sqrt(k)).astype(np.float32))
    b = rng.standard_normal(n).astype(np.float32) if n % 2 else None
    want = orc.vec_linear(x, w, b, act)
    y = torch.full((n + 1,), 7.0, dtype=torch.float32, device="cuda")
    rg.regione_vec_linear(ctx, torch.from_numpy(x).cuda(), rg.ACT_SILU if act == "silu" else rg.ACT_NONE,
                          torch.from_numpy(w).to(torch.bfloat16).cuda(), None if b is None else torch.from_numpy(b).cuda(), n, k, y)
    got = y.cpu().numpy()
    assert got[n] == 7.0
    # float32 products and sums of k terms of size ~1/sqrt(k): far inside 1e-5 for every k here
    assert np.abs(got[:n] - want).max() <= 1e-5, np.abs(got[:n] - want).max()


def test_vec_linear_argument_checks(ctx):
    x = torch.zeros(16, device="cuda"); w = torch.zeros((4, 16), dtype=torch.bfloat16, device="cuda"); y = torch.zeros(4, device="cuda")
    rg.regione_vec_linear(ctx, x, rg.ACT_NONE, w, None, 0, 16, y)          # no row: nothing happens
    with pytest.raises(rg.RegionEError):
        rg.regione_vec_linear(ctx, x, rg.ACT_GELU_TANH, w, None, 4, 16, y)  # not an input activation
    with pytest.raises(rg.RegionEError):
        rg.regione_vec_linear(ctx, x, rg.ACT_NONE, w, None, 4, 12, y)       # k not a multiple of 8
    with pytest.raises(rg.RegionEError):
        rg.regione_vec_linear(ctx, None, rg.ACT_NONE, w, None, 4, 16, y)


@pytest.mark.parametrize("t,dim", [(0.0, 8), (0.731, 256), (999.0, 256), (28.0, 3072)])
def test_timestep_embedding_matches_oracle(ctx, t, dim):
    out = torch.full((dim + 1,), 5.0, dtype=torch.float32, device="cuda")
    rg.regione_timestep_embedding(ctx, t, dim, 10000.0, out)
    got = out.cpu().numpy()
    assert got[dim] == 5.0
    assert np.abs(got[:dim] - orc.timestep_embedding(t, dim, 10000.0)).max() <= 1e-7
    with pytest.raises(rg.RegionEError):
        rg.regione_timestep_embedding(ctx, t, 7, 10000.0, out)


def test_modulation_vectors_feed_a_block(ctx):
    """Time -> embedding -> two layers -> SiLU -> [6H, H] matrix: the six vectors the block takes, against the oracle."""
    hidden = 256
    rng = np.random.default_rng(4100)
    w1 = inputs.bf16_round((rng.standard_normal((hidden, 256)) / 16).astype(np.float32))
    w2 = inputs.bf16_round((rng.standard_normal((hidden, hidden)) / 16).astype(np.float32))
    wm = inputs.bf16_round((rng.standard_normal((6 * hidden, hidden)) / 16).astype(np.float32))
    bm = rng.standard_normal(6 * hidden).astype(np.float32)
    e = orc.timestep_embedding(0.4375, 256)
    want = orc.vec_linear(orc.vec_linear(orc.vec_linear(e, w1), w2, None, "silu"), wm, bm, "silu")
    d = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    emb = torch.empty(256, device="cuda"); h1 = torch.empty(hidden, device="cuda"); h2 = torch.empty(hidden, device="cuda")
    mod = torch.empty(6 * hidden, device="cuda")
    rg.regione_timestep_embedding(ctx, 0.4375, 256, 10000.0, emb)
    rg.regione_vec_linear(ctx, emb, rg.ACT_NONE, d(w1), None, hidden, 256, h1)
    rg.regione_vec_linear(ctx, h1, rg.ACT_SILU, d(w2), None, hidden, hidden, h2)
    rg.regione_vec_linear(ctx, h2, rg.ACT_SILU, d(wm), torch.from_numpy(bm).cuda(), 6 * hidden, hidden, mod)
    assert np.abs(mod.cpu().numpy() - want).max() <= 2e-5


@pytest.mark.parametrize("kind", ["double", "single"])
def test_block_forms_its_modulation_vectors_itself(kind):
    """A block given the step's conditioning vector and each stream's modulation layer equals, bit for bit, the same block
    given the six (three) vectors that regione_vec_linear makes of them; against the oracle's block with the oracle's
    vectors it holds the block tolerance."""
    from gpu_util import dev, host, assert_close, block_to_device
    hidden, heads, d, mlp, n_txt, n_img = 256, 4, 64, 1024, 24, 200
    n = n_txt + n_img
    n_vec = 6 if kind == "double" else 3
    rng = np.random.default_rng(4200 + n_vec)
    streams = [inputs.stream_weights(rng, hidden, mlp, kind, "bf16", std=0.05) for _ in range(2 if kind == "double" else 1)]
    cond = rng.standard_normal(hidden).astype(np.float32)
    mods = [(inputs.bf16_round((rng.standard_normal((n_vec * hidden, hidden)) / 64).astype(np.float32)), (0.1 * rng.standard_normal(n_vec * hidden)).astype(np.float32))
            for _ in streams]
    names = ("shift1", "scale1", "gate1", "shift2", "scale2", "gate2")[:n_vec]
    for w, (wm, bm) in zip(streams, mods):          # the oracle's vectors for the oracle's block
        vec = orc.vec_linear(cond, wm, bm, "silu")
        for i, name in enumerate(names):
            w[name] = vec[i * hidden:(i + 1) * hidden].astype(np.float32)
        if kind == "double":
            w["gate1"] = w["gate1"] + 1.0; w["gate2"] = w["gate2"] + 1.0      # gates near one, as in the synthetic model
        else:
            w["gate1"] = w["gate1"] + 1.0
    for (wm, bm), w in zip(mods, streams):          # the same shift of the gates through the layer's bias
        for i, name in enumerate(names):
            if name.startswith("gate"):
                bm[i * hidden:(i + 1) * hidden] += 1.0
    h = inputs.bf16_round(rng.standard_normal((n, hidden)).astype(np.float32))
    n_txt_rows = n_txt if kind == "double" else 0
    want = orc.block_forward(streams, kind, h, n_txt_rows, None, None, None, 0, heads)
    ctx = rg.Context(hidden, heads, d, mlp, n, 64)
    btype = rg.BLOCK_DOUBLE if kind == "double" else rg.BLOCK_SINGLE
    # (a) vectors made by the caller with regione_vec_linear
    dcond = torch.from_numpy(cond).cuda()
    bw, keep = block_to_device(streams, kind, ctx)
    made = []
    for s_i, (wm, bm) in enumerate(mods):
        vec = torch.empty(n_vec * hidden, dtype=torch.float32, device="cuda")
        wmd, bmd = torch.from_numpy(wm).to(torch.bfloat16).cuda(), torch.from_numpy(bm).cuda()
        rg.regione_vec_linear(ctx, dcond, rg.ACT_SILU, wmd, bmd, n_vec * hidden, hidden, vec)
        made.append((vec, wmd, bmd))
        sw = bw.img if (kind == "single" or s_i == 1) else bw.txt
        for i, name in enumerate(names):
            setattr(sw, name, vec.data_ptr() + 4 * i * hidden)
    out_a = torch.empty((n, hidden), dtype=torch.bfloat16, device="cuda")
    rg.regione_block_forward(ctx, bw, btype, dev(h, "bf16"), out_a, rg.BF16, n, n_txt_rows, None, 0, None, None, 0, 0)
    # (b) the block forms them itself; its own six pointers hold nonsense that must not be read
    junk = torch.full((hidden,), 1e30, dtype=torch.float32, device="cuda")
    for s_i, (vec, wmd, bmd) in enumerate(made):
        sw = bw.img if (kind == "single" or s_i == 1) else bw.txt
        for name in names:
            setattr(sw, name, junk.data_ptr())
        sw.w_mod, sw.b_mod = wmd.data_ptr(), bmd.data_ptr()
    bw.cond = dcond.data_ptr()
    out_b = torch.empty_like(out_a)
    rg.regione_block_forward(ctx, bw, btype, dev(h, "bf16"), out_b, rg.BF16, n, n_txt_rows, None, 0, None, None, 0, 0)
    torch.cuda.synchronize()
    assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16))
    assert_close(host(out_b), want, f"{kind} block with modulation vectors formed inside the call", stored_bf16=True)
    ctx.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("n_vec,elems", [(28 * 3, 4096 * 64), (5, 8), (3, 1000), (1, 0)])
def test_sq_norms_match_float64_sums(ctx, dtype, n_vec, elems):
    rng = np.random.default_rng(4200 + n_vec + elems)
    x = rng.standard_normal((n_vec, elems)).astype(np.float32)
    if dtype == "bf16":
        x = inputs.bf16_round(x)
    d = torch.from_numpy(x).cuda()
    if dtype == "bf16":
        d = d.to(torch.bfloat16)
    out = torch.full((n_vec + 1,), -1.0, dtype=torch.float64, device="cuda")
    rg.regione_sq_norms(ctx, d, rg.BF16 if dtype == "bf16" else rg.FP32, n_vec, elems, out)
    got = out.cpu().numpy()
    assert got[n_vec] == -1.0
    want = (x.astype(np.float64) ** 2).sum(axis=1)
    # squares are exact in float64; only the order of the additions differs from numpy's
    assert np.allclose(got[:n_vec], want, rtol=1e-12, atol=0)
    out2 = torch.empty_like(out)
    rg.regione_sq_norms(ctx, d, rg.BF16 if dtype == "bf16" else rg.FP32, n_vec, elems, out2)
    assert torch.equal(out[:n_vec], out2[:n_vec])          # fixed summation order


def test_gamma_fit_from_device_norms(ctx):
    """Velocity traces that follow Eq.7 with a known table: norms on the device, fit on the host."""
    from oracle import regione_oracle as orc
    rng = np.random.default_rng(4300)
    T, S, n = 12, 4, 2048
    t = np.linspace(0.0, 1.0, T + 1)
    gamma = 1.0 + 0.05 * rng.standard_normal(T + 1)
    v = np.zeros((S, T + 1, n), dtype=np.float32)
    v[:, T] = rng.standard_normal((S, n))
    for j in range(T - 1, 0, -1):
        v[:, j] = v[:, j + 1] * np.float32(orc.decay_factor(t, gamma, j))
    sq = torch.zeros((S, T + 1), dtype=torch.float64, device="cuda")
    rg.regione_sq_norms(ctx, torch.from_numpy(v).cuda(), rg.FP32, S * (T + 1), n, sq)
    got = np.array(rg.regione_gamma_fit_host(sq.cpu().numpy(), t))
    assert np.allclose(got[1:T], gamma[1:T], rtol=1e-5)
    want = orc.fit_gamma(np.sqrt((v.astype(np.float64) ** 2).sum(axis=2)), t)
    assert np.allclose(got, want, rtol=1e-5)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_guidance_combine_matches_oracle(ctx, dtype):
    from oracle import regione_oracle as orc
    rng = np.random.default_rng(4400)
    n = 4096 * 64 + 5
    vc = rng.standard_normal(n).astype(np.float32); vu = rng.standard_normal(n).astype(np.float32)
    if dtype == "bf16":
        vc, vu = inputs.bf16_round(vc), inputs.bf16_round(vu)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    code = rg.BF16 if dtype == "bf16" else rg.FP32
    dc, du = torch.from_numpy(vc).cuda().to(tdt), torch.from_numpy(vu).cuda().to(tdt)
    out = torch.full((n + 1,), 3.0, dtype=tdt, device="cuda")
    rg.regione_guidance_combine(ctx, dc, du, 2.5, out, n, code)
    want = orc.guidance_combine(vc, vu, 2.5)
    got = out.float().cpu().numpy()
    assert got[n] == 3.0
    tol = 2.0 ** -8 * np.abs(want).max() if dtype == "bf16" else 1e-6 * np.abs(want).max()
    assert np.abs(got[:n] - want).max() <= tol
    # in place on the conditional velocity; scale 1 returns it, scale 0 the unconditional one
    rg.regione_guidance_combine(ctx, dc, du, 1.0, dc, n, code)
    assert np.abs(dc.float().cpu().numpy() - vc).max() <= (2.0 ** -8 if dtype == "bf16" else 1e-6) * np.abs(vc).max()
    rg.regione_guidance_combine(ctx, dc, du, 0.0, out, n, code)
    assert torch.equal(out[:n], du)
    rg.regione_guidance_combine(ctx, dc, du, 2.0, out, 0, code)      # nothing to do
