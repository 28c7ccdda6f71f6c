"""GPU parity of the float32 context (the arithmetic of the tiny float32 configuration): dense projection, attention
with the Region-Instruction KV cache (Eq.6) in its three key-source forms, one block in all modes of Algorithm 1's flag
pair for both block types, at max abs 1e-4 against the float64 oracle on float32 inputs that are NOT bf16-rounded."""
import numpy as np
import pytest
import torch

from oracle import regione_oracle as orc
from paper_2510_25590_amd import binding as rg
from paper_2510_25590_amd import inputs
from gpu_util import host, assert_close

pytestmark = pytest.mark.gpu

TOL = dict(max_abs=1e-4, mean_rel_tol=2e-5)   # float32 products and sums over at most 1280 terms of O(1) values: measured ~1e-6


def f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def _ctx(hidden=256, heads=4, d=64, mlp=1024, rows=1024):
    return rg.Context(hidden, heads, d, mlp, rows, 4096, compute_dtype=rg.FP32)


@pytest.mark.parametrize("m,n,k", [(1, 64, 64), (36, 256, 64), (70, 200, 128), (544, 1024, 256), (129, 40, 1024)])
@pytest.mark.parametrize("act", [rg.ACT_NONE, rg.ACT_GELU_TANH])
def test_linear_float32(m, n, k, act):
    rng = np.random.default_rng(100 + m + n)
    x = rng.standard_normal((m, k)).astype(np.float32)
    w = (0.1 * rng.standard_normal((n, k))).astype(np.float32)
    b = rng.standard_normal(n).astype(np.float32)
    ctx = _ctx()
    wp = rg.pack_weight(ctx, f32(w))
    y = torch.full((m, n), float("nan"), dtype=torch.float32, device="cuda")
    rg.regione_linear(ctx, f32(x), wp, f32(b), m, n, k, act, rg.FP32, y)
    want = orc.linear(x, w, b)
    if act == rg.ACT_GELU_TANH:
        want = orc.gelu_tanh(want)
    assert_close(host(y), want, f"float32 linear {m}x{n}x{k}", **TOL)
    ctx.close()


@pytest.mark.parametrize("d", [64, 128])
def test_attention_float32_three_key_sources(d):
    rng = np.random.default_rng(200 + d)
    heads, n_q, n_fresh, n_c = 3, 45, 45, 150
    q, kf, vf = (rng.standard_normal((n_q, heads, d)).astype(np.float32) for _ in range(3))
    kc, vc = (rng.standard_normal((n_c, heads, d)).astype(np.float32) for _ in range(2))
    idx = np.sort(rng.choice(n_c, size=70, replace=False)).astype(np.int32)
    ctx = _ctx(hidden=heads * d, heads=heads, d=d, mlp=64)
    out = torch.empty((n_q, heads, d), dtype=torch.float32, device="cuda")
    # fresh rows only (the variant without the cache), fresh + whole cache, fresh + listed cache rows
    rg.regione_attn_kvcache(ctx, f32(q), n_q, f32(kf), f32(vf), n_fresh, None, None, 0, None, 0, heads, d, 0.0, out)
    assert_close(host(out), orc.attention_kvcache(q, kf, vf), "float32 attention, fresh rows only", **TOL)
    rg.regione_attn_kvcache(ctx, f32(q), n_q, f32(kf), f32(vf), n_fresh, f32(kc), f32(vc), n_c, None, 0, heads, d, 0.0, out)
    assert_close(host(out), orc.attention_kvcache(q, kf, vf, kc, vc), "float32 attention, fresh + cache", **TOL)
    rg.regione_attn_kvcache(ctx, f32(q), n_q, f32(kf), f32(vf), n_fresh, f32(kc), f32(vc), n_c, torch.from_numpy(idx).cuda(), len(idx), heads, d, 0.0, out)
    assert_close(host(out), orc.attention_kvcache(q, kf, vf, kc, vc, idx), "float32 attention, fresh + listed cache rows", **TOL)
    # cache rows only, one key, and a scale of the caller's
    rg.regione_attn_kvcache(ctx, f32(q), n_q, None, None, 0, f32(kc[:1]), f32(vc[:1]), 1, None, 0, heads, d, 0.0, out)
    assert_close(host(out), np.broadcast_to(vc[:1], (n_q, heads, d)), "float32 attention, one key", **TOL)
    rg.regione_attn_kvcache(ctx, f32(q), n_q, f32(kf), f32(vf), n_fresh, None, None, 0, None, 0, heads, d, 0.05, out)
    assert_close(host(out), orc.attention_kvcache(q, kf, vf, scale=0.05), "float32 attention, given scale", **TOL)
    ctx.close()


def _block_to_device_f32(streams, kind, ctx):
    keep, bw = [], rg.BlockWeights()
    for name, w in zip(("txt", "img") if kind == "double" else ("img",), streams):
        t = {k: (rg.pack_weight(ctx, f32(a)) if k.startswith("w_") else f32(a)) for k, a in w.items()}
        keep.append(t)
        setattr(bw, name, rg.make_stream_weights(t))
    return bw, keep


@pytest.mark.parametrize("kind", ["double", "single"])
def test_tiny_block_float32_all_modes(kind):
    hidden, heads, d, mlp = 256, 4, 64, 1024
    n_txt, n_img = 32, 256
    n_all = n_txt + 2 * n_img
    rng = np.random.default_rng(inputs.workload_seed(1, 11))
    streams = [inputs.stream_weights(rng, hidden, mlp, kind, "f32", std=0.05) for _ in range(2 if kind == "double" else 1)]
    h = rng.standard_normal((n_all, hidden)).astype(np.float32)
    e = np.nonzero(inputs.rect_mask(rng, 16, 16, 6, 6))[0].astype(np.int32)
    ctx = _ctx(rows=n_all)
    bw, keep = _block_to_device_f32(streams, kind, ctx)
    btype = rg.BLOCK_DOUBLE if kind == "double" else rg.BLOCK_SINGLE
    kc_o = np.zeros((n_all, heads, d)); vc_o = np.zeros_like(kc_o)
    full_o = orc.block_forward(streams, kind, h, n_txt, np.arange(n_all), kc_o, vc_o, orc.FLAG_STORE, heads)
    kc = torch.zeros((n_all, heads, d), dtype=torch.float32, device="cuda"); vc = torch.zeros_like(kc)
    out = torch.empty((n_all, hidden), dtype=torch.float32, device="cuda")
    slots_all = torch.arange(n_all, dtype=torch.int32, device="cuda")
    rg.regione_block_forward(ctx, bw, btype, f32(h), out, rg.FP32, n_all, n_txt, slots_all, 0, kc, vc, n_all, rg.FLAG_STORE)
    assert_close(host(out), full_o, f"{kind} float32 storing full forward", **TOL)
    assert_close(host(kc), kc_o, "stored K (float32)", **TOL)
    assert_close(host(vc), vc_o, "stored V (float32)", **TOL)
    out2 = torch.empty_like(out)
    rg.regione_block_forward(ctx, bw, btype, f32(h), out2, rg.FP32, n_all, n_txt, None, 0, None, None, 0, 0)
    assert_close(host(out2), full_o, f"{kind} float32 plain full forward", **TOL)
    h2 = (h + 0.05 * rng.standard_normal(h.shape)).astype(np.float32)      # stale cache
    for mode, rows in (("edited rows fresh", n_txt + e), ("text + edited rows fresh", np.concatenate([np.arange(n_txt), n_txt + e]))):
        n_txt_fresh = 0 if rows[0] != 0 else n_txt
        want = orc.block_forward(streams, kind, h2[rows], n_txt_fresh, rows, kc_o, vc_o, orc.FLAG_RETRIEVE, heads)
        kc_before, vc_before = kc.clone(), vc.clone()
        o = torch.empty((len(rows), hidden), dtype=torch.float32, device="cuda")
        rg.regione_block_forward(ctx, bw, btype, f32(h2[rows]), o, rg.FP32, len(rows), n_txt_fresh, torch.from_numpy(rows.astype(np.int32)).cuda(), 0,
                                 kc, vc, n_all, rg.FLAG_RETRIEVE)
        assert_close(host(o), want, f"{kind} float32 region forward, {mode}", **TOL)
        untouched = np.setdiff1d(np.arange(n_all), rows)
        assert torch.equal(kc[untouched], kc_before[untouched]) and torch.equal(vc[untouched], vc_before[untouched])
        kc.copy_(kc_before); vc.copy_(vc_before)
    # two guidance branches in one call equal two calls
    hb = np.stack([h2[n_txt + e], (h2[n_txt + e] + 0.1).astype(np.float32)])
    kc2 = torch.stack([kc, kc]); vc2 = torch.stack([vc, vc])
    ob = torch.empty((2, len(e), hidden), dtype=torch.float32, device="cuda")
    rg.regione_block_forward_batched(ctx, bw, btype, f32(hb), ob, rg.FP32, 2, len(e), 0, torch.from_numpy(e).cuda(), n_txt, kc2, vc2, n_all, rg.FLAG_RETRIEVE)
    for b in range(2):
        want = orc.block_forward(streams, kind, hb[b], 0, n_txt + e, kc_o, vc_o, orc.FLAG_RETRIEVE, heads)
        assert_close(host(ob[b]), want, f"{kind} float32 batched region forward, branch {b}", **TOL)
    ctx.close()


def test_float32_context_refuses_bf16_only_features():
    ctx = _ctx()
    bw = rg.BlockWeights()
    h = torch.zeros((4, 256), dtype=torch.float32, device="cuda")
    with pytest.raises(rg.RegionEError) as ei:     # a bf16 residual stream in a float32 context
        rg.regione_block_forward(ctx, bw, rg.BLOCK_DOUBLE, h, h, rg.BF16, 4, 0, None, 0, None, None, 0, 0)
    assert ei.value.code == rg.ERR_INVALID_ARG
    bw.rope, bw.rope_rows = h.data_ptr(), 4
    with pytest.raises(rg.RegionEError) as ei:
        rg.regione_block_forward(ctx, bw, rg.BLOCK_DOUBLE, h, h, rg.FP32, 4, 0, None, 0, None, None, 0, 0)
    assert ei.value.code == rg.ERR_UNSUPPORTED
    with pytest.raises(rg.RegionEError) as ei:
        rg.regione_linear_fp8(ctx, h, h, h, h, None, 4, 64, 128, rg.ACT_NONE, rg.FP32, h)
    assert ei.value.code == rg.ERR_UNSUPPORTED
    ctx.close()
