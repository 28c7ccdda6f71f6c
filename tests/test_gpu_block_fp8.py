"""GPU parity of the double-stream block with its four projections in 8-bit floating point (regione_block_forward_fp8).

A code of the E4M3 format moves when its input moves by a part in a million, so the block's output cannot be compared
with a float64 block that quantises its own intermediates: a handful of flipped codes would differ by the format's
whole step.  The block is therefore checked STAGE BY STAGE: the library hands out every intermediate (taps), and every
stage is compared with the reference of that stage fed with the library's own input of the stage:
  LayerNorm + modulation + quantisation: the scale, the dequantised values within half a code step of the float64
      result, and the codes themselves equal to the reference quantiser's except where the float32 result sits on a
      rounding boundary (a fraction below 1e-3, each by one code step);
  quantisation of bf16 rows (attention output, MLP rows): codes and scales bit for bit;
  projections: exact products of the library's codes within the accumulation bound of the matrix-core instruction;
  attention: the float64 attention on the library's queries and cache rows.
A last comparison with the unquantised float64 block states what the format costs."""
import numpy as np
import pytest
import torch

from oracle import fp8_reference as f8
from oracle import regione_oracle as orc
from paper_2510_25590_amd import binding as rg
from paper_2510_25590_amd import inputs
from gpu_util import dev, host, assert_close, block_to_device, half_ulp_bf16

pytestmark = pytest.mark.gpu

MFMA_SUM_ERR = 2.0 ** -11      # accumulation bound of the 8-bit matrix-core instruction (see test_gpu_fp8.py)


def _check_ln_quant(what, h_rows, shift, scale, codes, row_scale):
    y = orc.modulate(orc.layer_norm(h_rows), shift, scale)                       # float64
    amax = np.max(np.abs(y), axis=1)
    assert np.allclose(row_scale, amax / 448.0, rtol=2e-5, atol=0), f"{what}: row scales"
    deq = f8.e4m3_decode(codes) * row_scale[:, None].astype(np.float64)
    tol = f8.e4m3_half_step(y / row_scale[:, None]) * row_scale[:, None] * 1.001 + np.abs(y) * 2e-5
    bad = np.abs(deq - y) > tol
    assert not bad.any(), f"{what}: {bad.sum()} dequantised values farther than half a code step from the float64 result"
    want_codes, _ = f8.quantize_rows(y.astype(np.float32))
    diff = codes != want_codes
    assert diff.mean() < 1e-3, f"{what}: {diff.mean():.2e} of the codes differ from the reference quantiser's"
    if diff.any():   # ... and those by one step: neighbouring codes of one sign, or +0 / -0
        step = np.abs(codes[diff].astype(np.int16) - want_codes[diff].astype(np.int16))
        assert np.all((step == 1) | (step == 128)), f"{what}: a code differs by more than one step"


def _check_linear(what, codes, row_scale, w_codes, w_scale, bias, got, post=None, lipschitz=1.0, out_bf16=False, cols=None):
    """got against post(x_scale * w_scale * codes . w_codes + bias) on the library's own codes."""
    if cols is not None:
        w_codes, w_scale, bias = w_codes[cols], w_scale[cols], bias[cols]
    lin = f8.linear_fp8(codes, row_scale, w_codes, w_scale, bias)
    mag = (np.abs(f8.e4m3_decode(codes)) @ np.abs(f8.e4m3_decode(w_codes)).T) * row_scale[:, None].astype(np.float64) * w_scale[None, :]
    want, bound = (lin, mag * MFMA_SUM_ERR) if post is None else post(lin, mag * MFMA_SUM_ERR)
    bound = bound * lipschitz + np.abs(want) * 2.0 ** -21 + 1e-30
    if out_bf16:
        bound = bound + half_ulp_bf16(want) * 1.01
    err = np.abs(got.astype(np.float64) - want)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert np.all(err <= bound), f"{what}: worst at {worst}: got {got[worst]!r} want {want[worst]!r} bound {bound[worst]:.3e}"


@pytest.mark.parametrize("hidden,heads,d,mlp,n_txt,n_img,n_e,h_dtype", [
    (256, 4, 64, 1024, 32, 256, 36, "bf16"),
    (256, 4, 64, 1024, 32, 256, 36, "f32"),
    (1024, 8, 128, 4096, 64, 400, 333, "bf16"),
    (3072, 24, 128, 12288, 128, 1024, 300, "bf16"),       # the headline block's widths
])
@pytest.mark.parametrize("mode", ["retrieve_img", "retrieve_txt_img", "store", "plain"])
def test_block_fp8_stage_by_stage(hidden, heads, d, mlp, n_txt, n_img, n_e, h_dtype, mode):
    if hidden == 3072 and mode != "retrieve_txt_img":
        pytest.skip("the 3072-wide block runs once, in the mode that uses both streams")
    n_all = n_txt + 2 * n_img
    rng = np.random.default_rng(inputs.workload_seed(8, hidden + n_e))
    streams = [inputs.stream_weights(rng, hidden, mlp, "double", "bf16", std=0.03 if hidden < 3072 else 0.02) for _ in range(2)]
    h_all = inputs.bf16_round(rng.standard_normal((n_all, hidden)).astype(np.float32))
    ctx = rg.Context(hidden, heads, d, mlp, n_all, 4096)
    bw, keep = block_to_device(streams, "double", ctx)
    w8 = rg.BlockWeightsFp8()
    w8.txt, keep_t = rg.make_stream_weights_fp8(ctx, {k: dev(v, "bf16") for k, v in streams[0].items() if k.startswith("w_")})
    w8.img, keep_i = rg.make_stream_weights_fp8(ctx, {k: dev(v, "bf16") for k, v in streams[1].items() if k.startswith("w_")})
    wq = [{k: (t[2].cpu().numpy(), t[1].cpu().numpy()) for k, t in kp.items()} for kp in (keep_t, keep_i)]   # codes, scales
    hcode = rg.BF16 if h_dtype == "bf16" else rg.FP32
    tdt = torch.bfloat16 if h_dtype == "bf16" else torch.float32

    # the cache of the region modes comes from a storing full forward of the bf16 block
    kc = torch.zeros((n_all, heads, d), dtype=torch.bfloat16, device="cuda"); vc = torch.zeros_like(kc)
    slots_all = torch.arange(n_all, dtype=torch.int32, device="cuda")
    tmp = torch.empty((n_all, hidden), dtype=torch.bfloat16, device="cuda")
    rg.regione_block_forward(ctx, bw, rg.BLOCK_DOUBLE, dev(h_all, "bf16"), tmp, rg.BF16, n_all, n_txt, slots_all, 0, kc, vc, n_all, rg.FLAG_STORE)

    e = np.sort(rng.choice(n_img, size=n_e, replace=False)).astype(np.int32)
    h_moved = inputs.bf16_round((h_all + 0.05 * rng.standard_normal(h_all.shape)).astype(np.float32))
    if mode == "retrieve_img":
        rows, n_txt_fresh, flags = n_txt + e, 0, rg.FLAG_RETRIEVE
    elif mode == "retrieve_txt_img":
        rows, n_txt_fresh, flags = np.concatenate([np.arange(n_txt), n_txt + e]), n_txt, rg.FLAG_RETRIEVE
    elif mode == "store":
        rows, n_txt_fresh, flags = np.arange(n_all), n_txt, rg.FLAG_STORE
    else:
        rows, n_txt_fresh, flags = np.arange(n_txt + n_img), n_txt, 0
    n = len(rows)
    h_in = h_moved[rows]
    dslots = torch.from_numpy(rows.astype(np.int32)).cuda() if flags else None
    kc_before, vc_before = kc.clone(), vc.clone()

    z8 = lambda c: torch.full((n, c), 0x55, dtype=torch.uint8, device="cuda")
    zf = lambda: torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
    t = {"u1_codes": z8(hidden), "u1_scale": zf(), "q": torch.zeros((n, hidden), dtype=torch.bfloat16, device="cuda"),
         "attn": torch.zeros((n, hidden), dtype=torch.bfloat16, device="cuda"), "a_codes": z8(hidden), "a_scale": zf(),
         "h1": torch.zeros((n, hidden), dtype=torch.float32, device="cuda"), "u2_codes": z8(hidden), "u2_scale": zf(),
         "m": torch.zeros((n, mlp), dtype=torch.bfloat16, device="cuda"), "m_codes": z8(mlp), "m_scale": zf()}
    out = torch.empty((n, hidden), dtype=tdt, device="cuda")
    rg.regione_block_forward_fp8(ctx, bw, w8, rg.BLOCK_DOUBLE, dev(h_in, h_dtype), out, hcode, n, n_txt_fresh, dslots, 0,
                                 kc if flags else None, vc if flags else None, n_all if flags else 0, flags, rg.make_fp8_taps(t))
    torch.cuda.synchronize()
    T = {k: (v.cpu().numpy() if v.dtype != torch.bfloat16 else host(v)) for k, v in t.items()}
    got_out = host(out)
    kc_h, vc_h = host(kc).reshape(n_all, hidden), host(vc).reshape(n_all, hidden)

    groups = [(np.arange(0, n_txt_fresh), 0), (np.arange(n_txt_fresh, n), 1)]
    H = hidden
    for g_rows, s in groups:
        if len(g_rows) == 0:
            continue
        w, (name, q8) = streams[s], ("text" if s == 0 else "image", wq[s])
        _check_ln_quant(f"{name}: first LayerNorm", h_in[g_rows], w["shift1"], w["scale1"], T["u1_codes"][g_rows], T["u1_scale"][g_rows])
        codes, sc = T["u1_codes"][g_rows], T["u1_scale"][g_rows]
        _check_linear(f"{name}: queries", codes, sc, q8["w_qkv"][0], q8["w_qkv"][1], w["b_qkv"], T["q"][g_rows], out_bf16=True, cols=slice(0, H))
        if flags:      # keys and values went to their cache slots
            _check_linear(f"{name}: keys", codes, sc, q8["w_qkv"][0], q8["w_qkv"][1], w["b_qkv"], kc_h[rows[g_rows]], out_bf16=True, cols=slice(H, 2 * H))
            _check_linear(f"{name}: values", codes, sc, q8["w_qkv"][0], q8["w_qkv"][1], w["b_qkv"], vc_h[rows[g_rows]], out_bf16=True, cols=slice(2 * H, 3 * H))
    if flags:
        untouched = np.setdiff1d(np.arange(n_all), rows)
        assert torch.equal(kc[untouched].view(torch.int16), kc_before[untouched].view(torch.int16))
        assert torch.equal(vc[untouched].view(torch.int16), vc_before[untouched].view(torch.int16))
        if flags == rg.FLAG_RETRIEVE:   # Eq.6 on the library's queries and the cache as it stands (fresh rows in their slots)
            want_attn = orc.attention_kvcache(T["q"].reshape(n, heads, d), kc_h.reshape(n_all, heads, d), vc_h.reshape(n_all, heads, d))
        else:                           # a storing forward attends over its own rows: the same rows, now in the cache
            want_attn = orc.attention_kvcache(T["q"].reshape(n, heads, d), kc_h.reshape(n_all, heads, d)[rows], vc_h.reshape(n_all, heads, d)[rows])
        assert_close(T["attn"], want_attn.reshape(n, hidden), "attention on the library's queries and cache rows")
    for g_rows, s in groups:
        if len(g_rows) == 0:
            continue
        w, (name, q8) = streams[s], ("text" if s == 0 else "image", wq[s])
        want_c, want_s = f8.quantize_rows(T["attn"][g_rows])
        assert np.array_equal(T["a_codes"][g_rows], want_c) and np.array_equal(T["a_scale"][g_rows].view(np.uint32), want_s.view(np.uint32)), f"{name}: codes of the attention output"
        gate1, gate2 = w["gate1"].astype(np.float64), w["gate2"].astype(np.float64)
        resid = h_in[g_rows].astype(np.float64)
        _check_linear(f"{name}: output projection + residual", T["a_codes"][g_rows], T["a_scale"][g_rows], q8["w_o"][0], q8["w_o"][1], w["b_o"], T["h1"][g_rows],
                      post=lambda lin, b: (resid + gate1 * lin, np.abs(gate1) * b))
        _check_ln_quant(f"{name}: second LayerNorm", T["h1"][g_rows], w["shift2"], w["scale2"], T["u2_codes"][g_rows], T["u2_scale"][g_rows])
        _check_linear(f"{name}: MLP up + GELU", T["u2_codes"][g_rows], T["u2_scale"][g_rows], q8["w_1"][0], q8["w_1"][1], w["b_1"], T["m"][g_rows],
                      post=lambda lin, b: (orc.gelu_tanh(lin), 1.13 * b), out_bf16=True)
        want_c, want_s = f8.quantize_rows(T["m"][g_rows])
        assert np.array_equal(T["m_codes"][g_rows], want_c) and np.array_equal(T["m_scale"][g_rows].view(np.uint32), want_s.view(np.uint32)), f"{name}: codes of the MLP rows"
        h1 = T["h1"][g_rows].astype(np.float64)
        _check_linear(f"{name}: MLP down + residual", T["m_codes"][g_rows], T["m_scale"][g_rows], q8["w_2"][0], q8["w_2"][1], w["b_2"], got_out[g_rows],
                      post=lambda lin, b: (h1 + gate2 * lin, np.abs(gate2) * b), out_bf16=(h_dtype == "bf16"))

    # what the format costs: the block's update against the unquantised float64 block on the same inputs
    if mode.startswith("retrieve"):
        kc_o, vc_o = host(kc_before).astype(np.float64), host(vc_before).astype(np.float64)
        want = orc.block_forward(streams, "double", h_in, n_txt_fresh, rows, kc_o, vc_o, orc.FLAG_RETRIEVE, heads)
        upd_got, upd_want = got_out - h_in, want - h_in
        rel = np.linalg.norm(upd_got - upd_want) / np.linalg.norm(upd_want)
        print(f"\n8-bit block against the float64 block ({mode}, hidden {hidden}): relative difference of the block's update {rel:.3%}")
        assert rel < 0.10
    ctx.close()


@pytest.mark.parametrize("hidden,heads,d,mlp,n_txt,n_img,n_e", [(256, 4, 64, 1024, 32, 256, 36), (1024, 8, 128, 4096, 64, 400, 333)])
@pytest.mark.parametrize("mode", ["retrieve", "store"])
def test_single_stream_block_fp8_stage_by_stage(hidden, heads, d, mlp, n_txt, n_img, n_e, mode):
    """The single-stream form: one projection [q | k | v | m] from the quantised LayerNorm result, attention, the joint
    row [attention | GELU(m)] quantised as one row, one projection back with the gated residual."""
    n_all = n_txt + 2 * n_img
    H = hidden
    rng = np.random.default_rng(inputs.workload_seed(9, hidden + n_e))
    w = inputs.stream_weights(rng, hidden, mlp, "single", "bf16", std=0.03)
    h_all = inputs.bf16_round(rng.standard_normal((n_all, hidden)).astype(np.float32))
    ctx = rg.Context(hidden, heads, d, mlp, n_all, 4096)
    bw, keep = block_to_device([w], "single", ctx)
    w8 = rg.BlockWeightsFp8()
    w8.img, keep8 = rg.make_stream_weights_fp8(ctx, {k: dev(v, "bf16") for k, v in w.items() if k.startswith("w_")})
    q8 = {k: (t[2].cpu().numpy(), t[1].cpu().numpy()) for k, t in keep8.items()}
    kc = torch.zeros((n_all, heads, d), dtype=torch.bfloat16, device="cuda"); vc = torch.zeros_like(kc)
    slots_all = torch.arange(n_all, dtype=torch.int32, device="cuda")
    tmp = torch.empty((n_all, hidden), dtype=torch.bfloat16, device="cuda")
    rg.regione_block_forward(ctx, bw, rg.BLOCK_SINGLE, dev(h_all, "bf16"), tmp, rg.BF16, n_all, 0, slots_all, 0, kc, vc, n_all, rg.FLAG_STORE)
    h_moved = inputs.bf16_round((h_all + 0.05 * rng.standard_normal(h_all.shape)).astype(np.float32))
    if mode == "retrieve":
        rows, flags = (n_txt + np.sort(rng.choice(n_img, size=n_e, replace=False))).astype(np.int32), rg.FLAG_RETRIEVE
    else:
        rows, flags = np.arange(n_all, dtype=np.int32), rg.FLAG_STORE
    n = len(rows)
    h_in = h_moved[rows]
    kc_before = kc.clone()
    t = {"u1_codes": torch.full((n, H), 0x55, dtype=torch.uint8, device="cuda"), "u1_scale": torch.full((n,), -1.0, device="cuda"),
         "q": torch.zeros((n, H), dtype=torch.bfloat16, device="cuda"), "attn": torch.zeros((n, H + mlp), dtype=torch.bfloat16, device="cuda"),
         "a_codes": torch.full((n, H + mlp), 0x55, dtype=torch.uint8, device="cuda"), "a_scale": torch.full((n,), -1.0, device="cuda")}
    out = torch.empty((n, hidden), dtype=torch.bfloat16, device="cuda")
    rg.regione_block_forward_fp8(ctx, bw, w8, rg.BLOCK_SINGLE, dev(h_in, "bf16"), out, rg.BF16, n, 0, torch.from_numpy(rows).cuda(), 0,
                                 kc, vc, n_all, flags, rg.make_fp8_taps(t))
    torch.cuda.synchronize()
    T = {k: (v.cpu().numpy() if v.dtype != torch.bfloat16 else host(v)) for k, v in t.items()}
    kc_h, vc_h = host(kc).reshape(n_all, hidden), host(vc).reshape(n_all, hidden)
    _check_ln_quant("LayerNorm", h_in, w["shift1"], w["scale1"], T["u1_codes"], T["u1_scale"])
    c1, s1 = q8["w_1"]
    args = (T["u1_codes"], T["u1_scale"], c1, s1, w["b_1"])
    _check_linear("queries", *args, T["q"], out_bf16=True, cols=slice(0, H))
    _check_linear("keys", *args, kc_h[rows], out_bf16=True, cols=slice(H, 2 * H))
    _check_linear("values", *args, vc_h[rows], out_bf16=True, cols=slice(2 * H, 3 * H))
    _check_linear("MLP part + GELU", *args, T["attn"][:, H:], post=lambda lin, b: (orc.gelu_tanh(lin), 1.13 * b), out_bf16=True, cols=slice(3 * H, 3 * H + mlp))
    untouched = np.setdiff1d(np.arange(n_all), rows)
    assert torch.equal(kc[untouched].view(torch.int16), kc_before[untouched].view(torch.int16))
    keys = np.arange(n_all) if flags == rg.FLAG_RETRIEVE else rows
    want_attn = orc.attention_kvcache(T["q"].reshape(n, heads, d), kc_h.reshape(n_all, heads, d)[keys], vc_h.reshape(n_all, heads, d)[keys])
    assert_close(T["attn"][:, :H], want_attn.reshape(n, hidden), "attention on the library's queries and cache rows")
    want_c, want_s = f8.quantize_rows(T["attn"])
    assert np.array_equal(T["a_codes"], want_c) and np.array_equal(T["a_scale"].view(np.uint32), want_s.view(np.uint32)), "codes of the joint row"
    gate1, resid = w["gate1"].astype(np.float64), h_in.astype(np.float64)
    _check_linear("projection back + residual", T["a_codes"], T["a_scale"], q8["w_2"][0], q8["w_2"][1], w["b_2"], host(out),
                  post=lambda lin, b: (resid + gate1 * lin, np.abs(gate1) * b), out_bf16=True)
    ctx.close()


def test_block_fp8_argument_checks():
    ctx = rg.Context(256, 4, 64, 1024, 64, 64)
    bw, w8 = rg.BlockWeights(), rg.BlockWeightsFp8()
    h = torch.zeros((8, 256), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(rg.RegionEError) as err:      # no weights
        rg.regione_block_forward_fp8(ctx, bw, w8, rg.BLOCK_DOUBLE, h, h, rg.BF16, 8, 0, None, 0, None, None, 0, 0)
    assert err.value.code == rg.ERR_INVALID_ARG
    rg.regione_block_forward_fp8(ctx, bw, w8, rg.BLOCK_SINGLE, None, None, rg.BF16, 0, 0, None, 0, None, None, 0, 0)     # no row: nothing happens
    ctx.close()
    ctx32 = rg.Context(256, 4, 64, 1024, 64, 64, compute_dtype=rg.FP32)
    with pytest.raises(rg.RegionEError) as err:
        rg.regione_block_forward_fp8(ctx32, bw, w8, rg.BLOCK_DOUBLE, h, h, rg.FP32, 8, 0, None, 0, None, None, 0, 0)
    assert err.value.code == rg.ERR_UNSUPPORTED
    ctx32.close()
