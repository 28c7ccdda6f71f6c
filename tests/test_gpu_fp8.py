"""GPU parity of the 8-bit floating point (E4M3) variant of the dense projections against oracle/fp8_reference.py:
the codes and scales bit for bit, the products within the float32 accumulation bound."""
import numpy as np
import pytest
import torch

from oracle import fp8_reference as f8
from paper_2510_25590_amd import binding as rg
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

# Accuracy of the sums.  Products of two E4M3 values are exact, but the 8-bit matrix-core instruction does not add its
# 64 products as float32 numbers: measured on MI355X (one product of 448 * 448 next to small ones), the products of a
# group of 8 are aligned to the largest of the group and cut below 2^-14 of its exponent's value before they are added;
# group sums and successive instructions are then added in float32.  So per group the error is below
# 7 * 2^-14 * max|product| and over a whole dot product below 7 * 2^-14 * sum|products| < 2^-11 * sum|products|, which
# also covers the float32 additions (2^-24 each).  For comparison, the quantisation itself costs up to 2^-4 per operand.
MFMA_SUM_ERR = 2.0 ** -11


@pytest.fixture(scope="module")
def ctx():
    return rg.Context(3072, 24, 128, 12288, 1024, 4096)


def _bf16(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)


def _rows(rng, rows, cols):
    """bf16-representable rows with the features that stress the quantiser: wide dynamic range inside a row, an all-zero
    row, a negative extreme, values far below the row's scale (subnormal and zero codes), exact ties."""
    x = rng.normal(0, 1, (rows, cols)) * np.exp2(rng.integers(-6, 3, (rows, cols)))
    if rows > 1:
        x[1] = 0.0
    if rows > 2:
        x[2] = rng.normal(0, 1e-3, cols)
        x[2, cols // 3] = -50.0
    if rows > 3:
        x[3] = np.exp2(rng.integers(-20, 4, cols)) * rng.choice([-1.0, 1.0], cols)
        x[3, 0] = 14.0                      # amax 14: multiplier 32, every power of two lands on a code or a tie
    if rows > 4:
        x[4] = 448.0 * rng.choice([0.0625 * 17 / 16, 0.0625 * 19 / 16, 1.0, -1.0, 2.0 ** -12, 3 * 2.0 ** -11], cols)
    return _bf16(x)


@pytest.mark.parametrize("rows,cols", [(1, 8), (7, 64), (130, 3072), (9, 12288), (33, 16384), (5, 4104), (1025, 512), (4100, 3072), (6, 2048)])
def test_quantize_rows_bit_exact(ctx, rows, cols):
    rng = np.random.default_rng(rows * 31 + cols)
    x = _rows(rng, rows, cols)
    want_q, want_s = f8.quantize_rows(x.float().numpy())
    xd = x.cuda()
    q = torch.full((rows, cols), 0x55, dtype=torch.uint8, device="cuda")
    s = torch.full((rows,), -1.0, dtype=torch.float32, device="cuda")
    rg.regione_quantize_rows_fp8(ctx, xd, rows, cols, q, s)
    torch.cuda.synchronize()
    got_q, got_s = q.cpu().numpy(), s.cpu().numpy()
    assert np.array_equal(got_s.view(np.uint32), want_s.view(np.uint32)), "scales differ"
    bad = np.argwhere(got_q != want_q)
    assert len(bad) == 0, f"{len(bad)} codes differ, first at {bad[0]}: got {got_q[tuple(bad[0])]:#x}, want {want_q[tuple(bad[0])]:#x}, x {x.float().numpy()[tuple(bad[0])]!r}"


def _codes(rng, rows, cols):
    """Random finite E4M3 codes (all exponents, both signs, zeros and subnormals included)."""
    c = rng.integers(0, 256, (rows, cols)).astype(np.uint8)
    c[(c & 0x7F) == 0x7F] = 0x38
    return c


def _linear_case(ctx, rng, m, n, k, act, out_dtype, tn, splits, bias=True):
    xq, wq = _codes(rng, m, k), _codes(rng, n, k)
    # mostly moderate magnitudes, so that sums do not vanish against one huge product
    xq[:, ::3] = (xq[:, ::3] & 0x87) | 0x30
    wq[:, 1::2] = (wq[:, 1::2] & 0x87) | 0x28
    sx = rng.uniform(0.5, 2.0, m).astype(np.float32) / 64
    sw = rng.uniform(0.5, 2.0, n).astype(np.float32) / 64
    b = rng.normal(0, 1, n).astype(np.float32) if bias else None
    want = f8.linear_fp8(xq, sx, wq, sw, b)
    mag = (np.abs(f8.e4m3_decode(xq)) @ np.abs(f8.e4m3_decode(wq)).T) * sx[:, None].astype(np.float64) * sw[None, :]
    if act == rg.ACT_GELU_TANH:
        from oracle import regione_oracle as orc
        want = orc.gelu_tanh(want)
    wq_d = torch.from_numpy(wq).cuda()
    packed = torch.zeros(rg.regione_packed_weight_elems(n, k), dtype=torch.uint8, device="cuda")
    rg.regione_pack_weight_fp8(ctx, wq_d, n, k, packed)
    y = torch.full((m, n), 7.0, dtype=torch.float32 if out_dtype == rg.FP32 else torch.bfloat16, device="cuda")
    rg.regione_tune_gemm(ctx, tn, splits)
    try:
        rg.regione_linear_fp8(ctx, torch.from_numpy(xq).cuda(), torch.from_numpy(sx).cuda(), packed, torch.from_numpy(sw).cuda(),
                              None if b is None else torch.from_numpy(b).cuda(), m, n, k, act, out_dtype, y)
        torch.cuda.synchronize()
    finally:
        rg.regione_tune_gemm(ctx, 0, 0)
    got = y.float().cpu().numpy().astype(np.float64)
    bound = mag * MFMA_SUM_ERR + np.abs(want) * 2.0 ** -22 + 1e-30
    if out_dtype == rg.BF16:
        bound = bound + gu.half_ulp_bf16(want) * 1.01
    err = np.abs(got - want)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert np.all(err <= bound), f"m {m} n {n} k {k} tn {tn} splits {splits}: worst at {worst}: got {got[worst]!r} want {want[worst]!r} bound {bound[worst]:.3e}"


@pytest.mark.parametrize("m,n,k", [(1, 32, 128), (127, 200, 384), (129, 1000, 1024), (300, 100, 256), (260, 520, 2048)])
@pytest.mark.parametrize("tn,splits", [(1, 1), (2, 1), (1, 3), (2, 2), (0, 0)])
def test_linear_fp8_matches_oracle(ctx, m, n, k, tn, splits):
    if splits > 1 and k // 128 < splits:
        pytest.skip("fewer K steps than splits")
    rng = np.random.default_rng(m * 7 + n * 3 + k + tn * 11 + splits)
    _linear_case(ctx, rng, m, n, k, rg.ACT_NONE, rg.FP32, tn, splits)


def test_linear_fp8_epilogue_forms(ctx):
    rng = np.random.default_rng(77)
    _linear_case(ctx, rng, 140, 256, 512, rg.ACT_GELU_TANH, rg.BF16, 0, 0)
    _linear_case(ctx, rng, 140, 256, 512, rg.ACT_NONE, rg.BF16, 2, 2, bias=False)
    _linear_case(ctx, rng, 70, 36, 128, rg.ACT_GELU_TANH, rg.FP32, 1, 1)     # n not a multiple of 8: element-wise epilogue


def test_quantise_pack_multiply_end_to_end(ctx):
    """The whole recipe on the device (quantise activations and weights, pack, multiply) against the oracle's recipe,
    and its distance from the unquantised product."""
    rng = np.random.default_rng(3)
    m, n, k = 333, 640, 3072
    x = _bf16(rng.normal(0, 1, (m, k)))
    w = _bf16(rng.normal(0, 0.02, (n, k)))
    xq_o, sx_o = f8.quantize_rows(x.float().numpy())
    wq_o, sw_o = f8.quantize_rows(w.float().numpy())
    want = f8.linear_fp8(xq_o, sx_o, wq_o, sw_o)
    xq = torch.empty((m, k), dtype=torch.uint8, device="cuda"); sx = torch.empty(m, dtype=torch.float32, device="cuda")
    wq = torch.empty((n, k), dtype=torch.uint8, device="cuda"); sw = torch.empty(n, dtype=torch.float32, device="cuda")
    rg.regione_quantize_rows_fp8(ctx, x.cuda(), m, k, xq, sx)
    rg.regione_quantize_rows_fp8(ctx, w.cuda(), n, k, wq, sw)
    packed = torch.zeros(rg.regione_packed_weight_elems(n, k), dtype=torch.uint8, device="cuda")
    rg.regione_pack_weight_fp8(ctx, wq, n, k, packed)
    y = torch.empty((m, n), dtype=torch.float32, device="cuda")
    rg.regione_linear_fp8(ctx, xq, sx, packed, sw, None, m, n, k, rg.ACT_NONE, rg.FP32, y)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    mag = (np.abs(f8.e4m3_decode(xq_o)) @ np.abs(f8.e4m3_decode(wq_o)).T) * sx_o[:, None].astype(np.float64) * sw_o[None, :]
    assert np.all(np.abs(got - want) <= mag * MFMA_SUM_ERR)
    # typical data has no dominant product: the error stays orders of magnitude inside the worst-case bound
    assert np.max(np.abs(got - want)) <= 2e-3 and gu.mean_rel(got, want) < 1e-4, (np.max(np.abs(got - want)), gu.mean_rel(got, want))
    exact = x.float().numpy().astype(np.float64) @ w.float().numpy().astype(np.float64).T
    rel = np.linalg.norm(got - exact) / np.linalg.norm(exact)
    assert 1e-3 < rel < 0.06, rel      # two 3-bit mantissas: a few per cent, stated as the variant's accuracy


def test_linear_fp8_full_width_sampled(ctx):
    """The QKV projection of the headline workload (820 x 9216 x 3072) in the configuration the planner picks; sampled
    outputs against the oracle computed one by one."""
    rng = np.random.default_rng(11)
    m, n, k = 820, 9216, 3072
    xq, wq = _codes(rng, m, k), _codes(rng, n, k)
    xq = (xq & 0x87) | 0x30
    wq = (wq & 0x87) | 0x28
    sx = rng.uniform(0.5, 2.0, m).astype(np.float32) / 64
    sw = rng.uniform(0.5, 2.0, n).astype(np.float32) / 64
    packed = torch.zeros(rg.regione_packed_weight_elems(n, k), dtype=torch.uint8, device="cuda")
    rg.regione_pack_weight_fp8(ctx, torch.from_numpy(wq).cuda(), n, k, packed)
    y = torch.empty((m, n), dtype=torch.float32, device="cuda")
    rg.regione_linear_fp8(ctx, torch.from_numpy(xq).cuda(), torch.from_numpy(sx).cuda(), packed, torch.from_numpy(sw).cuda(), None,
                          m, n, k, rg.ACT_NONE, rg.FP32, y)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    rows = np.concatenate([[0, 127, 128, 819], rng.integers(0, m, 12)])
    cols = np.concatenate([[0, 31, 32, 9215], rng.integers(0, n, 60)])
    want = f8.linear_fp8(xq[rows], sx[rows], wq[cols], sw[cols])
    mag = (np.abs(f8.e4m3_decode(xq[rows])) @ np.abs(f8.e4m3_decode(wq[cols])).T) * sx[rows][:, None].astype(np.float64) * sw[cols][None, :]
    assert np.all(np.abs(got[np.ix_(rows, cols)] - want) <= mag * MFMA_SUM_ERR + 1e-30)


def test_fp8_argument_errors(ctx):
    x = torch.zeros((4, 100), dtype=torch.bfloat16, device="cuda")
    q = torch.zeros((4, 100), dtype=torch.uint8, device="cuda")
    s = torch.zeros(4, dtype=torch.float32, device="cuda")
    with pytest.raises(rg.RegionEError):
        rg.regione_quantize_rows_fp8(ctx, x, 4, 100, q, s)          # cols not a multiple of 8
    with pytest.raises(rg.RegionEError):
        rg.regione_pack_weight_fp8(ctx, q, 4, 64, q)                # k not a multiple of 128
    y = torch.zeros((4, 32), dtype=torch.float32, device="cuda")
    with pytest.raises(rg.RegionEError):
        rg.regione_linear_fp8(ctx, q, s, q, None, None, 4, 32, 128, rg.ACT_NONE, rg.FP32, y)   # missing weight scales
    with pytest.raises(rg.RegionEError):
        rg.regione_linear_fp8(ctx, q, s, q, s, None, 4, 32, 192, rg.ACT_NONE, rg.FP32, y)      # k not a multiple of 128


def test_mfma_peak_probe_runs_and_reports_its_work(ctx):
    """The measurement aid: finite, reproducible output and the stated operation count; bad arguments are refused."""
    out = torch.full((4 * 256,), float("nan"), dtype=torch.float32, device="cuda")
    for fmt, k in ((0, 16), (1, 64)):
        flops = rg.regione_mfma_peak_probe(ctx, fmt, 5, 4, out)
        torch.cuda.synchronize()
        first = out.clone()
        assert flops == 4 * 4 * 5 * 4 * 2 * 32 * 32 * k
        assert bool(torch.isfinite(first).all()) and float(first.abs().max()) > 0
        rg.regione_mfma_peak_probe(ctx, fmt, 5, 4, out)
        torch.cuda.synchronize()
        assert torch.equal(out, first)
    for bad in ((2, 5, 4), (0, 0, 4), (0, 5, 0)):
        with pytest.raises(rg.RegionEError):
            rg.regione_mfma_peak_probe(ctx, *bad, out)


def test_linear_fp8_is_reproducible(ctx):
    """No atomics, fixed summation order: two runs (with another shape in between) give identical bits, with and
    without a K split."""
    rng = np.random.default_rng(21)
    m, n, k = 300, 1024, 2048
    xq = torch.from_numpy(_codes(rng, m, k)).cuda(); wq = torch.from_numpy(_codes(rng, n, k)).cuda()
    sx = torch.from_numpy(rng.uniform(0.5, 2, m).astype(np.float32)).cuda(); sw = torch.from_numpy(rng.uniform(0.5, 2, n).astype(np.float32)).cuda()
    packed = torch.zeros(rg.regione_packed_weight_elems(n, k), dtype=torch.uint8, device="cuda")
    rg.regione_pack_weight_fp8(ctx, wq, n, k, packed)
    for tn, splits in ((0, 0), (1, 4), (2, 2)):
        outs = []
        for rep in range(3):
            y = torch.full((m, n), 3.0, dtype=torch.float32, device="cuda")
            rg.regione_tune_gemm(ctx, tn, splits)
            try:
                rg.regione_linear_fp8(ctx, xq, sx, packed, sw, None, m, n, k, rg.ACT_NONE, rg.FP32, y)
                other = torch.empty((100, n), dtype=torch.float32, device="cuda")
                rg.regione_linear_fp8(ctx, xq, sx, packed, sw, None, 100, n, k, rg.ACT_NONE, rg.FP32, other)
            finally:
                rg.regione_tune_gemm(ctx, 0, 0)
            torch.cuda.synchronize()
            outs.append(y)
        assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2]), (tn, splits)
