"""Pins of the 8-bit floating point oracle (oracle/fp8_reference.py) against what the E4M3 format's public
definition and plain arithmetic fix, none of them a re-run of the oracle's own formula."""
import numpy as np
import pytest

from oracle import fp8_reference as f8

ALL = np.arange(256, dtype=np.uint8)
FINITE = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)


def test_code_values_fixed_by_the_format():
    # sign | 4-bit exponent, bias 7 | 3-bit mantissa; the values below are the format's own examples and limits
    fixed = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x0F: 1.875 * 2.0 ** -6, 0x38: 1.0, 0x39: 1.125,
             0x40: 2.0, 0x3C: 1.5, 0x77: 240.0, 0x78: 256.0, 0x7E: 448.0, 0xB8: -1.0, 0xFE: -448.0, 0x81: -(2.0 ** -9)}
    for code, val in fixed.items():
        assert f8.e4m3_decode([code])[0] == val, hex(code)
    assert np.isnan(f8.e4m3_decode([0x7F, 0xFF])).all()
    assert not np.isnan(f8.e4m3_decode(FINITE)).any() and not np.isinf(f8.e4m3_decode(ALL[~np.isnan(f8.e4m3_decode(ALL))])).any()


def test_decode_is_strictly_increasing_with_gaps_of_one_mantissa_step():
    v = f8.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    d = np.diff(v)
    assert (d > 0).all()
    # within one exponent the gap is constant; it doubles from one exponent to the next (and is 2^-9 for exponents 0 and 1)
    for e in range(16):
        gaps = d[e * 8: min(e * 8 + 8, 0x7E)]
        assert np.all(gaps == 2.0 ** (max(e, 1) - 7 - 3)), e
    # negative half mirrors the positive
    assert np.array_equal(f8.e4m3_decode(np.arange(0x80, 0xFF, dtype=np.uint8)), -v)


def test_round_trip_of_every_code():
    assert np.array_equal(f8.e4m3_encode(f8.e4m3_decode(FINITE)), FINITE)


def _nearest_brute(x):
    """Nearest finite code by exhaustive search; of two equally near codes the even one."""
    pos = np.arange(0x7F, dtype=np.uint8)
    table = f8.e4m3_decode(pos)
    out = []
    for val in np.asarray(x, dtype=np.float64):
        a = min(abs(val), 448.0)
        dist = np.abs(table - a)
        best = np.flatnonzero(dist == dist.min())
        code = int(best[0]) if len(best) == 1 else int([b for b in best if b % 2 == 0][0])
        out.append(code | (0x80 if np.signbit(val) else 0))
    return np.array(out, dtype=np.uint8)


def test_encode_is_round_to_nearest_even_by_brute_force():
    rng = np.random.default_rng(5)
    table = f8.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    mids = (table[:-1] + table[1:]) / 2           # every tie of the format (exact in float32)
    near = np.concatenate([mids * (1 + 2.0 ** -20), mids * (1 - 2.0 ** -20)])
    rand = np.concatenate([rng.uniform(-460, 460, 4000), rng.normal(0, 1, 4000), rng.normal(0, 0.01, 4000), rng.uniform(-2.0 ** -6, 2.0 ** -6, 2000)])
    special = np.array([0.0, -0.0, 448.0, 449.0, 464.0, 479.9, 480.0, 1e6, -1e6, 2.0 ** -10, 2.0 ** -10 * 1.0001, 2.0 ** -10 * 0.9999, 1e-30, -1e-30])
    x = np.concatenate([mids, -mids, near, rand, special]).astype(np.float32)
    assert np.array_equal(f8.e4m3_encode(x), _nearest_brute(x.astype(np.float64)))


def test_encode_hand_cases():
    # ties: 1.0625 lies between 1.0 (0x38, even) and 1.125 (0x39) -> 0x38; 1.1875 between 0x39 and 0x3A -> 0x3A
    assert list(f8.e4m3_encode([1.0625, 1.1875, -1.0625, 2.0 ** -10, 3 * 2.0 ** -10, 1000.0, -0.0])) == [0x38, 0x3A, 0xB8, 0x00, 0x02, 0x7E, 0x80]


def test_error_bound_of_three_mantissa_bits():
    rng = np.random.default_rng(6)
    x = rng.uniform(2.0 ** -6, 448.0, 20000).astype(np.float32)
    back = f8.e4m3_decode(f8.e4m3_encode(x))
    assert np.max(np.abs(back - x) / x) <= 2.0 ** -4            # half a step of 2^-3 relative
    sub = rng.uniform(0, 2.0 ** -6, 2000).astype(np.float32)
    assert np.max(np.abs(f8.e4m3_decode(f8.e4m3_encode(sub)) - sub)) <= 2.0 ** -10


def test_half_step_equals_half_the_gap_of_the_code_table():
    vals = f8.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))        # 0 .. 448, increasing
    gaps = np.diff(vals)
    mid = (vals[:-1] + vals[1:]) / 2
    assert np.array_equal(f8.e4m3_half_step(mid), gaps / 2)                      # anywhere inside a gap
    assert np.array_equal(f8.e4m3_half_step(vals[1:-1] * 1.0001), gaps[1:] / 2)  # just above a code: the gap above it
    assert np.array_equal(f8.e4m3_half_step(-mid), gaps / 2)
    # rounding never moves a value by more than the half step there
    x = np.random.default_rng(5).uniform(-448, 448, 20000).astype(np.float32)
    err = np.abs(f8.e4m3_decode(f8.e4m3_encode(x)) - x.astype(np.float64))
    assert np.all(err <= f8.e4m3_half_step(x))


def test_quantize_rows_scale_and_codes():
    rng = np.random.default_rng(7)
    x = rng.normal(0, 1, (9, 64)).astype(np.float32)
    x[3] = 0.0
    x[4, 5] = -7.0                                             # the row's extreme is negative
    q, s = f8.quantize_rows(x)
    assert q.dtype == np.uint8 and s.dtype == np.float32
    amax = np.abs(x).max(axis=1)
    # the extreme of every row lands on +-448 exactly and the scale maps it back within float32 rounding
    for r in range(9):
        if amax[r] == 0:
            assert s[r] == 1.0 and not q[r].any()
            continue
        c = int(np.argmax(np.abs(x[r])))
        assert q[r, c] == (0xFE if x[r, c] < 0 else 0x7E)
        assert abs(float(s[r]) * 448.0 - amax[r]) <= amax[r] * 2.0 ** -23
    # reconstruction error: half a mantissa step relative to the value, or half a subnormal step of the scaled range
    back = f8.e4m3_decode(q) * s[:, None].astype(np.float64)
    bound = np.maximum(np.abs(x) * (2.0 ** -4 + 2.0 ** -20), (s[:, None] * 2.0 ** -10) * (1 + 2.0 ** -20))
    assert np.all(np.abs(back - x) <= bound)
    # scaling a row by a power of two changes the scale by that power and no code
    q2, s2 = f8.quantize_rows(x * 8.0)
    assert np.array_equal(q2, q) and np.array_equal(s2[amax > 0], s[amax > 0] * 8.0)


def test_linear_on_exact_integers():
    # small integers are E4M3 values: with unit scales the product is the integer matrix product
    rng = np.random.default_rng(8)
    xi = rng.integers(-8, 9, (5, 32))
    wi = rng.integers(-8, 9, (7, 32))
    xq, wq = f8.e4m3_encode(xi), f8.e4m3_encode(wi)
    assert np.array_equal(f8.e4m3_decode(xq), xi) and np.array_equal(f8.e4m3_decode(wq), wi)
    b = rng.normal(0, 1, 7)
    y = f8.linear_fp8(xq, np.ones(5, np.float32), wq, np.ones(7, np.float32), b)
    assert np.array_equal(y, (xi @ wi.T).astype(np.float64) + b[None, :])
    # scales multiply rows and columns
    sx, sw = rng.uniform(0.5, 2, 5).astype(np.float32), rng.uniform(0.5, 2, 7).astype(np.float32)
    y2 = f8.linear_fp8(xq, sx, wq, sw, None)
    np.testing.assert_allclose(y2, (xi @ wi.T) * sx[:, None].astype(np.float64) * sw[None, :].astype(np.float64), rtol=1e-15)


def test_quantised_linear_approximates_the_plain_one():
    # the whole recipe against the unquantised product: error of two 3-bit mantissas, averaged over k
    rng = np.random.default_rng(9)
    x = rng.normal(0, 1, (16, 256)).astype(np.float32)
    w = (rng.normal(0, 1, (24, 256)) / 16).astype(np.float32)
    xq, sx = f8.quantize_rows(x)
    wq, sw = f8.quantize_rows(w)
    y = f8.linear_fp8(xq, sx, wq, sw)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    assert rel < 0.05, rel
    assert rel > 1e-4      # and it IS quantised
