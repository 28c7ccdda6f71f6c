"""CPU oracle for the 8-bit floating point variant of the dense projections.

TEST INFRASTRUCTURE ONLY (see regione_oracle.py): the product never imports this file and
this file imports nothing from the product.

The paper (arXiv 2510.25590) does not use 8-bit arithmetic; this variant is an extension of
its dense projections (section "Region-Aware Generation": the DiT runs on the edited rows),
so no passage of the paper defines what is computed here.  What fixes it instead:

  * the number format is E4M3 of the public OCP 8-bit floating point specification
    (sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities; S.1111.111 is NaN;
    largest finite value 448 = 0x7E; subnormals m * 2^-9);
  * the quantisation recipe is this build's own: every row of the activations and every row
    (output channel) of the weights gets one float32 scale, amax / 448, and its elements are
    multiplied by 448 / amax in float32, clamped to +-448 and rounded to the nearest E4M3
    value, ties to the even code.  The decision which code a value gets is taken in float32,
    the precision the kernel takes it in;
  * the product is the plain sum over k of the decoded values times both scales, plus bias,
    in float64.

Parity pins (tests/test_oracle_fp8.py): code values the format's definition fixes, brute
force nearest-value search with ties to even over the whole code table, the round trip of
all codes, powers of two scaling, the error bound of a 3-bit mantissa, and exact integer
matrix products; e4m3_half_step against the gaps of the decoded code table.

The 8-bit form of a whole block (regione_block_forward_fp8) has no reference of its own: it is checked stage by
stage with the functions of this file and of regione_oracle.py on the library's own input of every stage
(tests/test_gpu_block_fp8.py), because a block that quantises its own intermediates differs from any other
implementation by whole code steps wherever an input sits on a rounding boundary.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_decode(codes) -> np.ndarray:
    """Value of every E4M3 code (uint8) as float64; 0x7F and 0xFF decode to NaN."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = (c & 0x7).astype(np.float64)
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    subnormal = (m / 8.0) * 2.0 ** -6
    val = sign * np.where(e == 0, subnormal, normal)
    return np.where((c & 0x7F) == 0x7F, np.nan, val)


def e4m3_encode(values) -> np.ndarray:
    """Finite values (taken as float32) -> E4M3 codes: clamp to +-448, round to the nearest
    representable value, ties to the even code; the sign of a zero is kept."""
    x = np.asarray(values, dtype=np.float32).astype(np.float64)   # exact widening
    neg = np.signbit(x)
    a = np.minimum(np.abs(x), E4M3_MAX)
    # spacing of the E4M3 values around a: 2^(floor(log2 a) - 3) for normals, 2^-9 below 2^-6
    e = np.frexp(a)[1].astype(np.float64) - 1.0   # a = f * 2^(e+1) with f in [0.5, 1): e = floor(log2 a), exact
    e = np.maximum(e, -6.0)                       # (frexp gives 0 for a = 0; the clamp covers it)
    step = np.exp2(e - 3.0)
    n = np.rint(a / step)            # a / step is exact (power of two); rint rounds half to even
    # code of r: for normals mantissa = n - 8 at exponent e, carry into the next exponent when n = 16
    carry = n >= 16
    e2 = np.where(carry, e + 1, e)
    n2 = np.where(carry, 8.0, n)
    is_sub = n2 < 8                  # only possible at e = -6
    code = np.where(is_sub, n2, (e2 + 7) * 8 + (n2 - 8)).astype(np.int64)
    assert np.all(code <= 0x7E), "clamped input cannot reach the NaN code"
    return (code | np.where(neg, 0x80, 0)).astype(np.uint8)


def e4m3_half_step(values) -> np.ndarray:
    """Half the distance between the neighbouring E4M3 values around |v| (|v| <= 448): what rounding to the format may
    move a value by.  Spacing 2^(floor(log2 |v|) - 3) for normals, 2^-9 below 2^-6."""
    a = np.maximum(np.abs(np.asarray(values, dtype=np.float64)), 2.0 ** -9)
    e = np.maximum(np.floor(np.log2(a)), -6.0)
    return np.exp2(e - 3.0) / 2.0


def quantize_rows(x):
    """Per-row quantisation of a matrix of float32-representable values.
    Returns (codes uint8 [rows, cols], scale float32 [rows]) with x ~ scale * decode(codes).
    amax = max |x| of the row; scale = amax / 448 and the multiplier 448 / amax are both
    float32 quotients; the product x * multiplier is a float32 product.  A row of zeros
    has scale 1."""
    x32 = np.asarray(x, dtype=np.float32)
    amax = np.max(np.abs(x32), axis=1) if x32.shape[1] else np.zeros(x32.shape[0], dtype=np.float32)
    live = amax > 0
    safe = np.where(live, amax, np.float32(1.0)).astype(np.float32)
    scale = np.where(live, safe / np.float32(E4M3_MAX), np.float32(1.0)).astype(np.float32)
    mult = np.where(live, np.float32(E4M3_MAX) / safe, np.float32(1.0)).astype(np.float32)
    y = (x32 * mult[:, None]).astype(np.float32)
    return e4m3_encode(y), scale


def linear_fp8(x_codes, x_scale, w_codes, w_scale, b=None) -> np.ndarray:
    """y[m, n] = x_scale[m] * w_scale[n] * sum_k decode(x_codes[m, k]) * decode(w_codes[n, k]) + b[n], float64."""
    xd = e4m3_decode(x_codes)
    wd = e4m3_decode(w_codes)
    y = (xd @ wd.T) * np.asarray(x_scale, dtype=np.float64)[:, None] * np.asarray(w_scale, dtype=np.float64)[None, :]
    if b is not None:
        y = y + np.asarray(b, dtype=np.float64)[None, :]
    return y
