"""Pins for the oracle's query/key normalisation and rotary embedding: closed forms, invariants
and the complex-number form of the rotation, none of which repeats the oracle's own expression."""
import cmath
import math

import numpy as np
import pytest
import torch

from oracle import regione_oracle as orc


def test_rms_norm_hand_case_and_unit_rms():
    y = orc.rms_norm(np.array([[3.0, 4.0]]), eps=0.0)
    assert np.allclose(y, [[3.0 / math.sqrt(12.5), 4.0 / math.sqrt(12.5)]], rtol=0, atol=1e-15)
    rng = np.random.default_rng(1)
    x = rng.normal(size=(5, 3, 64)) * 7.0
    y = orc.rms_norm(x, eps=0.0)
    assert np.allclose(np.sqrt((y ** 2).mean(axis=-1)), 1.0, atol=1e-12)
    # positive scaling of the input does not change the result; a weight multiplies element-wise
    assert np.allclose(orc.rms_norm(3.5 * x, eps=0.0), y, atol=1e-12)
    w = rng.normal(size=64)
    assert np.allclose(orc.rms_norm(x, w, eps=0.0), y * w, atol=1e-12)


def test_rms_norm_matches_torch_library_routine():
    rng = np.random.default_rng(2)
    x = rng.normal(size=(7, 4, 128))
    w = rng.normal(size=128)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (128,), torch.from_numpy(w), eps=1e-6).numpy()
    assert np.allclose(orc.rms_norm(x, w, eps=1e-6), want, rtol=1e-12, atol=1e-12)


def test_rms_norm_eps_decides_the_zero_vector():
    assert np.all(orc.rms_norm(np.zeros((1, 8)), eps=1e-6) == 0.0)


def test_rope_angles_frequencies_and_axis_layout():
    # one axis: pair j turns by pos * theta^(-2j/a); first pair by pos itself
    ang = orc.rope_angles(np.array([[5]]), [8], theta=10000.0)
    assert ang.shape == (1, 4)
    assert ang[0, 0] == 5.0
    assert math.isclose(ang[0, 1], 5.0 * 10000.0 ** (-0.25), rel_tol=1e-15)
    assert math.isclose(ang[0, 3], 5.0 * 10000.0 ** (-0.75), rel_tol=1e-15)
    # three axes: each owns its own run of pairs and sees only its own coordinate
    ang = orc.rope_angles(np.array([[0, 3, 7]]), [4, 6, 6])
    assert ang.shape == (1, 8)
    assert np.all(ang[0, :2] == 0.0)
    assert ang[0, 2] == 3.0 and ang[0, 5] == 7.0
    assert math.isclose(ang[0, 4], 3.0 * 10000.0 ** (-4.0 / 6.0), rel_tol=1e-15)
    with pytest.raises(ValueError):
        orc.rope_angles(np.array([[1]]), [3])


def test_rope_is_complex_multiplication_of_interleaved_pairs():
    rng = np.random.default_rng(3)
    x = rng.normal(size=(4, 2, 8))
    ang = rng.normal(size=(4, 4)) * 3.0
    y = orc.rope_apply(x, ang)
    for n in range(4):
        for h in range(2):
            for j in range(4):
                z = complex(x[n, h, 2 * j], x[n, h, 2 * j + 1]) * cmath.exp(1j * ang[n, j])
                assert math.isclose(y[n, h, 2 * j], z.real, rel_tol=0, abs_tol=1e-14)
                assert math.isclose(y[n, h, 2 * j + 1], z.imag, rel_tol=0, abs_tol=1e-14)


def test_rope_quarter_turn_and_identity():
    x = np.array([[[1.0, 0.0, 0.0, 2.0]]])
    y = orc.rope_apply(x, np.array([[math.pi / 2, math.pi / 2]]))
    assert np.allclose(y, [[[0.0, 1.0, -2.0, 0.0]]], atol=1e-15)
    assert np.array_equal(orc.rope_apply(x, np.zeros((1, 2))), x)


def test_rope_keeps_norms_and_makes_scores_depend_on_relative_position():
    rng = np.random.default_rng(4)
    q = rng.normal(size=(1, 1, 16))
    k = rng.normal(size=(1, 1, 16))
    axes = [4, 6, 6]

    def score(pq, pk):
        a = orc.rope_apply(q, orc.rope_angles(np.array([pq]), axes))
        b = orc.rope_apply(k, orc.rope_angles(np.array([pk]), axes))
        return float((a * b).sum())

    assert math.isclose(score([0, 5, 9], [0, 2, 4]), score([0, 15, 12], [0, 12, 7]), rel_tol=1e-12)
    assert not math.isclose(score([0, 5, 9], [0, 2, 4]), score([0, 5, 9], [0, 3, 4]), rel_tol=1e-6)
    y = orc.rope_apply(q, orc.rope_angles(np.array([[1, 2, 3]]), axes))
    assert math.isclose(float((y ** 2).sum()), float((q ** 2).sum()), rel_tol=1e-13)


def _stream(rng, hidden, mlp, d, norm):
    w = {"w_qkv": rng.normal(size=(3 * hidden, hidden)) * 0.2, "b_qkv": rng.normal(size=3 * hidden) * 0.1,
         "w_o": rng.normal(size=(hidden, hidden)) * 0.2, "b_o": None,
         "w_1": rng.normal(size=(mlp, hidden)) * 0.2, "b_1": None,
         "w_2": rng.normal(size=(hidden, mlp)) * 0.2, "b_2": None}
    if norm:
        w["q_norm"] = 1.0 + 0.1 * rng.normal(size=d)
        w["k_norm"] = 1.0 + 0.1 * rng.normal(size=d)
    return w


def test_block_extras_gathered_rows_keep_their_positions():
    """With every cache row refreshed Eq.6 is plain attention, so a retrieve call over a PERMUTED
    list of all rows must reproduce the full forward row by row; it can only do so if each fresh
    row takes the angles of its own slot."""
    rng = np.random.default_rng(5)
    hidden, heads, mlp, n = 16, 2, 32, 12
    d = hidden // heads
    streams = [_stream(rng, hidden, mlp, d, True)]
    h = rng.normal(size=(n, hidden))
    rope = orc.rope_angles(np.stack([np.zeros(n), np.arange(n) // 4, np.arange(n) % 4], axis=1), [2, 4, 2])
    kc, vc = np.zeros((n, heads, d)), np.zeros((n, heads, d))
    full = orc.block_forward(streams, "double", h, 0, np.arange(n), kc, vc, orc.FLAG_STORE, heads, rope=rope)
    perm = rng.permutation(n)
    kc2, vc2 = kc.copy(), vc.copy()
    got = orc.block_forward(streams, "double", h[perm], 0, perm, kc2, vc2, orc.FLAG_RETRIEVE, heads, rope=rope)
    assert np.allclose(got, full[perm], rtol=1e-10, atol=1e-12)
    # and the extras do change the result
    plain = orc.block_forward([_strip(streams[0])], "double", h, 0, np.arange(n), kc.copy(), vc.copy(), orc.FLAG_STORE, heads)
    assert not np.allclose(plain, full, atol=1e-3)


def _strip(w):
    return {k: v for k, v in w.items() if k not in ("q_norm", "k_norm")}


def test_block_extras_cached_keys_are_normalised_and_rotated():
    rng = np.random.default_rng(6)
    hidden, heads, mlp, n = 8, 1, 16, 5
    streams = [_stream(rng, hidden, mlp, 8, True)]
    h = rng.normal(size=(n, hidden))
    rope = orc.rope_angles(np.arange(n)[:, None], [8])
    kc, vc = np.zeros((n, heads, 8)), np.zeros((n, heads, 8))
    _, q3, k3, v3 = orc.block_forward(streams, "double", h, 0, np.arange(n), kc, vc, orc.FLAG_STORE, heads, return_qkv=True, rope=rope)
    assert np.array_equal(kc, k3) and np.array_equal(vc, v3)
    # keys: unit RMS before the weight; undo weight and rotation to see it
    unrot = orc.rope_apply(k3, -rope)
    assert np.allclose(np.sqrt(((unrot / streams[0]["k_norm"]) ** 2).mean(axis=-1)), 1.0, atol=1e-4)
