"""Pins for the oracle's adaptive region partition, gather and scatter (CPU only).

What fixes the expected values: Eq.2 + Eq.5 of the paper (a straight trajectory is
recovered exactly by the one-step estimate), hand-computed cosine cases, torch's
cosine_similarity as an independent library routine, and brute-force list building.
"""
import numpy as np
import pytest
import torch

from oracle import regione_oracle as orc
from paper_2510_25590_amd import inputs


def test_one_step_estimate_recovers_x0_on_straight_trajectory():
    # Eq.2: X_t = (1-t) X_0 + t X_1, dX/dt = X_1 - X_0  =>  Eq.5 with t_f = 0 gives X_0.
    # Dyadic values keep every float32 operation exact, so equality is exact.
    rng = np.random.default_rng(0)
    x0 = rng.integers(-8, 9, size=(50, 16)).astype(np.float32) / 4
    x1 = rng.integers(-8, 9, size=(50, 16)).astype(np.float32) / 4
    for t in (0.25, 0.5, 0.75):
        x_t = ((1 - t) * x0 + t * x1).astype(np.float32)
        v = x1 - x0
        est = orc.one_step_estimate_f32(x_t, v, t)
        assert np.array_equal(est, x0)
        s = orc.cosine_scores(est, x0)
        nz = np.abs(x0).sum(axis=1) > 0
        assert np.allclose(s[nz], 1.0, atol=1e-7)


def test_one_step_estimate_sign_and_operand_order():
    # x_t - dt*v, not x_t + dt*v, not v - dt*x_t
    est = orc.one_step_estimate_f32(np.array([[3.0, 1.0]]), np.array([[2.0, -4.0]]), 0.5)
    assert np.array_equal(est, np.array([[2.0, 3.0]], dtype=np.float32))


def test_cosine_hand_cases():
    a = np.array([[1, 2, 3, 4], [1, 0, 0, 0], [1, 2, 3, 4], [0, 0, 0, 0], [3, 4, 0, 0]], dtype=np.float32)
    b = np.array([[2, 4, 6, 8], [0, 5, 0, 0], [-1, -2, -3, -4], [1, 1, 1, 1], [4, 3, 0, 0]], dtype=np.float32)
    s = orc.cosine_scores(a, b)
    assert s.dtype == np.float32
    assert s[0] == pytest.approx(1.0, abs=1e-7)      # parallel
    assert s[1] == 0.0                                # orthogonal
    assert s[2] == pytest.approx(-1.0, abs=1e-7)      # antiparallel
    assert s[3] == 0.0                                # zero vector -> 0 through eps
    assert s[4] == np.float32(24.0 / 25.0)            # 3-4-5: exact norms


def test_cosine_matches_torch_library():
    rng = np.random.default_rng(1)
    a = rng.standard_normal((300, 64))
    b = rng.standard_normal((300, 64))
    ref = torch.nn.functional.cosine_similarity(torch.from_numpy(a), torch.from_numpy(b), dim=1, eps=1e-8).numpy()
    s = orc.cosine_scores(a, b)
    assert np.max(np.abs(s.astype(np.float64) - ref)) < 1e-7
    # asymmetric inputs: swapping which side is normalised must not matter, scaling one side must not matter
    assert np.max(np.abs(orc.cosine_scores(3 * a, b) - s)) < 1e-6


def test_threshold_is_strict_and_nan_is_edited():
    score = np.array([0.95, 0.9, np.nextafter(np.float32(0.9), np.float32(1)), 0.1, np.nan], dtype=np.float32)
    m = orc.threshold_mask(score, 0.9)
    # float32(0.9) compared with float32(0.9): equal -> edited
    assert m.tolist() == [0, 1, 0, 1, 1]


def test_compact_brute_force_and_invariants():
    rng = np.random.default_rng(2)
    for n in (1, 63, 64, 65, 1000):
        for p in (0.0, 0.3, 1.0):
            mask = (rng.random(n) < p).astype(np.uint8)
            e, u = orc.compact(mask)
            assert e.dtype == np.int32 and u.dtype == np.int32
            assert e.tolist() == np.nonzero(mask)[0].tolist()
            assert u.tolist() == np.nonzero(mask == 0)[0].tolist()
            assert len(e) + len(u) == n and len(np.intersect1d(e, u)) == 0
            assert np.all(np.diff(e) > 0) and np.all(np.diff(u) > 0)


def test_config1_partition_returns_exactly_the_rectangle():
    # 16x16 grid, 6x6 rectangle perturbed, sigma 0.7, eta 0.9 (first benchmark configuration)
    rng = np.random.default_rng(inputs.workload_seed(1))
    want = inputs.rect_mask(rng, 16, 16, 6, 6)
    x_t, v, ref = inputs.latents_for_mask(rng, want, 64, 0.7, "f32")
    score, mask, e, u = orc.partition(x_t, v, ref, 0.7, 0.9)
    assert int(want.sum()) == 36
    assert np.array_equal(mask.astype(bool), want)
    assert e.tolist() == np.nonzero(want)[0].tolist() and len(e) == 36
    # margin that makes the mask independent of summation order in any float32/64 evaluation
    assert np.min(np.abs(score - np.float32(0.9))) > 1e-3
    assert score[~want].min() > 0.99 and score[want].max() < 0.88


def test_partition_bf16_inputs_have_margin():
    rng = np.random.default_rng(inputs.workload_seed(2))
    want = inputs.rect_mask_fraction(rng, 64, 64, 819)
    assert abs(int(want.sum()) - 819) <= 4
    x_t, v, ref = inputs.latents_for_mask(rng, want, 64, 0.7, "bf16")
    score, mask, e, u = orc.partition(x_t, v, ref, 0.7, 0.9)
    assert np.array_equal(mask.astype(bool), want)
    assert np.min(np.abs(score - np.float32(0.9))) > 1e-3


def test_gather_scatter_roundtrip_bit_identical():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((100, 8)).astype(np.float32)
    mask = rng.random(100) < 0.3
    e, u = orc.compact(mask.astype(np.uint8))
    g = orc.gather(x, e)
    assert np.array_equal(g, x[mask])
    y = x.copy()
    orc.scatter(y, e, g + 1.0)
    assert np.array_equal(y[~mask].view(np.uint32), x[~mask].view(np.uint32))  # unedited rows untouched
    assert np.array_equal(y[mask], x[mask] + 1.0)
    ident = np.arange(100, dtype=np.int32)
    assert np.array_equal(orc.gather(x, ident), x)
    perm = rng.permutation(100).astype(np.int32)
    z = np.zeros_like(x)
    orc.scatter(z, perm, orc.gather(x, perm))
    assert np.array_equal(z, x)


def test_blob_mask_has_exact_count():
    rng = np.random.default_rng(4)
    for n_e in (0, 1, 205, 819, 2048, 4096):
        assert int(inputs.blob_mask(rng, 64, 64, n_e).sum()) == n_e


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1e-40], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 (even mantissa) and 1 + 2^-7 -> 1.0 ; 1 + 3*2^-8 ties to 1 + 2^-6
    r = inputs.bf16_round(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.015625 and r[3] == -2.5
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r.view(np.uint32), t.view(np.uint32))
    rng = np.random.default_rng(5)
    y = rng.standard_normal(10000).astype(np.float32)
    assert np.array_equal(inputs.bf16_round(y), torch.from_numpy(y).to(torch.bfloat16).to(torch.float32).numpy())
