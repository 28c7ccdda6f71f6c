"""Pins for the oracle's conditioning path: SiLU, the one-vector linear layer and the sinusoidal
embedding, against torch's library routines, closed forms and hand cases."""
import math

import numpy as np
import pytest
import torch

from oracle import regione_oracle as orc


def test_silu_against_torch_and_closed_values():
    x = np.linspace(-20, 20, 401)
    want = torch.nn.functional.silu(torch.from_numpy(x)).numpy()
    assert np.allclose(orc.silu(x), want, rtol=1e-13, atol=1e-15)
    assert orc.silu(np.array([0.0]))[0] == 0.0
    assert math.isclose(orc.silu(np.array([1.0]))[0], 1.0 / (1.0 + math.exp(-1.0)), rel_tol=1e-15)
    # silu(x) - silu(-x) = x
    assert np.allclose(orc.silu(x) - orc.silu(-x), x, atol=1e-12)


def test_vec_linear_against_torch_linear():
    rng = np.random.default_rng(1)
    x = rng.normal(size=96)
    w = rng.normal(size=(40, 96))
    b = rng.normal(size=40)
    want = torch.nn.functional.linear(torch.nn.functional.silu(torch.from_numpy(x)), torch.from_numpy(w), torch.from_numpy(b)).numpy()
    assert np.allclose(orc.vec_linear(x, w, b, "silu"), want, rtol=1e-12, atol=1e-12)
    want = torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(w)).numpy()
    assert np.allclose(orc.vec_linear(x, w), want, rtol=1e-12, atol=1e-12)
    with pytest.raises(ValueError):
        orc.vec_linear(x, w, b, "relu")


def test_vec_linear_hand_case_catches_a_transposed_operand():
    w = np.array([[1.0, 2.0, 3.0], [0.0, -1.0, 4.0]])
    assert np.array_equal(orc.vec_linear(np.array([1.0, 1.0, 2.0]), w, np.array([10.0, 20.0])), [19.0, 27.0])


def test_timestep_embedding_closed_forms():
    e = orc.timestep_embedding(0.0, 8)
    assert np.array_equal(e, [1, 1, 1, 1, 0, 0, 0, 0])
    e = orc.timestep_embedding(2.5, 8, max_period=10000.0)
    for j in range(4):
        f = 10000.0 ** (-j / 4)
        assert math.isclose(e[j], math.cos(2.5 * f), rel_tol=1e-14, abs_tol=1e-15)
        assert math.isclose(e[4 + j], math.sin(2.5 * f), rel_tol=1e-14, abs_tol=1e-15)
    # first frequency is 1: the pair (cos t, sin t)
    e = orc.timestep_embedding(math.pi / 2, 4)
    assert abs(e[0]) < 1e-15 and math.isclose(e[2], 1.0)
    # every (cos, sin) pair has unit norm
    e = orc.timestep_embedding(731.25, 256)
    assert np.allclose(e[:128] ** 2 + e[128:] ** 2, 1.0, atol=1e-14)
    with pytest.raises(ValueError):
        orc.timestep_embedding(1.0, 7)
