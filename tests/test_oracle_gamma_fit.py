"""Pins for the oracle's fit of the timestep-aware factor of Eq.7."""
import numpy as np

from oracle import regione_oracle as orc


def _schedule(T):
    return np.linspace(0.0, 1.0, T + 1)


def test_fit_recovers_the_factors_that_generated_the_norms():
    T, S = 12, 7
    rng = np.random.default_rng(1)
    t = _schedule(T) ** 1.5                      # uneven steps
    gamma = 1.0 + 0.1 * rng.standard_normal(T + 1)
    norms = np.zeros((S, T + 1))
    norms[:, T] = rng.uniform(1.0, 3.0, S)
    for j in range(T - 1, 0, -1):                # Eq.7 exactly, with a different scale per sample
        norms[:, j] = norms[:, j + 1] * orc.decay_factor(t, gamma, j)
    got = orc.fit_gamma(norms, t)
    assert np.allclose(got[1:T], gamma[1:T], rtol=1e-12)
    assert got[0] == 1.0 and got[T] == 1.0


def test_fit_is_the_least_squares_slope():
    T, S = 5, 40
    rng = np.random.default_rng(2)
    t = _schedule(T)
    norms = rng.uniform(0.5, 2.0, (S, T + 1))
    got = orc.fit_gamma(norms, t)
    for j in range(1, T):
        slope = np.linalg.lstsq(norms[:, j + 1:j + 2], norms[:, j], rcond=None)[0][0]
        assert np.isclose(got[j], slope / (1.0 - (t[j + 1] - t[j])), rtol=1e-12)


def test_solver_only_decay_gives_gamma_one():
    """Norms that shrink by the solver's own factor (1 - dt) per step (appendix Eq.13) need no correction."""
    T = 28
    t = _schedule(T)
    norms = np.ones((3, T + 1))
    for j in range(T - 1, 0, -1):
        norms[:, j] = norms[:, j + 1] * (1.0 - (t[j + 1] - t[j]))
    assert np.allclose(orc.fit_gamma(norms, t), 1.0, rtol=1e-12)
    # and the fitted table drives the cache decision exactly like gamma = 1
    st_a, st_b = orc.AvdState(), orc.AvdState()
    g = orc.fit_gamma(norms, t)
    for j in range(T - 1, 0, -1):
        assert orc.avd_decision(t, g, 0.04, j, st_a)[0] == orc.avd_decision(t, np.ones(T + 1), 0.04, j, st_b)[0]


def test_guidance_combine_special_cases_and_linearity():
    rng = np.random.default_rng(3)
    vc, vu = rng.normal(size=(5, 4)), rng.normal(size=(5, 4))
    assert np.array_equal(orc.guidance_combine(vc, vu, 1.0), vu + (vc - vu))
    assert np.allclose(orc.guidance_combine(vc, vu, 1.0), vc, atol=1e-15)
    assert np.array_equal(orc.guidance_combine(vc, vu, 0.0), vu)
    # extrapolation: scale 2.5 moves 1.5 times the difference past the conditional velocity
    assert np.allclose(orc.guidance_combine(vc, vu, 2.5), vc + 1.5 * (vc - vu), atol=1e-14)
    assert np.array_equal(orc.guidance_combine(np.array([3.0]), np.array([1.0]), 4.0), [9.0])
