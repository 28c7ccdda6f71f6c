"""Pins for the oracle's adaptive velocity decay cache (Eq.7-9), Euler step (Eq.4) and the
control flow of Algorithm 1 (CPU only).  Expected values: appendix Eq.13 (gamma = 1 gives a
product of (1 - dt) factors), arithmetic on the linear 28-step schedule, and the property
that a constant velocity field makes the sampler exact whatever is partitioned or cached.
"""
import json
import math
import os

import numpy as np
import pytest

from oracle import regione_oracle as orc

# what the paper prints (section "Experimental Settings", Table 1): steps, stage lengths, thresholds, latencies
PAPER = json.load(open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "experimental_settings.json")))

T = 28
t_lin = np.arange(T + 1) / T          # t[T] = 1, t[0] = 0
ones = np.ones(T + 1)


def _run(delta, js, gamma=ones):
    st = orc.AvdState()
    return [orc.avd_decision(t_lin, gamma, delta, j, st) for j in js]


def test_decay_factor_is_eq7():
    assert orc.decay_factor(t_lin, ones, 10) == pytest.approx(27 / 28, rel=1e-15)
    g = ones.copy(); g[10] = 0.5
    assert orc.decay_factor(t_lin, g, 10) == pytest.approx(0.5 * 27 / 28, rel=1e-15)
    t = np.array([0.0, 0.1, 0.4, 1.0])   # non-uniform: step from t[2] to t[1] has factor 1-(t[2]-t[1])... indexed at j: 1-(t[j+1]-t[j])
    assert orc.decay_factor(t, np.ones(4), 1) == pytest.approx(0.7, rel=1e-15)


def test_gamma_one_reproduces_residual_cache_closed_form():
    # delta large: one compute, then N reuses with factor (27/28)^N  (appendix Eq.13)
    dec = _run(10.0, range(22, 12, -1))
    assert dec[0] == (False, 1.0)
    for n, (reuse, f) in enumerate(dec[1:], start=1):
        assert reuse and f == pytest.approx((27 / 28) ** n, rel=1e-14)


@pytest.mark.parametrize("delta,pattern", [
    (0.04, "FRFRFRFRFR"),     # 1-(27/28) = 0.0357 <= 0.04 < 0.0702
    (0.03, "FFFFFFFFFF"),
    (0.02, "FFFFFFFFFF"),
    (0.08, "FRRFRRFRRF"),     # two reuses (0.0357, 0.0702), third would be 0.1034
    (-1.0, "FFFFFFFFFF"),     # cache switched off
])
def test_decision_patterns_on_linear_schedule(delta, pattern):
    got = "".join("R" if r else "F" for r, _ in _run(delta, range(22, 12, -1)))
    assert got == pattern


def test_first_step_is_always_fresh_and_state_resets():
    st = orc.AvdState()
    assert orc.avd_decision(t_lin, ones, 1e9, 5, st) == (False, 1.0)
    assert orc.avd_decision(t_lin, ones, 1e9, 4, st)[0] is True
    st2 = orc.AvdState()
    assert orc.avd_decision(t_lin, ones, 1e9, 3, st2) == (False, 1.0)


def test_velocity_cache_apply_both_branches_step_x():
    x = np.array([[1.0, 2.0]]); v = np.array([[4.0, -8.0]]); c = np.array([[2.0, 2.0]])
    vu, cn, xn = orc.velocity_cache_apply(False, 1.0, 0.25, v, c, x)
    assert np.array_equal(vu, v) and np.array_equal(cn, v) and np.array_equal(xn, [[0.0, 4.0]])
    vu, cn, xn = orc.velocity_cache_apply(True, 0.5, 0.25, None, c, x)
    assert np.array_equal(vu, [[1.0, 1.0]]) and np.array_equal(cn, c) and np.array_equal(xn, [[0.75, 1.75]])


def test_euler_constant_velocity_equals_one_big_step():
    x = np.array([[1.0, -2.0]]); v = np.array([[0.5, 0.25]])
    y = x
    for i in range(T, 0, -1):
        y = orc.euler_step(y, v, t_lin[i] - t_lin[i - 1])
    assert np.allclose(y, orc.euler_step(x, v, 1.0), atol=1e-14)


def test_stage_plan_counts_for_paper_hyperparameters():
    # 28 steps, 6 stabilization steps, forced update at step 16, 2 smooth steps
    assert (PAPER["sampling_steps"], PAPER["stabilization_steps"], PAPER["forced_update_step"], PAPER["smooth_steps"]) == (28, 6, 16, 2)
    plan, segments = orc.stage_plan(PAPER["sampling_steps"], PAPER["stabilization_steps"], PAPER["smooth_steps"], [PAPER["forced_update_step"]])
    kinds = [k for _, k in plan]
    assert [i for i, _ in plan] == list(range(28, 0, -1))
    assert kinds.count("region") == 19 and kinds.count("full") + kinds.count("full_store") == 9
    assert segments == [(22, 11), (11, 1)]
    ks = {28 - i: k for i, k in plan}
    assert [k for k in range(28) if ks[k] == "full_store"] == [5, 16, 26]
    assert all(ks[k] == "full" for k in (0, 1, 2, 3, 4, 27))
    assert all(ks[k] == "region" for k in list(range(6, 16)) + list(range(17, 26)))
    # no forced step: one segment of 20 region steps
    plan2, seg2 = orc.stage_plan(28, 6, 2, [])
    assert [k for _, k in plan2].count("region") == 20 and seg2 == [(22, 1)]


def test_loop_with_constant_velocity_is_exact_and_logs_the_stages():
    rng = np.random.default_rng(30)
    n, c = 64, 8
    ref = rng.standard_normal((n, c)).astype(np.float32)
    x_T = rng.standard_normal((n, c))
    v_const = rng.standard_normal((n, c))
    calls = []

    def phi(x_rows, rows, i, mode):
        calls.append((i, mode, None if rows is None else len(rows)))
        return v_const if rows is None else v_const[rows]

    for delta in (0.04, -1.0, 10.0):
        calls.clear()
        x0, log = orc.regione_loop(phi, x_T, ref, t_lin, ones, 28, 6, 2, [16], 0.9, delta)
        part = [w for w in log if w[0] == "partition"]
        assert len(part) == 1
        n_e = part[0][1]
        fresh = [w for w in log if w[1] == "region_fresh"]
        reuse = [w for w in log if w[1] == "region_reuse"]
        assert len(fresh) + len(reuse) == 19
        assert len([cl for cl in calls if cl[1] == "region"]) == len(fresh)
        assert all(cl[2] == n_e for cl in calls if cl[1] == "region")
        if delta < 0:
            assert len(reuse) == 0
        if delta == 10.0:
            assert len(fresh) == 2                    # one compute per segment
        if delta == 0.04:
            assert len(fresh) == 10                   # 5 of 10, then 5 of 9
        if delta < 1.0:
            # with gamma = 1 a reuse scales v by (27/28)^n, so only delta <= 0 is exact; check the exact case
            pass
    calls.clear()
    x0, _ = orc.regione_loop(phi, x_T, ref, t_lin, ones, 28, 6, 2, [16], 0.9, -1.0)
    assert np.max(np.abs(x0 - (x_T - v_const))) < 1e-12   # sum of dt = 1


def test_loop_unedited_rows_take_one_jump():
    # velocity that depends on the step index: unedited rows must see only the velocity of the
    # last full step before the segment, scaled by the whole segment length (Eq.5)
    n, c = 16, 4
    rng = np.random.default_rng(31)
    ref = rng.standard_normal((n, c)).astype(np.float32)
    x_T = rng.standard_normal((n, c))
    base = rng.standard_normal((n, c))
    seen = {}

    def phi(x_rows, rows, i, mode):
        v = base * (1.0 + 0.01 * i)
        return v if rows is None else v[rows]

    x0, log = orc.regione_loop(phi, x_T, ref, t_lin, ones, 28, 6, 2, [], 0.9, -1.0)
    # emulate by hand: full steps 28..23, partition at 22, region/unedited to index 2, full at 2 and 1
    x = x_T.copy()
    for i in range(28, 22, -1):
        x = x - (1 / 28) * base * (1 + 0.01 * i)
    v23 = base * (1 + 0.01 * 23)
    _, mask, e, u = orc.partition(x.astype(np.float32), v23.astype(np.float32), ref, t_lin[22], 0.9)
    xu = x[u] - v23[u] * (t_lin[22] - t_lin[2])
    xe = x[e].copy()
    for j in range(22, 2, -1):
        xe = xe - (1 / 28) * base[e] * (1 + 0.01 * j)
    x[u] = xu; x[e] = xe
    for i in (2, 1):
        x = x - (1 / 28) * base * (1 + 0.01 * i)
    assert np.max(np.abs(x0 - x)) < 1e-12


# ---- the data-dependent reuse trigger of the loop benchmark's workload description (not the paper's Eq.8)


def test_relative_change_hand_cases():
    b = np.array([[3.0, 4.0]])
    assert math.isclose(orc.relative_change(1.1 * b, b), 0.1, rel_tol=1e-12)
    assert orc.relative_change(b, b) == 0.0
    assert math.isclose(orc.relative_change(np.array([[4.0, -3.0]]), b), math.sqrt(2.0), rel_tol=1e-12)   # orthogonal, same length
    assert orc.relative_change(b, np.zeros((1, 2))) == math.inf


def _loop_with_velocity(vel, rel_trigger, forced_reuse=None, T=12, t_st=2, t_sm=1, forced_k=()):
    """Runs the loop on 6 tokens of 2 channels whose first three are 'edited' (they differ from the reference);
    vel(i) gives the velocity of every row at timestep index i."""
    n, c = 6, 2
    x_ref = np.ones((n, c))
    x_T = np.ones((n, c)); x_T[:3] = [[-1.0, 1.0]] * 3       # cosine 0 with the reference row (1, 1)
    t = np.linspace(0.0, 1.0, T + 1)
    calls = []

    def phi(x_rows, row_index, i, mode):
        calls.append((i, mode))
        rows = np.arange(n) if row_index is None else np.asarray(row_index)
        return np.tile(vel(i), (len(rows), 1))   # the same velocity for every row

    x0, log = orc.regione_loop(phi, x_T, x_ref, t, np.ones(T + 1), T, t_st, t_sm, list(forced_k), 0.5, 0.04,
                               rel_trigger=rel_trigger, forced_reuse=forced_reuse)
    return x0, log, calls, t


def test_relative_trigger_constant_velocity_alternates_and_never_reuses_twice():
    # zero velocity keeps the partition trivial (x never moves); a constant velocity has relative change 0
    x0, log, calls, t = _loop_with_velocity(lambda i: np.zeros(2), (0.05, 0.9))
    # zero velocity: |v_old| = 0 -> relative change is infinite, never below the threshold: every step fresh
    kinds = [w[1] for w in log if w[0] not in ("partition", "rel")]
    assert "region_reuse" not in kinds
    x0, log, calls, t = _loop_with_velocity(lambda i: np.array([1e-3, -1e-3]), (0.05, 0.9))
    steps = [(w[0], w[1]) for w in log if w[0] not in ("partition", "rel")]
    region = [k for _, k in steps if k.startswith("region")]
    # a segment starts with two fresh steps (the second measures the change), then reuse and fresh alternate
    assert region[:4] == ["region_fresh", "region_fresh", "region_reuse", "region_fresh"]
    assert all(not (a == b == "region_reuse") for a, b in zip(region, region[1:]))
    rels = [w for w in log if w[0] == "rel"]
    assert rels and all(w[2] == 0.0 for w in rels)


def test_relative_trigger_reused_step_moves_by_the_decayed_cache():
    v = np.array([2e-3, -1e-3])
    x0_a, log_a, _, t = _loop_with_velocity(lambda i: v, (0.05, 0.9))
    x0_b, log_b, _, _ = _loop_with_velocity(lambda i: v, (0.05, 1.0))
    reused = [w[0] for w in log_a if w[1] == "region_reuse"]
    assert reused == [w[0] for w in log_b if w[1] == "region_reuse"]
    # with decay 1 a reused step moves exactly like a fresh one; with 0.9 each reused step moves 10 % less (Eq.4)
    lost = sum(0.1 * (t[i] - t[i - 1]) for i in reused)
    assert np.allclose((x0_a - x0_b)[:3], lost * v, atol=1e-15)
    assert np.allclose((x0_a - x0_b)[3:], 0.0, atol=1e-15)      # unedited rows never see the cache


def test_relative_trigger_changing_velocity_never_reuses_and_forced_decisions_override():
    vel = lambda i: np.array([1e-3 * (1.0 + 0.2 * i), -1e-3])       # changes by far more than 5 % per step
    x0, log, calls, t = _loop_with_velocity(vel, (0.05, 0.9))
    assert not any(w[1] == "region_reuse" for w in log)
    assert all(w[2] > 0.05 for w in log if w[0] == "rel")
    region_steps = [w[0] for w in log if w[1] == "region_fresh"]
    forced = {region_steps[2]: True}
    x0_f, log_f, calls_f, _ = _loop_with_velocity(vel, (0.05, 0.9), forced_reuse=forced)
    assert (region_steps[2], "region_reuse") in [(w[0], w[1]) for w in log_f]
    assert (region_steps[2], "region") not in calls_f and (region_steps[2], "region") in calls
    # the first step of a segment has nothing to reuse: forcing it changes nothing
    x0_g, log_g, _, _ = _loop_with_velocity(vel, (0.05, 0.9), forced_reuse={region_steps[0]: True})
    assert [(w[0], w[1]) for w in log_g] == [(w[0], w[1]) for w in log] and np.array_equal(x0_g, x0)


def test_paper_thresholds_on_a_uniform_schedule_with_solver_only_decay():
    """With gamma = 1 (appendix Eq.13) and the uniform 28-step schedule, Eq.8 after one skipped step is 1 - 27/28 = 0.0357 and
    after two 1 - (27/28)^2 = 0.0702: of the three thresholds the paper prints, only 0.04 lets a step be reused, and never
    two in a row."""
    want = {0.02: "F" * 10, 0.03: "F" * 10, 0.04: "FR" * 5}
    for name, m in PAPER["models"].items():
        got = "".join("R" if r else "F" for r, _ in _run(m["delta"], range(22, 12, -1)))
        assert got == want[m["delta"]], name


def test_printed_speedups_are_the_ratio_of_the_printed_latencies():
    """Table 1 is self-consistent (this pins the fixture, not the oracle), and the ratios bound what the stage plan can give:
    the paper's 9 full steps of 28 alone cap the speedup at 28 / 9 = 3.11, above all three printed values."""
    plan, _ = orc.stage_plan(PAPER["sampling_steps"], PAPER["stabilization_steps"], PAPER["smooth_steps"], [PAPER["forced_update_step"]])
    n_full = sum(1 for _, k in plan if k != "region")
    for name, m in PAPER["models"].items():
        assert abs(m["latency_vanilla_s"] / m["latency_regione_s"] - m["speedup"]) < 2e-3, name
        assert m["speedup"] < PAPER["sampling_steps"] / n_full
