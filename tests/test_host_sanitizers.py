"""The library's host-only entry points (stage plan of Algorithm 1, cache decisions of Eq.7-8, the relative-change trigger,
the fit of Eq.7's factor) compiled for the CPU with the address and undefined-behaviour sanitizers and run on the cases the
ABI tests use: same results, bit for bit, as the shipped library, and no sanitizer report."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from paper_2510_25590_amd import binding as rg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host C++ compiler here")
    exe = str(tmp_path_factory.mktemp("san") / "host_driver")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "paper_2510_25590_amd", "csrc", "host_logic.cpp"),
           os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and "static-lib" in r.stderr:      # a toolchain without the static sanitizer runtimes
        cmd = [c for c in cmd if not c.startswith("-static-lib")]
        r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr

    def run(text: str):
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
        env.pop("LD_PRELOAD", None)       # the sanitizer runtime has to come first in the process
        p = subprocess.run([exe], input=text, capture_output=True, text=True, env=env, timeout=60)
        assert p.returncode == 0 and "ERROR" not in p.stderr and "runtime error" not in p.stderr, p.stderr
        return p.stdout.split("\n")
    return run


def _fl(tok: str) -> float:
    return float.fromhex(tok) if tok not in ("inf", "-inf", "nan") else float(tok)


@pytest.mark.parametrize("T,t_st,t_sm,forced", [(28, 6, 2, [16]), (28, 6, 2, []), (50, 10, 3, [20, 35]), (4, 1, 1, []), (28, 6, 2, [3]), (28, 20, 10, [])])
def test_stage_plan_under_sanitizers(driver, T, t_st, t_sm, forced):
    out = driver(f"plan {T} {t_st} {t_sm} {len(forced)} {' '.join(map(str, forced))} {T + 1}")
    rc, n = map(int, out[0].split())
    try:
        want = rg.regione_stage_plan_host(T, t_st, t_sm, forced)
    except rg.RegionEError as e:
        assert rc == e.code
        return
    assert rc == 0 and n == len(want)
    got = [tuple(map(int, line.split())) for line in out[1:1 + n]]
    assert got == [(s.i, s.kind, s.seg_first, s.seg_next) for s in want]


def test_stage_plan_too_small_output_under_sanitizers(driver):
    out = driver("plan 28 6 2 1 16 5")            # room for 5 of 28 steps: an error, nothing written past the room
    assert int(out[0].split()[0]) == rg.ERR_INVALID_ARG and "do not fit" in out[1]


@pytest.mark.parametrize("delta", [0.04, 0.08, -1.0, 10.0])
def test_velocity_decision_under_sanitizers(driver, delta):
    T = 28
    rng = np.random.default_rng(3)
    t = (np.arange(T + 1) / T).astype(np.float32)
    gamma = (1.0 + 0.02 * rng.standard_normal(T + 1)).astype(np.float32)
    js = list(range(22, 12, -1))
    out = driver(f"avd {T} {float(np.float32(delta))!r} {len(js)} {' '.join(map(str, js))} " + " ".join(repr(float(v)) for v in t) + " " + " ".join(repr(float(v)) for v in gamma))
    st = rg.AvdState(0, 1.0)
    for j, line in zip(js, out):
        rc, reuse, factor, valid, prod = line.split()
        want = rg.regione_velocity_decision_host(t, gamma, T, delta, j, st)
        assert int(rc) == 0 and bool(int(reuse)) == want[0] and _fl(factor) == want[1]
        assert int(valid) == st.valid and _fl(prod) == st.prod


def test_gamma_fit_under_sanitizers(driver):
    T, S = 12, 5
    rng = np.random.default_rng(4)
    t = (np.arange(T + 1) / T).astype(np.float32)
    sq = rng.random((S, T + 1)) * 3.0 + 0.5
    out = driver(f"gamma {S} {T} " + " ".join(repr(float(v)) for v in sq.ravel()) + " " + " ".join(repr(float(v)) for v in t))
    assert int(out[0]) == 0
    got = [_fl(v) for v in out[1:T + 2]]
    assert got == rg.regione_gamma_fit_host(sq, t)
    bad = sq.copy(); bad[2, 3] = -1.0
    out = driver(f"gamma {S} {T} " + " ".join(repr(float(v)) for v in bad.ravel()) + " " + " ".join(repr(float(v)) for v in t))
    assert int(out[0]) == rg.ERR_INVALID_ARG and "negative" in out[1]


def test_relative_change_trigger_under_sanitizers(driver):
    import ctypes as C
    thr, decay = 0.05, 0.9
    ops = [(0,), (2,), (0,), (1, 0.04, 4.0), (0,), (1, 1e-4, 4.0), (0,), (0,), (1, 9.0, 0.0), (0,)]
    text = f"rel {thr} {decay} {len(ops)} " + " ".join(" ".join(repr(x) if isinstance(x, float) else str(x) for x in op) for op in ops)
    out = driver(text)
    st = rg.RelState()
    for op, line in zip(ops, out):
        f = line.split()
        if op[0] == 0:
            reuse, factor = rg.regione_rel_decision_host(st, decay)
            assert (int(f[0]), bool(int(f[1])), _fl(f[2]), int(f[3]), int(f[4])) == (0, reuse, factor, st.have_cache, st.reuse_next)
        else:
            sums = (C.c_double * 2)(op[1], op[2]) if op[0] == 1 else None
            rel = rg.regione_rel_update_host(st, sums, thr)
            assert (int(f[0]), _fl(f[1]), int(f[2]), int(f[3])) == (0, rel, st.have_cache, st.reuse_next)


def test_null_arguments_under_sanitizers(driver):
    assert [int(v) for v in driver("nulls")[0].split()] == [rg.ERR_INVALID_ARG] * 5
