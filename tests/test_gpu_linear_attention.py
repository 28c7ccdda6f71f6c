"""GPU parity: the bf16 MFMA GEMM (regione_linear) and the attention with the Region-Instruction
KV cache (regione_attn_kvcache, Eq.6) against the float64 oracle on the same bf16-rounded inputs."""
import numpy as np
import pytest
import torch

from oracle import regione_oracle as orc
from paper_2510_25590_amd import binding as rg
from paper_2510_25590_amd import inputs
from gpu_util import dev, host, assert_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = rg.Context(3072, 24, 128, 12288, 1024, 4096)
    yield c
    c.close()


@pytest.mark.parametrize("m,n,k", [(1, 8, 64), (37, 100, 64), (129, 257, 128), (300, 520, 256), (64, 64, 64),
                                   (819, 1000, 512), (130, 3072, 1024), (33, 96, 3072), (820, 640, 3072), (700, 256, 6144)])
@pytest.mark.parametrize("act", [rg.ACT_NONE, rg.ACT_GELU_TANH])
def test_linear_matches_oracle(ctx, m, n, k, act):
    rng = np.random.default_rng(1000 + m + n + k)
    x = inputs.bf16_round(rng.standard_normal((m, k)).astype(np.float32))
    w = inputs.bf16_round((rng.standard_normal((n, k)) / np.sqrt(k)).astype(np.float32))
    b = rng.standard_normal(n).astype(np.float32)
    want = orc.linear(x, w, b)
    if act == rg.ACT_GELU_TANH:
        want = orc.gelu_tanh(want)
    db = torch.from_numpy(b).cuda()
    wp = rg.pack_weight(ctx, dev(w, "bf16"))
    for out_dtype, tdt in ((rg.FP32, torch.float32), (rg.BF16, torch.bfloat16)):
        y = torch.full((m + 1, n), 77.0, dtype=tdt, device="cuda")
        rg.regione_linear(ctx, dev(x, "bf16"), wp, db, m, n, k, act, out_dtype, y)
        got = host(y)
        assert np.all(got[m] == 77.0)                       # the row after the last is untouched
        if out_dtype == rg.FP32:
            assert_close(got[:m], want, f"linear f32 {m}x{n}x{k}", max_abs=2e-4, mean_rel_tol=1e-5)
        else:
            assert_close(got[:m], want, f"linear bf16 {m}x{n}x{k}")
    # no bias
    y = torch.empty((m, n), dtype=torch.float32, device="cuda")
    rg.regione_linear(ctx, dev(x, "bf16"), wp, None, m, n, k, rg.ACT_NONE, rg.FP32, y)
    assert_close(host(y), orc.linear(x, w, None), "linear no bias", max_abs=2e-4, mean_rel_tol=1e-5)
    # every kernel variant (1, 2: weights straight to registers; 3, 4: both operands through LDS; 5, 6: the same with
    # 256-row tiles), wave-tile width and K split gives the same result
    for tn, splits in ((1, 1), (2, 1), (1, 3), (2, 2), (2, 4), (3, 1), (4, 1), (4, 2), (5, 1), (6, 1), (6, 3)):
        rg.regione_tune_gemm(ctx, tn, splits)
        y2 = torch.full((m + 1, n), 77.0, dtype=torch.float32, device="cuda")
        rg.regione_linear(ctx, dev(x, "bf16"), wp, db, m, n, k, act, rg.FP32, y2)
        assert np.all(host(y2)[m] == 77.0)
        assert_close(host(y2)[:m], want, f"linear tn={tn} splits={splits}", max_abs=2e-4, mean_rel_tol=1e-5)
    rg.regione_tune_gemm(ctx, 0, 0)


def test_linear_integer_values_are_exact(ctx):
    # small integers: every partial sum is exact in float32, so the result must equal the integer product
    rng = np.random.default_rng(1100)
    x = rng.integers(-4, 5, size=(200, 192)).astype(np.float32)
    w = rng.integers(-4, 5, size=(333, 192)).astype(np.float32)
    y = torch.empty((200, 333), dtype=torch.float32, device="cuda")
    rg.regione_linear(ctx, dev(x, "bf16"), rg.pack_weight(ctx, dev(w, "bf16")), None, 200, 333, 192, rg.ACT_NONE, rg.FP32, y)
    assert np.array_equal(host(y), (x.astype(np.int64) @ w.astype(np.int64).T).astype(np.float32))


def _attn_case(rng, n_q, n_fresh, n_c, heads, d, q_scale=1.0):
    mk = lambda n: inputs.bf16_round(rng.standard_normal((n, heads, d)).astype(np.float32))
    q = inputs.bf16_round((q_scale * rng.standard_normal((n_q, heads, d))).astype(np.float32))
    return q, mk(n_fresh), mk(n_fresh), mk(n_c), mk(n_c)


def _run_attn(ctx, q, kf, vf, kc, vc, idx, heads, d, scale=0.0):
    n_q, n_fresh, n_c = q.shape[0], kf.shape[0], kc.shape[0]
    out = torch.full((n_q + 1, heads, d), 55.0, dtype=torch.bfloat16, device="cuda")
    didx = None if idx is None else torch.from_numpy(idx.astype(np.int32)).cuda()
    rg.regione_attn_kvcache(ctx, dev(q, "bf16"), n_q, dev(kf, "bf16") if n_fresh else None, dev(vf, "bf16") if n_fresh else None, n_fresh,
                            dev(kc, "bf16") if n_c else None, dev(vc, "bf16") if n_c else None, n_c,
                            didx, 0 if idx is None else len(idx), heads, d, scale, out)
    got = host(out)
    assert np.all(got[n_q] == 55.0)
    return got[:n_q]


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("n_q,n_fresh,n_c", [(1, 1, 0), (5, 5, 3), (36, 36, 508), (130, 130, 200), (129, 0, 777),
                                             (64, 64, 0), (257, 257, 1023), (33, 33, 4000)])
def test_attention_matches_oracle(ctx, d, n_q, n_fresh, n_c):
    heads = 3
    rng = np.random.default_rng(2000 + n_q + n_c + d)
    q, kf, vf, kc, vc = _attn_case(rng, n_q, n_fresh, n_c, heads, d)
    want = orc.attention_kvcache(q, kf, vf, kc, vc)
    got = _run_attn(ctx, q, kf, vf, kc, vc, None, heads, d)
    assert_close(got, want, f"attention d={d} n_q={n_q} fresh={n_fresh} cache={n_c}")


@pytest.mark.parametrize("d", [128, 64])
def test_attention_with_cache_index_list(ctx, d):
    heads = 2
    rng = np.random.default_rng(2100 + d)
    q, kf, vf, kc, vc = _attn_case(rng, 50, 50, 900, heads, d)
    idx = np.sort(rng.choice(900, size=611, replace=False))
    want = orc.attention_kvcache(q, kf, vf, kc, vc, idx)
    got = _run_attn(ctx, q, kf, vf, kc, vc, idx, heads, d)
    assert_close(got, want, "attention with index list")
    # rows outside the list must not matter: poison them
    kc2 = kc.copy(); vc2 = vc.copy()
    outside = np.setdiff1d(np.arange(900), idx)
    kc2[outside] = 30.0; vc2[outside] = -1000.0
    got2 = _run_attn(ctx, q, kf, vf, kc2, vc2, idx, heads, d)
    assert np.array_equal(got, got2)


def test_attention_peaked_softmax_and_custom_scale(ctx):
    # large logits: one key dominates; checks max subtraction and the scale argument
    heads, d = 2, 128
    rng = np.random.default_rng(2200)
    q, kf, vf, kc, vc = _attn_case(rng, 70, 70, 300, heads, d, q_scale=6.0)
    want = orc.attention_kvcache(q, kf, vf, kc, vc, None, scale=0.2)
    got = _run_attn(ctx, q, kf, vf, kc, vc, None, heads, d, scale=0.2)
    assert_close(got, want, "peaked attention")


def test_attention_closed_forms_on_gpu(ctx):
    heads, d = 2, 64
    rng = np.random.default_rng(2300)
    q, kf, vf, kc, vc = _attn_case(rng, 40, 10, 90, heads, d)
    # identical keys -> mean of values
    kf[:] = kf[0]; kc[:] = kf[0]
    got = _run_attn(ctx, q, kf, vf, kc, vc, None, heads, d)
    mean_v = np.concatenate([vf, vc]).mean(axis=0)
    assert np.max(np.abs(got - mean_v[None])) < 1e-2
    # key order of the cache does not matter
    q, kf, vf, kc, vc = _attn_case(rng, 40, 10, 90, heads, d)
    perm = rng.permutation(90)
    a = _run_attn(ctx, q, kf, vf, kc, vc, None, heads, d)
    b = _run_attn(ctx, q, kf, vf, kc[perm], vc[perm], None, heads, d)
    assert np.max(np.abs(a - b)) < 1e-2


def test_attention_config2_shape_sampled(ctx):
    # 24 heads x 128, 819 edited queries, 8704 keys (819 fresh + 7885 cached): the split-KV launch; oracle on sampled rows
    heads, d, n_q, n_c = 24, 128, 819, 8704 - 819
    rng = np.random.default_rng(2400)
    q, kf, vf, kc, vc = _attn_case(rng, n_q, n_q, n_c, heads, d)
    got = _run_attn(ctx, q, kf, vf, kc, vc, None, heads, d)
    rows = np.sort(rng.choice(n_q, size=48, replace=False))
    rows[:3] = [0, 127, 818]
    want = orc.attention_kvcache(q[rows], kf, vf, kc, vc)
    assert_close(got[rows], want, "attention config-2 shape (sampled rows)")


def test_attention_errors(ctx):
    q = torch.zeros((4, 2, 32), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(rg.RegionEError) as e:
        rg.regione_attn_kvcache(ctx, q, 4, q, q, 4, None, None, 0, None, 0, 2, 32, 0.0, q)
    assert e.value.code == rg.ERR_UNSUPPORTED
    q = torch.zeros((4, 2, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(rg.RegionEError) as e:
        rg.regione_attn_kvcache(ctx, q, 4, None, None, 0, None, None, 0, None, 0, 2, 64, 0.0, q)
    assert e.value.code == rg.ERR_BAD_SHAPE
    rg.regione_attn_kvcache(ctx, q, 0, None, None, 0, None, None, 0, None, 0, 2, 64, 0.0, q)   # no query: no-op


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("n_fresh,use_index", [(0, False), (50, False), (50, True)])
def test_attention_runs_are_bit_identical(ctx, d, n_fresh, use_index):
    """No atomics and no order that depends on timing: the same call gives the same bits, for every source layout
    (one array, fresh + cache, cache through an index list) and with key splits.  A read of matrix-core results that
    did not wait for them once showed up exactly here, as one-ulp differences between runs."""
    heads = 2
    rng = np.random.default_rng(2300 + d + n_fresh)
    q, kf, vf, kc, vc = _attn_case(rng, 130, n_fresh, 900, heads, d)
    idx = np.sort(rng.choice(900, size=700, replace=False)) if use_index else None
    for splits in (1, 3):
        rg.regione_tune_attention(ctx, splits)
        runs = [_run_attn(ctx, q, kf, vf, kc, vc, idx, heads, d) for _ in range(4)]
        rg.regione_tune_attention(ctx, 0)
        for r in runs[1:]:
            assert np.array_equal(runs[0], r), f"splits {splits}: max difference between identical runs {np.abs(runs[0] - r).max()}"


def test_linear_runs_are_bit_identical(ctx):
    rng = np.random.default_rng(2400)
    m, n, k = 300, 520, 1024
    x = dev(inputs.bf16_round(rng.standard_normal((m, k)).astype(np.float32)), "bf16")
    wp = rg.pack_weight(ctx, dev(inputs.bf16_round((0.05 * rng.standard_normal((n, k))).astype(np.float32)), "bf16"))
    for tn, sp in ((0, 0), (1, 2), (2, 1), (4, 2), (6, 1)):
        rg.regione_tune_gemm(ctx, tn, sp)
        outs = []
        for _ in range(3):
            y = torch.zeros((m, n), dtype=torch.bfloat16, device="cuda")
            rg.regione_linear(ctx, x, wp, None, m, n, k, rg.ACT_NONE, rg.BF16, y)
            outs.append(host(y))
        rg.regione_tune_gemm(ctx, 0, 0)
        assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2]), (tn, sp)
