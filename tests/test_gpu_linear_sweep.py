"""Seeded sweep of odd shapes through every GEMM kernel variant and K split (forced plans), bf16 and E4M3, against the
oracle: rows and columns that are not multiples of the tiles, K from one step up, the remainder loop behind the pipelined
part, partial sums."""
import random

import numpy as np
import pytest
import torch

from oracle import fp8_reference as f8
from oracle import regione_oracle as orc
from paper_2510_25590_amd import binding as rg

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    return rg.Context(3072, 24, 128, 12288, 2048, 16)


def _cases(seed, count, k_unit):
    rnd = random.Random(seed)
    out = []
    for _ in range(count):
        m = rnd.choice([1, 5, 31, 64, 127, 128, 129, 255, 300, 513, 820])
        n = rnd.choice([8, 32, 40, 64, 96, 128, 200, 256, 520, 1000])
        k = k_unit * rnd.choice([1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 31])
        tn = rnd.choice([0, 1, 2, 3, 4, 5, 6] if k_unit == 64 else [0, 1, 2])
        splits = rnd.choice([1, 1, 2, 3, 4]) if tn else 0
        if splits > k // k_unit:
            splits = 1
        out.append((m, n, k, tn, splits))
    return out


@pytest.mark.parametrize("m,n,k,tn,splits", _cases(11, 36, 64))
def test_linear_bf16_forced_plans(ctx, m, n, k, tn, splits):
    rng = np.random.default_rng(m * 131 + n * 17 + k + tn)
    x = torch.from_numpy(rng.standard_normal((m, k)).astype(np.float32)).to(torch.bfloat16)
    w = torch.from_numpy((rng.standard_normal((n, k)) * 0.05).astype(np.float32)).to(torch.bfloat16)
    b = rng.standard_normal(n).astype(np.float32)
    want = orc.linear(x.float().numpy(), w.float().numpy(), b)
    wp = rg.pack_weight(ctx, w.cuda())
    y = torch.full((m, n), 7.0, dtype=torch.float32, device="cuda")
    rg.regione_tune_gemm(ctx, tn, splits)
    try:
        rg.regione_linear(ctx, x.cuda(), wp, torch.from_numpy(b).cuda(), m, n, k, rg.ACT_NONE, rg.FP32, y)
        torch.cuda.synchronize()
    finally:
        rg.regione_tune_gemm(ctx, 0, 0)
    # bf16 operands, exact products, float32 sums: a few 2^-24 of the sum of magnitudes
    mag = np.abs(x.float().numpy().astype(np.float64)) @ np.abs(w.float().numpy().astype(np.float64)).T + np.abs(b)[None, :]
    assert np.all(np.abs(y.cpu().numpy() - want) <= mag * 2.0 ** -19 + 1e-30)


@pytest.mark.parametrize("m,n,k,tn,splits", _cases(12, 20, 128))
def test_linear_fp8_forced_plans(ctx, m, n, k, tn, splits):
    rng = np.random.default_rng(m * 7 + n * 5 + k + tn)
    xq = ((rng.integers(0, 256, (m, k)).astype(np.uint8) & 0x87) | 0x30).astype(np.uint8)
    wq = ((rng.integers(0, 256, (n, k)).astype(np.uint8) & 0x87) | 0x28).astype(np.uint8)
    sx = rng.uniform(0.5, 1.5, m).astype(np.float32); sw = rng.uniform(0.5, 1.5, n).astype(np.float32)
    want = f8.linear_fp8(xq, sx, wq, sw)
    mag = (np.abs(f8.e4m3_decode(xq)) @ np.abs(f8.e4m3_decode(wq)).T) * sx[:, None].astype(np.float64) * sw[None, :]
    packed = torch.zeros(rg.regione_packed_weight_elems(n, k), dtype=torch.uint8, device="cuda")
    rg.regione_pack_weight_fp8(ctx, torch.from_numpy(wq).cuda(), n, k, packed)
    y = torch.full((m, n), 7.0, dtype=torch.float32, device="cuda")
    rg.regione_tune_gemm(ctx, tn, splits)
    try:
        rg.regione_linear_fp8(ctx, torch.from_numpy(xq).cuda(), torch.from_numpy(sx).cuda(), packed, torch.from_numpy(sw).cuda(), None,
                              m, n, k, rg.ACT_NONE, rg.FP32, y)
        torch.cuda.synchronize()
    finally:
        rg.regione_tune_gemm(ctx, 0, 0)
    assert np.all(np.abs(y.cpu().numpy() - want) <= mag * 2.0 ** -11 + 1e-30)


def _attn_cases(seed, count):
    rnd = random.Random(seed)
    out = []
    for _ in range(count):
        d = rnd.choice([64, 128])
        n_q = rnd.choice([1, 7, 32, 33, 127, 128, 129, 200, 300])
        n_fresh = rnd.choice([0, 0, 1, 17, 64, 65, n_q])
        n_c = rnd.choice([0, 1, 63, 64, 65, 191, 500, 1200, 2100])
        if n_fresh + n_c == 0:
            n_c = 70
        use_index = n_c > 2 and rnd.random() < 0.4
        splits = rnd.choice([0, 1, 2, 3, 5, 8])
        out.append((d, n_q, n_fresh, n_c, use_index, splits))
    return out


@pytest.mark.parametrize("d,n_q,n_fresh,n_c,use_index,splits", _attn_cases(21, 30))
def test_attention_forced_key_splits(ctx, d, n_q, n_fresh, n_c, use_index, splits):
    """Eq.6 in all three key-source forms (contiguous cache, fresh + cache, fresh + cache rows by index list) with every
    number of key-range splits, on key counts around the 64-key tile."""
    from tests.gpu_util import assert_close
    heads = 2
    rng = np.random.default_rng(d + 3 * n_q + 5 * n_fresh + 7 * n_c + splits)
    bf = lambda a: torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16)
    q, kf, vf = bf(rng.standard_normal((n_q, heads, d))), bf(rng.standard_normal((n_fresh, heads, d))), bf(rng.standard_normal((n_fresh, heads, d)))
    kc, vc = bf(rng.standard_normal((n_c, heads, d))), bf(rng.standard_normal((n_c, heads, d)))
    idx = np.sort(rng.choice(n_c, size=max(1, (2 * n_c) // 3), replace=False)).astype(np.int32) if use_index else None
    want = orc.attention_kvcache(q.float().numpy(), kf.float().numpy(), vf.float().numpy(), kc.float().numpy() if n_c else None,
                                 vc.float().numpy() if n_c else None, idx)
    out = torch.full((n_q, heads, d), 55.0, dtype=torch.bfloat16, device="cuda")
    rg.regione_tune_attention(ctx, splits)
    try:
        rg.regione_attn_kvcache(ctx, q.cuda(), n_q, kf.cuda() if n_fresh else None, vf.cuda() if n_fresh else None, n_fresh,
                                kc.cuda() if n_c else None, vc.cuda() if n_c else None, n_c,
                                None if idx is None else torch.from_numpy(idx).cuda(), 0 if idx is None else len(idx), heads, d, 0.0, out)
        torch.cuda.synchronize()
    finally:
        rg.regione_tune_attention(ctx, 0)
    assert_close(out.float().cpu().numpy(), want, f"attention d={d} q={n_q} fresh={n_fresh} cache={n_c} index={use_index} splits={splits}")
