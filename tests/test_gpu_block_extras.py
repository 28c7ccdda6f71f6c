"""GPU parity of the block's query/key extras (RMS normalisation over the head dimension, rotary
embedding with the positions of the full sequence) against the float64 oracle, and of the
rotation table itself."""
import numpy as np
import pytest
import torch

from oracle import regione_oracle as orc
from paper_2510_25590_amd import binding as rg
from paper_2510_25590_amd import inputs
from gpu_util import dev, host, assert_close, block_to_device

pytestmark = pytest.mark.gpu


def _positions(n_txt, grid, n_ref_grids):
    """[P | X | I]: text at (0,0,0), image tokens at (0,y,x), reference image tokens at (1,y,x)."""
    rows = [np.zeros((n_txt, 3), dtype=np.int32)]
    yy, xx = np.meshgrid(np.arange(grid), np.arange(grid), indexing="ij")
    for img in range(1 + n_ref_grids):
        rows.append(np.stack([np.full(grid * grid, img), yy.ravel(), xx.ravel()], axis=1).astype(np.int32))
    return np.concatenate(rows, axis=0)


@pytest.mark.parametrize("d,axes", [(128, (16, 56, 56)), (64, (8, 28, 28))])
def test_rope_table_matches_oracle_angles(d, axes):
    ctx = rg.Context(4 * d, 4, d, 8 * d, 64, 64)
    pos = _positions(7, 9, 1)
    pos[5] = [3, 4000, 77]          # large coordinates: the angle is formed in float64
    n = len(pos)
    table = torch.full((n + 1, d), 9.0, dtype=torch.float32, device="cuda")
    rg.regione_rope_table(ctx, torch.from_numpy(pos).cuda(), n, list(axes), 10000.0, table)
    got = host(table)
    ang = orc.rope_angles(pos, axes, 10000.0)
    assert np.all(got[n] == 9.0)
    assert np.abs(got[:n, :d // 2] - np.cos(ang)).max() <= 1e-7
    assert np.abs(got[:n, d // 2:] - np.sin(ang)).max() <= 1e-7
    with pytest.raises(rg.RegionEError):
        rg.regione_rope_table(ctx, torch.from_numpy(pos).cuda(), n, [16, 56, 40], 10000.0, table)   # axes do not fill the head
    with pytest.raises(rg.RegionEError):
        rg.regione_rope_table(ctx, torch.from_numpy(pos).cuda(), n, [15, 57, 56], 10000.0, table)   # odd share
    ctx.close()


def _with_norms(streams, rng, d):
    for w in streams:
        w["q_norm"] = inputs.bf16_round((1.0 + 0.2 * rng.standard_normal(d)).astype(np.float32))
        w["k_norm"] = inputs.bf16_round((1.0 + 0.2 * rng.standard_normal(d)).astype(np.float32))
    return streams


@pytest.mark.parametrize("kind", ["double", "single"])
@pytest.mark.parametrize("extras", ["norm+rope", "rope", "norm"])
def test_block_extras_all_modes(kind, extras):
    hidden, heads, d, mlp = 256, 4, 64, 1024
    n_txt, grid = 32, 16
    n_img = grid * grid
    n_all = n_txt + 2 * n_img
    rng = np.random.default_rng(inputs.workload_seed(1, 31))
    streams = [inputs.stream_weights(rng, hidden, mlp, kind, "bf16", std=0.05) for _ in range(2 if kind == "double" else 1)]
    if "norm" in extras:
        streams = _with_norms(streams, rng, d)
    pos = _positions(n_txt, grid, 1)
    axes = (8, 28, 28)
    rope_o = orc.rope_angles(pos, axes) if "rope" in extras else None
    h = inputs.bf16_round(rng.standard_normal((n_all, hidden)).astype(np.float32))
    e = np.nonzero(inputs.rect_mask(rng, grid, grid, 6, 6))[0].astype(np.int32)

    ctx = rg.Context(hidden, heads, d, mlp, n_all, 4096)
    bw, keep = block_to_device(streams, kind, ctx)
    if rope_o is not None:
        table = torch.empty((n_all, d), dtype=torch.float32, device="cuda")
        rg.regione_rope_table(ctx, torch.from_numpy(pos).cuda(), n_all, list(axes), 10000.0, table)
        bw.rope, bw.rope_rows = table.data_ptr(), n_all
    btype = rg.BLOCK_DOUBLE if kind == "double" else rg.BLOCK_SINGLE

    kc_o = np.zeros((n_all, heads, d)); vc_o = np.zeros_like(kc_o)
    full_o = orc.block_forward(streams, kind, h, n_txt, np.arange(n_all), kc_o, vc_o, orc.FLAG_STORE, heads, rope=rope_o)
    slots_all = torch.arange(n_all, dtype=torch.int32, device="cuda")
    kc = torch.zeros((n_all, heads, d), dtype=torch.bfloat16, device="cuda"); vc = torch.zeros_like(kc)
    out = torch.empty((n_all, hidden), dtype=torch.bfloat16, device="cuda")
    rg.regione_block_forward(ctx, bw, btype, dev(h, "bf16"), out, rg.BF16, n_all, n_txt, slots_all, 0, kc, vc, n_all, rg.FLAG_STORE)
    assert_close(host(out), full_o, f"{kind} {extras}: storing full forward", stored_bf16=True)
    assert_close(host(kc), kc_o, f"{kind} {extras}: stored K (normalised, rotated)", stored_bf16=True)
    assert_close(host(vc), vc_o, f"{kind} {extras}: stored V", stored_bf16=True)
    # no cache, no slot list: row i is position i
    out2 = torch.empty_like(out)
    rg.regione_block_forward(ctx, bw, btype, dev(h, "bf16"), out2, rg.BF16, n_all, n_txt, None, 0, None, None, 0, 0)
    assert_close(host(out2), full_o, f"{kind} {extras}: plain full forward", stored_bf16=True)

    # region forward on a moved hidden state: gathered rows keep their positions
    h2 = inputs.bf16_round((h + 0.05 * rng.standard_normal(h.shape)).astype(np.float32))
    for mode, rows in (("B", n_txt + e), ("A", np.concatenate([np.arange(n_txt), n_txt + e]))):
        n_txt_fresh = 0 if mode == "B" else n_txt
        kc_ref, vc_ref = kc_o.copy(), vc_o.copy()
        want = orc.block_forward(streams, kind, h2[rows], n_txt_fresh, rows, kc_ref, vc_ref, orc.FLAG_RETRIEVE, heads, rope=rope_o)
        kc_before, vc_before = kc.clone(), vc.clone()
        o = torch.empty((len(rows), hidden), dtype=torch.bfloat16, device="cuda")
        rg.regione_block_forward(ctx, bw, btype, dev(h2[rows], "bf16"), o, rg.BF16, len(rows), n_txt_fresh,
                                 torch.from_numpy(rows.astype(np.int32)).cuda(), 0, kc, vc, n_all, rg.FLAG_RETRIEVE)
        assert_close(host(o), want, f"{kind} {extras}: region forward, mode {mode}", stored_bf16=True)
        kc.copy_(kc_before); vc.copy_(vc_before)
    # slot list given as E_index plus an offset
    rows = n_txt + e
    o = torch.empty((len(rows), hidden), dtype=torch.bfloat16, device="cuda")
    rg.regione_block_forward(ctx, bw, btype, dev(h[rows], "bf16"), o, rg.BF16, len(rows), 0, torch.from_numpy(e).cuda(), n_txt, kc, vc, n_all, rg.FLAG_RETRIEVE)
    assert_close(host(o), full_o[rows], f"{kind} {extras}: same-step cache", stored_bf16=True)
    if rope_o is not None:
        bw.rope_rows = n_all - 1
        with pytest.raises(rg.RegionEError):
            rg.regione_block_forward(ctx, bw, btype, dev(h, "bf16"), out, rg.BF16, n_all, n_txt, slots_all, 0, kc, vc, n_all, rg.FLAG_STORE)
    ctx.close()


def test_block_extras_wide_heads_sampled():
    """Head dimension 128 (16 lanes per head vector) at hidden 1024, region forward with both extras."""
    hidden, heads, d, mlp = 1024, 8, 128, 2048
    n_txt, grid = 64, 24
    n_img = grid * grid
    n_all = n_txt + 2 * n_img
    rng = np.random.default_rng(inputs.workload_seed(2, 33))
    streams = _with_norms([inputs.stream_weights(rng, hidden, mlp, "double", "bf16", std=0.03) for _ in range(2)], rng, d)
    pos = _positions(n_txt, grid, 1)
    axes = (16, 56, 56)
    rope_o = orc.rope_angles(pos, axes)
    h = inputs.bf16_round(rng.standard_normal((n_all, hidden)).astype(np.float32))
    e = np.nonzero(inputs.rect_mask(rng, grid, grid, 9, 11))[0].astype(np.int32)
    ctx = rg.Context(hidden, heads, d, mlp, n_all, 4096)
    bw, keep = block_to_device(streams, "double", ctx)
    table = torch.empty((n_all, d), dtype=torch.float32, device="cuda")
    rg.regione_rope_table(ctx, torch.from_numpy(pos).cuda(), n_all, list(axes), 10000.0, table)
    bw.rope, bw.rope_rows = table.data_ptr(), n_all
    kc_o = np.zeros((n_all, heads, d)); vc_o = np.zeros_like(kc_o)
    full_o = orc.block_forward(streams, "double", h, n_txt, np.arange(n_all), kc_o, vc_o, orc.FLAG_STORE, heads, rope=rope_o)
    kc = torch.zeros((n_all, heads, d), dtype=torch.bfloat16, device="cuda"); vc = torch.zeros_like(kc)
    out = torch.empty((n_all, hidden), dtype=torch.bfloat16, device="cuda")
    rg.regione_block_forward(ctx, bw, rg.BLOCK_DOUBLE, dev(h, "bf16"), out, rg.BF16, n_all, n_txt,
                             torch.arange(n_all, dtype=torch.int32, device="cuda"), 0, kc, vc, n_all, rg.FLAG_STORE)
    assert_close(host(out), full_o, "d=128 storing full forward with extras", stored_bf16=True)
    assert_close(host(kc), kc_o, "d=128 stored K", stored_bf16=True)
    rows = n_txt + e
    h2 = inputs.bf16_round((h[rows] + 0.05 * rng.standard_normal((len(rows), hidden))).astype(np.float32))
    want = orc.block_forward(streams, "double", h2, 0, rows, kc_o, vc_o, orc.FLAG_RETRIEVE, heads, rope=rope_o)
    o = torch.empty((len(rows), hidden), dtype=torch.bfloat16, device="cuda")
    rg.regione_block_forward(ctx, bw, rg.BLOCK_DOUBLE, dev(h2, "bf16"), o, rg.BF16, len(rows), 0, torch.from_numpy(e).cuda(), n_txt, kc, vc, n_all, rg.FLAG_RETRIEVE)
    assert_close(host(o), want, "d=128 region forward with extras", stored_bf16=True)
    ctx.close()
