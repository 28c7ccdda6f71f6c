"""GPU test of regione_partition_static, the entry point that allocates nothing: through the C ABI, against
regione_partition on the same inputs, bit for bit, on two calls in a row (the second with a smaller input, so that
whatever the first call left in the library's static scratch array is still there), and the size limit."""
import numpy as np
import pytest
import torch

from paper_2510_25590_amd import binding as rg
from paper_2510_25590_amd import inputs

pytestmark = pytest.mark.gpu


def _case(seed, n_tokens, c, dtype):
    rng = np.random.default_rng(seed)
    want = rng.random(n_tokens) < 0.3
    x_t, v, x_ref = inputs.latents_for_mask(rng, want, c, 0.7, dtype)
    t = (lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()) if dtype == "bf16" else (lambda a: torch.from_numpy(a).cuda())
    return t(x_t), t(v), t(x_ref)


def _outputs(n):
    dev = "cuda"
    return dict(score=torch.full((n,), -7.0, dtype=torch.float32, device=dev), mask=torch.full((n,), 9, dtype=torch.uint8, device=dev),
                e=torch.full((n,), -1, dtype=torch.int32, device=dev), u=torch.full((n,), -1, dtype=torch.int32, device=dev),
                cnt=torch.full((1,), -1, dtype=torch.int32, device=dev))


@pytest.mark.parametrize("dtype,c", [("bf16", 64), ("f32", 16)])
def test_partition_static_equals_partition_on_two_calls_in_a_row(dtype, c):
    code = rg.BF16 if dtype == "bf16" else rg.FP32
    ctx = rg.Context(256, 4, 64, 1024, 16, 3_000_000)
    # the first call spans several thousand blocks (the scan kernel's path), the second a few blocks (one launch path)
    for seed, n in ((1, 2_500_000), (2, 70_001), (3, 4096), (4, 1), (5, 0)):
        x_t, v, x_ref = _case(seed, max(n, 1), c, dtype)
        a, b = _outputs(max(n, 1)), _outputs(max(n, 1))
        n_ref = rg.regione_partition(ctx, x_t, v, x_ref, n, c, code, 0.7, 0.9, a["score"], a["mask"], a["e"], a["u"], a["cnt"])
        rg.regione_partition_static(torch.cuda.current_stream(), x_t, v, x_ref, n, c, code, 0.7, 0.9, b["score"], b["mask"], b["e"], b["u"], b["cnt"])
        torch.cuda.synchronize()
        assert int(b["cnt"].item()) == n_ref == int(a["cnt"].item())
        for name in ("score", "mask", "e", "u"):
            assert torch.equal(a[name], b[name]), (name, n)      # includes everything past the counts: nothing else written
        if n >= 4096:
            assert 0.2 * n < n_ref < 0.4 * n
    ctx.close()


def test_partition_static_without_any_context_and_on_the_default_stream():
    x_t, v, x_ref = _case(7, 5000, 64, "bf16")
    o = _outputs(5000)
    rg.regione_partition_static(None, x_t, v, x_ref, 5000, 64, rg.BF16, 0.7, 0.9, None, o["mask"], o["e"], o["u"], o["cnt"])
    torch.cuda.synchronize()
    n = int(o["cnt"].item())
    mask = o["mask"].cpu().numpy()
    assert n == int(mask.sum())
    assert np.array_equal(o["e"].cpu().numpy()[:n], np.nonzero(mask)[0])
    assert np.array_equal(o["u"].cpu().numpy()[:5000 - n], np.nonzero(mask == 0)[0])


def test_partition_static_rejects_sizes_beyond_its_limit():
    x_t, v, x_ref = _case(8, 16, 64, "bf16")
    o = _outputs(16)
    with pytest.raises(rg.RegionEError) as ei:
        rg.regione_partition_static(None, x_t, v, x_ref, (1 << 22) + 1, 64, rg.BF16, 0.7, 0.9, None, o["mask"], o["e"], o["u"], o["cnt"])
    assert ei.value.code == rg.ERR_WORKSPACE and "limit" in str(ei.value)
    with pytest.raises(rg.RegionEError):
        rg.regione_partition_static(None, x_t, v, x_ref, 16, 64, rg.BF16, 0.7, 0.9, None, o["mask"], o["e"], o["u"], None)
