"""regione_region_step (one call per region-aware step, Algorithm 1's region-aware stage) against the same step made
of the separate calls: identical kernels, so every output is compared bit for bit."""
import dataclasses

import pytest
import torch

from paper_2510_25590_amd import step

pytestmark = pytest.mark.gpu


def _outputs(wl, n):
    torch.cuda.synchronize()
    keys = ("mask", "score", "h_next", "x_next", "k_cache", "v_cache")
    out = {k: getattr(wl, k).clone() for k in keys}
    out["e_index"] = wl.e_index[:n].clone()
    out["u_index"] = wl.u_index[:wl.n_img - n].clone()
    for k in ("v_e", "c_a", "x_e", "h_e_out"):
        out[k] = getattr(wl, k)[:n].clone()
    return out


CASES = [step.CONFIG_TINY, step.CONFIG_TINY_BF16, dataclasses.replace(step.CONFIG_TINY_BF16, text_fresh=True),
         dataclasses.replace(step.CONFIG_TINY_BF16, kind="single"), step.CONFIG_BLOCK,
         dataclasses.replace(step.CONFIG_TINY_BF16, n_edited=1, name="tiny bf16, one token edited"),
         dataclasses.replace(step.CONFIG_TINY_BF16, n_edited=256, name="tiny bf16, every token edited"),
         dataclasses.replace(step.CONFIG_TINY_BF16, n_edited=77, mask="blob", text_fresh=True, extras=True, name="tiny bf16, blobs, extras")]


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: f"{c.name[:24]}-{c.dtype}-{c.kind}-{'txt' if c.text_fresh else 'img'}")
def test_single_call_step_equals_separate_calls(cfg):
    wl = step.RegionStepWorkload(cfg)
    try:
        n_sep = wl.step_separate()
        want = _outputs(wl, n_sep)
        wl.h_next.copy_(wl.h_now); wl.x_next.copy_(wl.x_t)      # as before the first step: a call that writes nothing cannot pass
        wl.v_e.fill_(0); wl.c_a.fill_(0)
        for rep in range(3):                    # the pinned count word is reused from call to call: tickets must not mix
            n = wl.step()
            assert n == n_sep > 0
            got = _outputs(wl, n)
            for k, w in want.items():
                assert torch.equal(got[k], w), (k, rep)
    finally:
        wl.close()


def test_single_call_step_without_edited_tokens():
    cfg = step.CONFIG_TINY_BF16
    wl = step.RegionStepWorkload(cfg)
    try:
        wl.x_t.copy_(wl.x_ref); wl.v_prev.zero_()          # the estimate equals the reference: every score is 1
        before = wl.h_next.clone()
        assert wl.step() == 0
        torch.cuda.synchronize()
        assert int(wl.mask.sum().item()) == 0 and torch.equal(wl.h_next, before)
    finally:
        wl.close()
