"""The statistics entry point that allocates nothing: wmdec_gn_stats_noalloc keeps its partial moments and ticket
counters in a device array built into the library.  Checked through the C ABI against wmdec_gn_stats (same kernels,
hence the same bits) and the oracle, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2602_00608_amd import synth, wmdec
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def both(x_dev, groups, eps):
    n = x_dev.shape[0]
    mean = torch.empty(n * groups, dtype=torch.float32, device="cuda")
    rstd = torch.empty(n * groups, dtype=torch.float32, device="cuda")
    wmdec.gn_stats_noalloc(x_dev, groups, eps, mean, rstd)
    want_mean, want_rstd = G.gn_stats(x_dev, groups, eps)
    torch.cuda.synchronize()
    return mean, rstd, want_mean, want_rstd


def test_noalloc_matches_workspace_entry_point_on_two_calls_in_a_row():
    groups, eps = 32, 1e-6
    r = np.random.default_rng(synth.SEED_BASE + 500)
    # a large input first (many slabs, all 256 slots per group in use), then a smaller one of another layout, then
    # a shape of the general (two-launch) path, then the large one again: the array keeps the last call's contents
    shapes = [("f16", 2, 128, 240, 360), ("f16", 1, 256, 17, 23), ("bf16", 3, 24, 9, 11), ("f32", 1, 64, 32, 32),
              ("f16", 2, 128, 240, 360)]
    for dtype, n, c, h, w in shapes:
        g = groups if c % groups == 0 else 3
        x = G.stored(r.standard_normal((n, c, h, w)) * 1.7 + 0.6, dtype)
        xd = G.dev_nhwc(x, dtype)
        mean, rstd, wm, wr = both(xd, g, eps)
        assert torch.equal(mean, wm) and torch.equal(rstd, wr), (dtype, n, c, h, w)
        om, orr = ref.gn_stats(x, g, eps)
        assert np.max(np.abs(mean.cpu().numpy() - om.ravel()) * orr.ravel()) < 2e-5
        assert np.max(np.abs(rstd.cpu().numpy() / orr.ravel() - 1.0)) < 2e-5


def test_noalloc_rejects_sizes_beyond_the_built_in_scratch():
    # two-launch path (96 channels: 12 vectors per pixel do not divide 1024): 127 slabs x 8 samples x 96 groups x
    # 12 bytes = 1 170 432 bytes, above the 1 048 576 of built-in scratch
    x = torch.zeros((8, 360, 360, 96), dtype=torch.float16, device="cuda")
    mean = torch.full((8 * 96,), 7.0, dtype=torch.float32, device="cuda")
    rstd = mean.clone()
    with pytest.raises(wmdec.WmdecError) as e:
        wmdec.gn_stats_noalloc(x, 96, 1e-6, mean, rstd)
    assert e.value.status == wmdec.ERR_WORKSPACE and "limit" in str(e.value)
    # more samples than the 64 built-in ticket counters
    x = torch.zeros((65, 2, 2, 32), dtype=torch.float16, device="cuda")
    with pytest.raises(wmdec.WmdecError) as e:
        wmdec.gn_stats_noalloc(x, 32, 1e-6, torch.zeros(65 * 32, device="cuda"), torch.zeros(65 * 32, device="cuda"))
    assert e.value.status == wmdec.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((mean == 7.0).all()) and bool((rstd == 7.0).all())      # nothing was launched
