"""The allocation-free entry point, dp_per_example_grad_static (built-in 32 MiB device scratch instead of a
caller workspace), against dp_per_example_grad on the same inputs: same kernels, so the same bits.  Two calls in
a row, the second on a smaller input, so stale scratch contents of the first call would show."""
import numpy as np
import pytest
import torch

import paper_2109_12191_amd as dp
from gpu_util import dev
from workloads import conv, dense, gn_affine

pytestmark = pytest.mark.gpu


def _both(layer, n, dtype, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n,) + tuple(layer.x_shape)).astype(np.float32)
    dy = (rng.standard_normal((n,) + tuple(layer.dy_shape)) * 0.01).astype(np.float32)
    xd, dyd = dev(x, dtype), dev(dy, dtype)
    d = dp.make_desc(layer, n, dtype)
    pw, pb = dp.dp_weight_count(d), dp.dp_bias_count(d)
    need = dp.dp_workspace_bytes(d)
    assert need <= dp.dp_static_scratch_bytes()
    res = []
    for static in (False, True):
        gw = torch.full((n, pw), 7.0, device="cuda:0")
        gb = torch.full((n, max(pb, 1)), 7.0, device="cuda:0")
        sq = torch.full((n,), -1.0, device="cuda:0")
        if static:
            dp.dp_per_example_grad_static(d, xd, dyd, gw, gb if pb else None, sq)
        else:
            ws = torch.empty(max(16, need), dtype=torch.uint8, device="cuda:0")
            dp.dp_per_example_grad(d, xd, dyd, gw, gb if pb else None, sq, ws)
        torch.cuda.synchronize()
        res.append((gw, gb, sq))
    (gw0, gb0, sq0), (gw1, gb1, sq1) = res
    assert torch.equal(gw0, gw1) and torch.equal(gb0, gb1) and torch.equal(sq0, sq1)
    assert float(sq1.min()) > 0.0
    # norms only (no gradient written) through the built-in scratch as well
    sq2 = torch.full((n,), -1.0, device="cuda:0")
    dp.dp_per_example_grad_static(d, xd, dyd, None, None, sq2)
    torch.cuda.synchronize()
    ws = torch.empty(max(16, need), dtype=torch.uint8, device="cuda:0")
    sq3 = torch.full((n,), -1.0, device="cuda:0")
    dp.dp_per_example_grad(d, xd, dyd, None, None, sq3, ws)
    torch.cuda.synchronize()
    assert torch.equal(sq2, sq3)


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    assert dp.dp_static_scratch_bytes() == 32 << 20
    # first call: K sliced over workgroups (partial tiles and partial norms go through the scratch)
    _both(conv(64, 64, 3, 1, 56, bias=True), 6, "f32", 1)
    # second call, smaller input, other kernels: partial norms of a 1x1 layer, bf16
    _both(conv(96, 72, 1, 1, 14), 3, "bf16", 2)
    # and the layer kinds without a contraction
    _both(dense(100, 36, tokens=3), 4, "f32", 3)
    _both(gn_affine(32, 10, 8), 5, "f32", 4)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    big = dp.make_desc(conv(64, 64, 3, 1, 56, bias=True), 32, "f32")        # K sliced at n = 32: 45 MiB of partial tiles
    assert dp.dp_workspace_bytes(big) > dp.dp_static_scratch_bytes()
    x = torch.zeros(16, device="cuda:0")
    with pytest.raises(dp.DpError) as ei:
        dp.dp_per_example_grad_static(big, x, x, None, None, x)
    assert ei.value.status == 3 and "built-in scratch" in str(ei.value)
