"""The allocation-free entry point (library-owned static workspace) against wq_conv_forward."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2412_19867_amd import workloads

pytestmark = pytest.mark.gpu


def _setup(wq, d, variant=None):
    lay = d.layer
    plan = wq.Plan(lay.N, lay.H, lay.W, lay.Cin, lay.Cout, lay.m, lay.group_size)
    if variant:
        plan.tune(0, variant)
    blob, ws = plan.alloc_blob(), plan.alloc_workspace()
    x = torch.from_numpy(d.x).cuda()
    plan.weight_prepare(torch.from_numpy(d.w).cuda(), torch.from_numpy(d.bias).cuda(), blob)
    want = plan.alloc_output()
    plan.forward(x, blob, ws, want)
    torch.cuda.synchronize()
    return plan, blob, x, want


def test_static_workspace_entry_point_matches_the_plain_one(wq):
    """Two calls in a row on the same GPU, the second with a smaller layer (the static array then
    still holds the first call's data beyond the second layer's workspace): both equal
    wq_conv_forward's output bit for bit.  Covers a one-kernel and a two-kernel variant."""
    big = workloads.small_layer(301, 2, 40, 36, 128, 96, 4, 64)          # ~6 MB of workspace
    small = workloads.small_layer(302, 1, 9, 11, 64, 40, 6, 32)
    for variants in ((None, None), ("gemm_64x64", "lds_row_64x64"), ("lds_full_64x64", "fused_16x16")):
        ctx = [_setup(wq, d, v) for d, v in zip((big, small), variants)]
        assert ctx[0][0].layout.ws_bytes > ctx[1][0].layout.ws_bytes
        for plan, blob, x, want in ctx:                                   # big first, then small
            assert plan.layout.ws_bytes <= wq.STATIC_WORKSPACE_BYTES
            y = plan.alloc_output()
            y.fill_(float("nan"))
            mem = torch.cuda.memory_allocated()
            plan.forward_static(x, blob, y)
            assert torch.cuda.memory_allocated() == mem
            torch.cuda.synchronize()
            assert torch.equal(y, want)
        for plan, blob, x, want in ctx:                                   # and once more, same order
            y = torch.empty_like(want)
            plan.forward_static(x, blob, y)
            torch.cuda.synchronize()
            assert torch.equal(y, want)


def test_static_workspace_entry_point_rejects_what_does_not_fit(wq):
    lay = workloads.CONFIGS[5][0]                                         # 119 MB of workspace
    plan = wq.Plan(lay.N, lay.H, lay.W, lay.Cin, lay.Cout, lay.m, lay.group_size)
    assert plan.layout.ws_bytes > wq.STATIC_WORKSPACE_BYTES
    x = torch.zeros(lay.N * lay.H * lay.W * lay.Cin, device="cuda")
    y = plan.alloc_output()
    blob = plan.alloc_blob()
    with pytest.raises(wq.WqError) as e:
        plan.forward_static(x, blob, y)
    assert e.value.status == 5                                            # WQ_ERR_WORKSPACE
    assert wq.lib().wq_conv_forward_static(None, None, None, None, 0, None) == 1
