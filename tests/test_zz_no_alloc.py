"""The entry point that allocates nothing (conv_direct_noalloc) against conv_direct, through the C ABI."""
import gc

import numpy as np
import pytest

from paper_2012_15667_amd.inputs import make_inputs

pytestmark = pytest.mark.gpu


def test_noalloc_entry_point_matches_conv_direct_on_two_calls_in_a_row():
    import torch
    from paper_2012_15667_amd import binding as B
    assert torch.cuda.is_available()
    B.lib()
    # two calls in a row, the second with a smaller layer: what the first left in the shared scratch array
    # must not leak into the second
    first = True
    for (N, C, H, W, K, R, S, stride, pad) in [(4, 40, 28, 28, 96, 3, 3, 1, 1), (2, 12, 14, 14, 32, 3, 3, 1, 1),
                                               (2, 5, 9, 11, 6, 3, 3, 2, 1), (3, 16, 16, 16, 64, 1, 1, 1, 0)]:
        x, w = make_inputs(N, C, H, W, K, R, S, "u11", "he", seed=900 + C)
        xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
        ref = B.conv_direct(xd, wd, stride, pad)
        y = torch.full_like(ref, float("nan"))
        if first:
            # set-up on the first call on a device: the code object with the static array is loaded, its address
            # looked up; device memory is taken then, not by later calls
            B.conv_direct_noalloc(xd, wd, stride, pad, y)
            y.fill_(float("nan"))
            first = False
        # nothing may be allocated by the call: neither through torch (its count of allocations made so far, which
        # frees by the garbage collector do not change) nor behind its back (free device memory does not shrink)
        gc.collect()
        torch.cuda.synchronize()
        allocations = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
        free_before = torch.cuda.mem_get_info()[0]
        B.conv_direct_noalloc(xd, wd, stride, pad, y)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats().get("allocation.all.allocated", 0) == allocations
        assert torch.cuda.mem_get_info()[0] >= free_before
        assert torch.equal(y, ref), (N, C, H, W, K)


def test_noalloc_entry_point_rejects_layers_beyond_its_scratch():
    import ctypes
    import torch
    from paper_2012_15667_amd import binding as B
    L = B.lib()
    limit = L.conv_direct_noalloc_max_weight_floats()
    assert limit == 4 << 20
    # 1024 x 1024 kernels of 3 x 3: 9.4 M floats of re-laid-out weights; nothing may be written
    N, C, H, W, K = 1, 1024, 8, 8, 1024
    xd = torch.zeros((N, C, H, W), device="cuda")
    wd = torch.zeros((K, C, 3, 3), device="cuda")
    y = torch.full((N, K, H, W), 7.0, device="cuda")
    with pytest.raises(B.IolbError) as e:
        B.conv_direct_noalloc(xd, wd, 1, 1, y)
    assert e.value.code == -4
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
    assert L.conv_direct_noalloc(None, None, None, 1, 1, 4, 4, 1, 3, 3, 1, 1) == -1
