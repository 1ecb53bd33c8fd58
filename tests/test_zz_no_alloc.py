"""qmm_scale_static (the entry point for callers that cannot allocate: its scratch is an array of the library's device
image) against qmm_scale, through the C ABI, on two calls in a row, the second on a smaller input: step sizes bit
for bit equal, every plan of the scale kernels, and the size limit reported as an error."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2408_02897_amd import qmm, workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def both(L, x, contract_axis, fmt, per_channel, groups):
    t, g = qmm.tensor_desc(x, contract_axis), qmm.granularity(per_channel, groups)
    n = L.qmm_num_scales(ctypes.byref(t), ctypes.byref(g))
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    need = L.qmm_scale_workspace_size(ctypes.byref(t), ctypes.byref(g))
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
    want = torch.full((n,), -1.0, dtype=torch.float32, device=DEV)
    got = torch.full((n,), -2.0, dtype=torch.float32, device=DEV)
    assert L.qmm_scale(ctypes.byref(t), fmt, ctypes.byref(g), want.data_ptr(), ws.data_ptr(), ws.numel(), stream) == 0
    assert L.qmm_scale_static(ctypes.byref(t), fmt, ctypes.byref(g), got.data_ptr(), stream) == 0
    torch.cuda.synchronize()
    return got.cpu().numpy().view(np.uint32), want.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("contract_axis,per_channel,groups", [(1, False, 1), (1, True, 1), (0, True, 1), (1, False, 4), (0, True, 2)])
def test_static_scratch_call_equals_workspace_call_twice_in_a_row(contract_axis, per_channel, groups):
    L = qmm.lib()
    big = W.student_t((4, 1536, 1024), 4, seed=5).to(DEV)             # second call smaller: stale partial maxima of the
    small = W.student_t((4, 200, 136), 4, seed=6).mul(1e-3).to(torch.bfloat16).to(DEV)   # first (larger) must not leak in
    for x in (big, small):
        got, want = both(L, x, contract_axis, qmm.E4M3, per_channel, groups)
        assert np.array_equal(got, want)
    # a third call on an all-zero tensor: every group's step size is 1, whatever the scratch still holds
    z = torch.zeros((4, 64, 64), dtype=torch.bfloat16, device=DEV)
    got, want = both(L, z, contract_axis, qmm.INT8, per_channel, groups)
    assert np.array_equal(got, want) and np.all(got.view(np.float32) == 1.0)


def test_limit_is_an_error_and_leaves_the_output_alone():
    L = qmm.lib()
    # one step size per column of a [batch 8, 8 x 40960] tensor contracting over rows: 8 * 1 * 40960 words > 1 MiB
    x = torch.zeros((8, 8, 40960), dtype=torch.bfloat16, device=DEV)
    t, g = qmm.tensor_desc(x, 0), qmm.granularity(True, 1)
    assert L.qmm_scale_workspace_size(ctypes.byref(t), ctypes.byref(g)) > (1 << 20)
    out = torch.full((40960,), 7.0, dtype=torch.float32, device=DEV)
    assert L.qmm_scale_static(ctypes.byref(t), qmm.E4M3, ctypes.byref(g), out.data_ptr(), None) == 8
    assert "capacity" in qmm.status_string(8)
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)
