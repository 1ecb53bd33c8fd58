"""CPU-only checks of the C-ABI library: it loads, exports every symbol include/qmm.h declares, and
rejects bad arguments before touching the GPU (so these calls are safe without one)."""
import ctypes
import os
import re

import pytest

from paper_2408_02897_amd import qmm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(qmm.LIB_PATH):
        from paper_2408_02897_amd import build
        build.build()
    return qmm.lib()


def test_exports_match_header(L):
    hdr = open(os.path.join(ROOT, "include", "qmm.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(qmm_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(qmm.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name
    assert L.qmm_version() == 100
    assert qmm.status_string(0) == "ok" and "NULL" in qmm.status_string(1)


def test_num_scales_and_workspace_sizes(L):
    t = qmm.Tensor(None, qmm.DT_BF16, 1, 4, 10, 32, 320, 32)
    g = qmm.granularity(False, 1)
    assert L.qmm_num_scales(ctypes.byref(t), ctypes.byref(g)) == 1
    g = qmm.granularity(True, 2)
    assert L.qmm_num_scales(ctypes.byref(t), ctypes.byref(g)) == 20
    t.contract_axis = 0
    assert L.qmm_num_scales(ctypes.byref(t), ctypes.byref(g)) == 64
    assert L.qmm_scale_workspace_size(ctypes.byref(t), ctypes.byref(g)) >= 4 * 32 * 4
    assert L.qmm_metric_workspace_size(0) >= 128 and L.qmm_metric_workspace_size(1 << 30) <= 2048 * 128


def test_argument_errors_are_reported_before_any_launch(L):
    g = qmm.granularity(False, 1)
    t = qmm.Tensor(None, qmm.DT_BF16, 1, 1, 4, 16, 64, 16)
    fake = ctypes.c_void_p(0x1000)
    # NULL output
    assert L.qmm_scale(ctypes.byref(t), qmm.E4M3, ctypes.byref(g), None, fake, 1024, None) == 1
    # bad format / bad axis / bad shape / missing workspace
    assert L.qmm_scale(ctypes.byref(t), 7, ctypes.byref(g), fake, fake, 1024, None) == 3
    t2 = qmm.Tensor(None, qmm.DT_BF16, 2, 1, 4, 16, 64, 16)
    assert L.qmm_scale(ctypes.byref(t2), qmm.E4M3, ctypes.byref(g), fake, fake, 1024, None) == 3
    t3 = qmm.Tensor(None, qmm.DT_BF16, 1, 1, 4, 16, 64, 8)
    assert L.qmm_scale(ctypes.byref(t3), qmm.E4M3, ctypes.byref(g), fake, fake, 1024, None) == 2
    t4 = qmm.Tensor(fake, qmm.DT_BF16, 1, 1, 4, 16, 64, 16)
    assert L.qmm_scale(ctypes.byref(t4), qmm.E4M3, ctypes.byref(g), fake, None, 0, None) == 6
    assert L.qmm_quantize(ctypes.byref(t4), qmm.E4M3, ctypes.byref(g), fake, 5, 0, 0, fake, None) == 3
    # the entry point with the library's own scratch: same argument errors, and its size limit, all on the host
    assert L.qmm_scale_static(ctypes.byref(t), qmm.E4M3, ctypes.byref(g), None, None) == 1
    assert L.qmm_scale_static(ctypes.byref(t), 7, ctypes.byref(g), fake, None) == 3
    assert L.qmm_scale_static(ctypes.byref(t3), qmm.E4M3, ctypes.byref(g), fake, None) == 2
    wide = qmm.Tensor(fake, qmm.DT_BF16, 0, 8, 8, 40960, 8 * 40960, 40960)      # per-column maxima of 8 matrices: > 1 MiB of partials
    assert L.qmm_scale_static(ctypes.byref(wide), qmm.E4M3, ctypes.byref(qmm.granularity(True, 1)), fake, None) == 8
    bad = qmm.granularity(False, 1, -1)                       # negative run length of the scale groups
    assert L.qmm_scale(ctypes.byref(t4), qmm.E4M3, ctypes.byref(bad), fake, fake, 1024, None) == 3
    assert L.qmm_quantize(ctypes.byref(t4), qmm.E4M3, ctypes.byref(bad), fake, 0, 0, 0, fake, None) == 3
    assert L.qmm_quantize(ctypes.byref(t4), qmm.E4M3, ctypes.byref(g), None, 0, 0, 0, fake, None) == 1
    oa = qmm.Operand(fake, qmm.E4M3, 1, fake, g); ob = qmm.Operand(fake, qmm.INT8, 1, fake, g)
    assert L.qmm_gemm(ctypes.byref(oa), ctypes.byref(ob), 1, 16, 16, 16, fake, 1, None, None, 0, None) == 5
    ob = qmm.Operand(fake, qmm.E5M2, 1, fake, g)
    assert L.qmm_gemm(ctypes.byref(oa), ctypes.byref(ob), 1, 16, 16, 24, fake, 1, None, None, 0, None) == 4
    assert L.qmm_gemm(ctypes.byref(oa), ctypes.byref(ob), 1, 16, 16, 32, None, 1, None, None, 0, None) == 1
    assert L.qmm_gemm(ctypes.byref(oa), ctypes.byref(ob), 1, -1, 16, 32, fake, 1, None, None, 0, None) == 2
    assert L.qmm_metric(fake, 1, fake, None, 8, None, fake, 1 << 20, None) == 1
    assert L.qmm_metric(fake, 1, fake, None, 8, fake, None, 0, None) == 6
    assert L.qmm_metric(fake, 9, fake, None, 8, fake, fake, 1 << 20, None) == 3
    # split-K shapes need the workspace they ask for
    assert L.qmm_gemm_workspace_size(ctypes.byref(oa), ctypes.byref(ob), 1, 256, 256, 8192) == 8 * 256 * 256 * 4
    assert L.qmm_gemm_workspace_size(ctypes.byref(oa), ctypes.byref(ob), 1, 4096, 4096, 8192) == 0
    assert L.qmm_gemm(ctypes.byref(oa), ctypes.byref(ob), 1, 256, 256, 8192, fake, 1, None, None, 0, None) == 6
    assert L.qmm_gemm(ctypes.byref(oa), ctypes.byref(ob), 1, 16, 16, (1 << 22) + 16, fake, 1, None, None, 0, None) == 5
    # moments
    assert L.qmm_moments_workspace_size(0) >= 56 and L.qmm_moments_workspace_size(1 << 34) <= 2048 * 56
    assert L.qmm_moments(fake, 0, 8, 0.0, None, fake, 1 << 20, None) == 1
    assert L.qmm_moments(fake, 5, 8, 0.0, fake, fake, 1 << 20, None) == 3
    assert L.qmm_moments(fake, 0, -1, 0.0, fake, fake, 1 << 20, None) == 2
    assert L.qmm_moments(fake, 0, 8, float("nan"), fake, fake, 1 << 20, None) == 2
    assert L.qmm_moments(fake, 0, 8, float("inf"), fake, fake, 1 << 20, None) == 2
    assert L.qmm_moments(fake, 0, 8, 0.0, fake, None, 0, None) == 6
    assert L.qmm_moments(ctypes.c_void_p(0x1004), 0, 8, 0.0, fake, fake, 1 << 20, None) == 4
    # matrix-rate probe
    assert L.qmm_mfma_rate(qmm.E4M3, qmm.INT8, fake, 1024, 1, 1, fake, ctypes.byref(ctypes.c_double()), None) == 5
    assert L.qmm_mfma_rate(qmm.E4M3, qmm.E4M3, None, 1024, 1, 1, fake, ctypes.byref(ctypes.c_double()), None) == 1
    assert L.qmm_mfma_rate(qmm.E4M3, qmm.E4M3, fake, 8, 1, 1, fake, ctypes.byref(ctypes.c_double()), None) == 2
    # dequantize
    assert L.qmm_dequantize(fake, 1, 4, 16, qmm.E4M3, ctypes.byref(g), fake, None, 1, None) == 1
    assert L.qmm_dequantize(fake, 1, 4, 16, 9, ctypes.byref(g), fake, fake, 1, None) == 3
    assert L.qmm_dequantize(fake, 1, -4, 16, qmm.E4M3, ctypes.byref(g), fake, fake, 1, None) == 2
    assert L.qmm_dequantize(None, 1, 4, 16, qmm.E4M3, ctypes.byref(g), fake, fake, 1, None) == 1
    assert L.qmm_dequantize(fake, 1, 4, 16, qmm.E4M3, ctypes.byref(g), fake, ctypes.c_void_p(0x1002), 1, None) == 4
    assert L.qmm_dequantize(None, 0, 4, 16, qmm.E4M3, ctypes.byref(g), None, fake, 1, None) == 0


def test_gemm_nsr_argument_errors(L):
    fake = ctypes.c_void_p(0x1000)
    ga = qmm.granularity(False, 1)
    codes = qmm.Operand(fake, qmm.E4M3, 1, fake, ga)
    raw = qmm.Operand(fake, qmm.E4M3, 0, fake, ga)               # quantize-on-load operand
    bf = qmm.Operand(fake, qmm.BF16, 0, None, ga)
    need = L.qmm_gemm_nsr_workspace_size(1, 256, 256)
    assert need >= 4 * 4 * 16 and L.qmm_gemm_nsr_workspace_size(-1, 1, 1) == 0
    args = (1, 256, 256, 128)
    call = lambda a, b, y, ref, out2, ws, nws: L.qmm_gemm_nsr(ctypes.byref(a), ctypes.byref(b), *args, y, qmm.DT_BF16, ref, out2, ws, nws, None)
    assert call(codes, codes, fake, None, fake, fake, need) == 1            # no reference
    assert call(codes, codes, None, fake, fake, fake, need) == 1            # no output
    assert call(codes, codes, fake, fake, None, fake, need) == 1            # no place for the sums
    assert call(raw, codes, fake, fake, fake, fake, need) == 5              # quantize-on-load operand
    assert call(bf, bf, fake, fake, fake, fake, need) == 5                  # reference product
    assert call(codes, codes, fake, fake, fake, None, 0) == 6               # no workspace
    assert call(codes, codes, fake, fake, fake, fake, need - 1) == 6        # workspace too small
    assert call(codes, codes, fake, ctypes.c_void_p(0x1004), fake, fake, need) == 4   # misaligned reference


def test_multi_tensor_argument_errors(L):
    """qmm_scale_multi / qmm_quantize_multi report argument errors before any launch (no GPU needed)."""
    n = 2
    ts = (qmm.Tensor * n)(qmm.Tensor(None, qmm.DT_BF16, 1, 1, 4, 16, 64, 16), qmm.Tensor(None, qmm.DT_BF16, 1, 1, 8, 32, 256, 32))
    gs = (qmm.Granularity * n)(qmm.granularity(False, 1), qmm.granularity(False, 1))
    fake = ctypes.c_void_p(0x1000)
    ptrs = (ctypes.c_void_p * n)(0x1000, 0x2000)
    need = L.qmm_scale_multi_workspace_size(n, ts, gs)
    assert need >= 32 and need % 16 == 0
    assert L.qmm_scale_multi_workspace_size(0, ts, gs) == 0
    assert L.qmm_scale_multi(0, ts, qmm.E4M3, gs, ptrs, None, 0, None) == 0            # nothing to do
    assert L.qmm_scale_multi(-1, ts, qmm.E4M3, gs, ptrs, fake, 1024, None) == 2
    assert L.qmm_scale_multi(n, None, qmm.E4M3, gs, ptrs, fake, 1024, None) == 1
    assert L.qmm_scale_multi(n, ts, 9, gs, ptrs, fake, 1024, None) == 3
    assert L.qmm_scale_multi(n, ts, qmm.E4M3, gs, ptrs, fake, need - 1, None) == 6
    assert L.qmm_scale_multi(n, ts, qmm.E4M3, gs, ptrs, ctypes.c_void_p(0x1004), 1024, None) == 4
    assert L.qmm_quantize_multi(0, ts, qmm.E4M3, gs, ptrs, qmm.RTNE, 0, None, ptrs, None) == 0
    assert L.qmm_quantize_multi(-1, ts, qmm.E4M3, gs, ptrs, qmm.RTNE, 0, None, ptrs, None) == 2
    assert L.qmm_quantize_multi(n, ts, qmm.E4M3, gs, None, qmm.RTNE, 0, None, ptrs, None) == 1
    assert L.qmm_quantize_multi(n, ts, 9, gs, ptrs, qmm.RTNE, 0, None, ptrs, None) == 3
    assert L.qmm_quantize_multi(n, ts, qmm.E4M3, gs, ptrs, 5, 0, None, ptrs, None) == 3
    # tensors with NULL data go to the single-tensor code, which reports them
    assert L.qmm_quantize_multi(n, ts, qmm.E4M3, gs, ptrs, qmm.RTNE, 0, None, ptrs, None) == 1


def test_measurement_aids_reject_bad_arguments(L):
    fake = ctypes.c_void_p(0x1000)
    assert L.qmm_hbm_rate(None, None, 1024, 64, fake, None) == 1            # no source
    assert L.qmm_hbm_rate(fake, None, 1024, 64, None, None) == 1            # read-only needs a sink
    assert L.qmm_hbm_rate(fake, None, -16, 64, fake, None) == 2
    assert L.qmm_hbm_rate(fake, None, 1024, 0, fake, None) == 2
    assert L.qmm_hbm_rate(fake, None, 1000, 64, fake, None) == 4            # not a multiple of 16 bytes
    assert L.qmm_hbm_rate(ctypes.c_void_p(0x1008), None, 1024, 64, fake, None) == 4
    assert L.qmm_hbm_rate(fake, None, 0, 64, fake, None) == 0               # nothing to do, nothing launched
