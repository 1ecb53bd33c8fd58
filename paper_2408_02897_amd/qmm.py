"""Thin ctypes binding of libqmm.so (include/qmm.h).  Argument marshalling only: every step of the
path runs in the HIP kernels.  torch is used for device memory and the current stream.  There is no
CPU fallback: a missing or unloadable library raises."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqmm.so")

INT8, E4M3, E5M2, BF16 = 0, 1, 2, 3
DT_BF16, DT_F32 = 0, 1
RTNE, STOCHASTIC = 0, 1
FORMATS = {"int8": INT8, "e4m3": E4M3, "e5m2": E5M2, "bf16": BF16}
EXPORTS = ["qmm_num_scales", "qmm_scale_workspace_size", "qmm_scale", "qmm_scale_static", "qmm_quantize", "qmm_scale_multi_workspace_size", "qmm_scale_multi", "qmm_quantize_multi",
           "qmm_gemm_workspace_size",
           "qmm_gemm", "qmm_gemm_nsr_workspace_size", "qmm_gemm_nsr", "qmm_metric_workspace_size", "qmm_metric", "qmm_dequantize", "qmm_moments_workspace_size", "qmm_moments", "qmm_mfma_rate", "qmm_hbm_rate", "qmm_status_string", "qmm_version"]


class QmmError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


class Tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("dtype", ctypes.c_int32), ("contract_axis", ctypes.c_int32),
                ("batch", ctypes.c_int64), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("batch_stride", ctypes.c_int64), ("row_stride", ctypes.c_int64)]


class Granularity(ctypes.Structure):
    _fields_ = [("per_channel", ctypes.c_int32), ("batch_inner", ctypes.c_int32), ("batch_groups", ctypes.c_int64)]


class Operand(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("format", ctypes.c_int32), ("is_codes", ctypes.c_int32),
                ("delta", ctypes.c_void_p), ("gran", Granularity)]


_lib = None


def lib():
    """Load libqmm.so (built in-tree by paper_2408_02897_amd.build).  Raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2408_02897_amd.build` first "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, u64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int, ctypes.c_size_t
        TP, GP, OP = ctypes.POINTER(Tensor), ctypes.POINTER(Granularity), ctypes.POINTER(Operand)
        L.qmm_num_scales.restype = i64; L.qmm_num_scales.argtypes = [TP, GP]
        L.qmm_scale_workspace_size.restype = sz; L.qmm_scale_workspace_size.argtypes = [TP, GP]
        L.qmm_scale.restype = i32; L.qmm_scale.argtypes = [TP, i32, GP, vp, vp, sz, vp]
        L.qmm_scale_static.restype = i32; L.qmm_scale_static.argtypes = [TP, i32, GP, vp, vp]
        L.qmm_quantize.restype = i32; L.qmm_quantize.argtypes = [TP, i32, GP, vp, i32, u64, u64, vp, vp]
        L.qmm_scale_multi_workspace_size.restype = sz; L.qmm_scale_multi_workspace_size.argtypes = [i32, vp, vp]
        L.qmm_scale_multi.restype = i32; L.qmm_scale_multi.argtypes = [i32, vp, i32, vp, vp, vp, sz, vp]
        L.qmm_quantize_multi.restype = i32; L.qmm_quantize_multi.argtypes = [i32, vp, i32, vp, vp, i32, u64, vp, vp, vp]
        L.qmm_gemm_workspace_size.restype = sz; L.qmm_gemm_workspace_size.argtypes = [OP, OP, i64, i64, i64, i64]
        L.qmm_gemm.restype = i32; L.qmm_gemm.argtypes = [OP, OP, i64, i64, i64, i64, vp, i32, vp, vp, sz, vp]
        L.qmm_gemm_nsr_workspace_size.restype = sz; L.qmm_gemm_nsr_workspace_size.argtypes = [i64, i64, i64]
        L.qmm_gemm_nsr.restype = i32; L.qmm_gemm_nsr.argtypes = [OP, OP, i64, i64, i64, i64, vp, i32, vp, vp, vp, sz, vp]
        L.qmm_metric_workspace_size.restype = sz; L.qmm_metric_workspace_size.argtypes = [i64]
        L.qmm_metric.restype = i32; L.qmm_metric.argtypes = [vp, i32, vp, vp, i64, vp, vp, sz, vp]
        L.qmm_dequantize.restype = i32; L.qmm_dequantize.argtypes = [vp, i64, i64, i64, i32, GP, vp, vp, i32, vp]
        L.qmm_moments_workspace_size.restype = sz; L.qmm_moments_workspace_size.argtypes = [i64]
        L.qmm_moments.restype = i32; L.qmm_moments.argtypes = [vp, i32, i64, ctypes.c_double, vp, vp, sz, vp]
        L.qmm_mfma_rate.restype = i32
        L.qmm_mfma_rate.argtypes = [i32, i32, vp, i64, i64, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.qmm_hbm_rate.restype = i32; L.qmm_hbm_rate.argtypes = [vp, vp, i64, i32, vp, vp]
        L.qmm_status_string.restype = ctypes.c_char_p; L.qmm_status_string.argtypes = [i32]
        L.qmm_version.restype = i32; L.qmm_version.argtypes = []
        _lib = L
    return _lib


def status_string(status):
    return lib().qmm_status_string(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise QmmError(status, where)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return DT_BF16
    if t.dtype == torch.float32:
        return DT_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def tensor_desc(x, contract_axis):
    """Descriptor of a 2-D [rows, cols] or 3-D [batch, rows, cols] device tensor with contiguous columns."""
    if x.dim() == 2:
        x = x.unsqueeze(0)
    assert x.dim() == 3 and x.is_cuda
    assert x.stride(2) == 1 or x.shape[2] <= 1, "columns must be contiguous"
    b, r, c = x.shape
    return Tensor(x.data_ptr(), _dtype_code(x), contract_axis, b, r, c, x.stride(0), x.stride(1))


def granularity(per_channel=False, batch_groups=1, batch_inner=1):
    """Scale group of matrix b: (b // batch_inner) % batch_groups."""
    return Granularity(int(per_channel), int(batch_inner), int(batch_groups))


def _workspace(nbytes, device):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


def scale(x, contract_axis, fmt, per_channel=False, batch_groups=1, out=None, workspace=None, batch_inner=1):
    """qmm_scale: step sizes (float32 device tensor of qmm_num_scales elements)."""
    L = lib()
    t, g = tensor_desc(x, contract_axis), granularity(per_channel, batch_groups, batch_inner)
    n = L.qmm_num_scales(ctypes.byref(t), ctypes.byref(g))
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=x.device)
    need = L.qmm_scale_workspace_size(ctypes.byref(t), ctypes.byref(g))
    if workspace is None:
        workspace = _workspace(need, x.device)
    _check(L.qmm_scale(ctypes.byref(t), fmt, ctypes.byref(g), out.data_ptr(), workspace.data_ptr(),
                       workspace.numel(), _stream()), "qmm_scale")
    return out


def scale_static(x, contract_axis, fmt, per_channel=False, batch_groups=1, out=None, batch_inner=1):
    """qmm_scale_static: qmm_scale with the library's own scratch array (no workspace, nothing allocated by the call
    itself when `out` is given)."""
    L = lib()
    t, g = tensor_desc(x, contract_axis), granularity(per_channel, batch_groups, batch_inner)
    if out is None:
        out = torch.empty(L.qmm_num_scales(ctypes.byref(t), ctypes.byref(g)), dtype=torch.float32, device=x.device)
    _check(L.qmm_scale_static(ctypes.byref(t), fmt, ctypes.byref(g), out.data_ptr(), _stream()), "qmm_scale_static")
    return out


def quantize(x, contract_axis, fmt, delta, per_channel=False, batch_groups=1, mode=RTNE, seed=0, offset=0, out=None,
             batch_inner=1):
    """qmm_quantize: uint8 codes [batch, non-contracting, contracting]."""
    L = lib()
    t, g = tensor_desc(x, contract_axis), granularity(per_channel, batch_groups, batch_inner)
    nc, kc = (t.rows, t.cols) if contract_axis == 1 else (t.cols, t.rows)
    if out is None:
        out = torch.empty((t.batch, nc, kc), dtype=torch.uint8, device=x.device)
    assert delta.dtype == torch.float32 and delta.numel() == L.qmm_num_scales(ctypes.byref(t), ctypes.byref(g))
    _check(L.qmm_quantize(ctypes.byref(t), fmt, ctypes.byref(g), delta.data_ptr(), mode, seed, offset,
                          out.data_ptr(), _stream()), "qmm_quantize")
    return out


class MultiDesc:
    """Host-side argument arrays of qmm_scale_multi / qmm_quantize_multi for a fixed list of tensors (built once,
    reused: the arrays hold raw pointers, the object keeps their owners alive)."""
    def __init__(self, xs, contract_axis=1, per_channel=False, batch_groups=1):
        n = len(xs)
        self.count = n
        self.t = (Tensor * n)(*[tensor_desc(x, contract_axis) for x in xs])
        self.g = (Granularity * n)(*[granularity(per_channel, batch_groups) for _ in xs])
        self._keep = list(xs)
        self.device = xs[0].device
        self.shapes = [(d.batch, d.rows, d.cols) if contract_axis == 1 else (d.batch, d.cols, d.rows) for d in self.t]
        self.num_scales = [lib().qmm_num_scales(ctypes.byref(self.t[i]), ctypes.byref(self.g[i])) for i in range(n)]

    @staticmethod
    def pointers(tensors):
        arr = (ctypes.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
        arr._keep = list(tensors)
        return arr


def scale_multi(desc, fmt, outs=None, workspace=None, out_ptrs=None):
    """qmm_scale_multi on a MultiDesc: list of step-size tensors."""
    L = lib()
    if outs is None:
        outs = [torch.empty(n, dtype=torch.float32, device=desc.device) for n in desc.num_scales]
    if out_ptrs is None:
        out_ptrs = MultiDesc.pointers(outs)
    if workspace is None:
        workspace = _workspace(L.qmm_scale_multi_workspace_size(desc.count, desc.t, desc.g), desc.device)
    _check(L.qmm_scale_multi(desc.count, desc.t, fmt, desc.g, out_ptrs, workspace.data_ptr(), workspace.numel(), _stream()),
           "qmm_scale_multi")
    return outs


def quantize_multi(desc, fmt, deltas, mode=RTNE, seed=0, offsets=None, outs=None, delta_ptrs=None, out_ptrs=None):
    """qmm_quantize_multi on a MultiDesc: list of uint8 code tensors."""
    L = lib()
    if outs is None:
        outs = [torch.empty(s, dtype=torch.uint8, device=desc.device) for s in desc.shapes]
    if delta_ptrs is None:
        delta_ptrs = MultiDesc.pointers(deltas)
    if out_ptrs is None:
        out_ptrs = MultiDesc.pointers(outs)
    offs = (ctypes.c_uint64 * desc.count)(*offsets) if offsets is not None else None
    _check(L.qmm_quantize_multi(desc.count, desc.t, fmt, desc.g, delta_ptrs, mode, seed, offs, out_ptrs, _stream()),
           "qmm_quantize_multi")
    return outs


def operand(data, fmt, delta=None, per_channel=False, batch_groups=1, is_codes=True, batch_inner=1):
    assert data.is_contiguous()
    op = Operand(data.data_ptr(), fmt, int(is_codes), delta.data_ptr() if delta is not None else None,
                 granularity(per_channel, batch_groups, batch_inner))
    op._keep = (data, delta)   # the struct holds raw device pointers: keep their owners alive with it
    return op


def gemm(a, b, out_dtype=torch.float32, want_acc=False, out=None, acc_out=None, want_y=True):
    """qmm_gemm on two (data, Operand) pairs built by `operand`: a = (tensor [batch,M,K], Operand) etc.
    Returns y (and the raw accumulators when want_acc)."""
    L = lib()
    (ta, oa), (tb, ob) = a, b
    if ta.dim() == 2:
        ta = ta.unsqueeze(0); tb = tb.unsqueeze(0)
    bt, m, k = ta.shape
    n = tb.shape[1]
    assert tb.shape[0] == bt and tb.shape[2] == k
    dev = ta.device
    y = out
    if y is None and want_y:
        y = torch.empty((bt, m, n), dtype=out_dtype, device=dev)
    acc = acc_out
    if acc is None and want_acc:
        acc = torch.empty((bt, m, n), dtype=torch.int32 if oa.format == INT8 else torch.float32, device=dev)
    need = L.qmm_gemm_workspace_size(ctypes.byref(oa), ctypes.byref(ob), bt, m, n, k)
    ws = _workspace(need, dev)
    ydt = DT_BF16 if (y is not None and y.dtype == torch.bfloat16) else DT_F32
    _check(L.qmm_gemm(ctypes.byref(oa), ctypes.byref(ob), bt, m, n, k, y.data_ptr() if y is not None else None, ydt,
                      acc.data_ptr() if acc is not None else None, ws.data_ptr(), ws.numel(), _stream()), "qmm_gemm")
    return (y, acc) if want_acc else y


def gemm_nsr(a, b, y_ref, out_dtype=torch.bfloat16, out=None, out2=None, workspace=None):
    """qmm_gemm_nsr: y as `gemm` gives it, and a device tensor of 2 float64: sum (y - y_ref)^2, sum y_ref^2."""
    L = lib()
    (ta, oa), (tb, ob) = a, b
    if ta.dim() == 2:
        ta = ta.unsqueeze(0); tb = tb.unsqueeze(0)
    bt, m, k = ta.shape
    n = tb.shape[1]
    assert tb.shape[0] == bt and tb.shape[2] == k
    assert y_ref.dtype == torch.float32 and y_ref.is_contiguous() and y_ref.numel() == bt * m * n
    dev = ta.device
    y = out if out is not None else torch.empty((bt, m, n), dtype=out_dtype, device=dev)
    if out2 is None:
        out2 = torch.empty(2, dtype=torch.float64, device=dev)
    ws = workspace if workspace is not None else _workspace(L.qmm_gemm_nsr_workspace_size(bt, m, n), dev)
    ydt = DT_BF16 if y.dtype == torch.bfloat16 else DT_F32
    _check(L.qmm_gemm_nsr(ctypes.byref(oa), ctypes.byref(ob), bt, m, n, k, y.data_ptr(), ydt, y_ref.data_ptr(),
                          out2.data_ptr(), ws.data_ptr(), ws.numel(), _stream()), "qmm_gemm_nsr")
    return y, out2


def quantized_operand(x, contract_axis, fmt, per_channel=False, batch_groups=1, mode=RTNE, seed=0, batch_inner=1):
    """scale + quantize; returns ((codes, Operand), delta)."""
    d = scale(x, contract_axis, fmt, per_channel, batch_groups, batch_inner=batch_inner)
    c = quantize(x, contract_axis, fmt, d, per_channel, batch_groups, mode, seed, batch_inner=batch_inner)
    return (c, operand(c, fmt, d, per_channel, batch_groups, batch_inner=batch_inner)), d


def reference_gemm(x, w, out=None):
    """High-precision product of bfloat16 operands x [batch,M,K], w [batch,N,K] -> float32."""
    assert x.dtype == torch.bfloat16 and w.dtype == torch.bfloat16
    x = x.contiguous(); w = w.contiguous()
    return gemm((x, operand(x, BF16, is_codes=False)), (w, operand(w, BF16, is_codes=False)), torch.float32, out=out)


def metric(y, y_ref, denom=None, out=None, workspace=None):
    """qmm_metric: 16 float64 on the device (layout in include/qmm.h)."""
    L = lib()
    assert y.is_contiguous() and y_ref.is_contiguous() and y_ref.dtype == torch.float32
    n = y.numel()
    assert y_ref.numel() == n and (denom is None or (denom.numel() == n and denom.dtype == torch.float32))
    if out is None:
        out = torch.empty(16, dtype=torch.float64, device=y.device)
    if workspace is None:
        workspace = _workspace(L.qmm_metric_workspace_size(n), y.device)
    _check(L.qmm_metric(y.data_ptr(), _dtype_code(y), y_ref.data_ptr(), denom.data_ptr() if denom is not None else None,
                        n, out.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()), "qmm_metric")
    return out


def dequantize(codes, fmt, delta, per_channel=False, batch_groups=1, out_dtype=torch.float32, out=None, batch_inner=1):
    """qmm_dequantize: values of the uint8 device tensor codes [batch, rows, K] (or [rows, K])."""
    L = lib()
    assert codes.dtype == torch.uint8 and codes.is_contiguous() and codes.is_cuda
    c3 = codes if codes.dim() == 3 else codes.unsqueeze(0)
    b, r, k = c3.shape
    g = granularity(per_channel, batch_groups, batch_inner)
    assert delta.dtype == torch.float32 and delta.numel() == batch_groups * (r if per_channel else 1)
    if out is None:
        out = torch.empty(codes.shape, dtype=out_dtype, device=codes.device)
    _check(L.qmm_dequantize(codes.data_ptr(), b, r, k, fmt, ctypes.byref(g), delta.data_ptr(), out.data_ptr(),
                            _dtype_code(out), _stream()), "qmm_dequantize")
    return out


MOMENT_FIELDS = ("n", "mean", "m2", "m3", "m4", "absmax", "nan_cnt", "rsv")


def moments(x, center=0.0, out=None, workspace=None):
    """qmm_moments over all elements of the contiguous device tensor x: 8 float64 on the device (MOMENT_FIELDS)."""
    L = lib()
    assert x.is_contiguous() and x.is_cuda
    n = x.numel()
    if out is None:
        out = torch.empty(8, dtype=torch.float64, device=x.device)
    if workspace is None:
        workspace = _workspace(L.qmm_moments_workspace_size(n), x.device)
    _check(L.qmm_moments(x.data_ptr(), _dtype_code(x), n, float(center), out.data_ptr(), workspace.data_ptr(),
                         workspace.numel(), _stream()), "qmm_moments")
    return out


def mfma_rate(codes, fmt_a, fmt_b, rounds=2000, workgroups=None, sink=None):
    """qmm_mfma_rate on the bytes of the uint8 device tensor `codes`; returns (sink tensor, operations launched)."""
    L = lib()
    assert codes.dtype == torch.uint8 and codes.is_contiguous() and codes.is_cuda
    if workgroups is None:
        workgroups = torch.cuda.get_device_properties(codes.device).multi_processor_count
    if sink is None:
        sink = torch.empty(workgroups * 256, dtype=torch.float32, device=codes.device)
    assert sink.numel() >= workgroups * 256 and sink.dtype == torch.float32
    flops = ctypes.c_double(0.0)
    _check(L.qmm_mfma_rate(fmt_a, fmt_b, codes.data_ptr(), codes.numel(), int(rounds), int(workgroups), sink.data_ptr(),
                           ctypes.byref(flops), _stream()), "qmm_mfma_rate")
    return sink, flops.value


def hbm_rate(src, dst=None, workgroups=1024, sink=None):
    """qmm_hbm_rate over the bytes of the contiguous device tensor src (copied to dst when given); returns the sink."""
    L = lib()
    assert src.is_contiguous() and src.is_cuda and (dst is None or (dst.is_contiguous() and dst.numel() * dst.element_size() == src.numel() * src.element_size()))
    if sink is None:
        sink = torch.empty(workgroups * 256, dtype=torch.int32, device=src.device)
    _check(L.qmm_hbm_rate(src.data_ptr(), dst.data_ptr() if dst is not None else None, src.numel() * src.element_size(),
                          int(workgroups), sink.data_ptr(), _stream()), "qmm_hbm_rate")
    return sink


METRIC_FIELDS = ("S_ee", "S_rr", "S_ae", "S_ar", "M_e", "M_r", "RE_sum", "RE_max", "RE_cnt",
                 "BE_sum", "BE_max", "BE_cnt", "n", "nan_cnt", "rsv0", "rsv1")
