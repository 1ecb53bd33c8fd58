"""numpy-facing wrapper of the CPU oracle (oracle/qmm_oracle.c).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this module;
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg do.  It
shares no code with the HIP library: its own C file, its own enums, its own
build step.  All arrays are host numpy arrays; bfloat16 inputs are widened to
float32 by the caller (exact).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qmm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

INT8, E4M3, E5M2 = 0, 1, 2
RTNE, STOCHASTIC = 0, 1
FORMATS = {"int8": INT8, "e4m3": E4M3, "e5m2": E5M2}

METRIC_FIELDS = ("S_ee", "S_rr", "S_ae", "S_ar", "M_e", "M_r", "RE_sum", "RE_max", "RE_cnt",
                 "BE_sum", "BE_max", "BE_cnt", "n", "nan_cnt", "rsv0", "rsv1")


def build(force=False):
    """Compile the oracle with gcc (plain C, OpenMP only over independent output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
               "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i64, u64, i32, u32 = ctypes.c_int64, ctypes.c_uint64, ctypes.c_int, ctypes.c_uint32
        vp, f32, f64 = ctypes.c_void_p, ctypes.c_float, ctypes.c_double
        L.orc_num_threads.restype = i32; L.orc_num_threads.argtypes = []
        L.orc_qmax.restype = f64; L.orc_qmax.argtypes = [i32]
        L.orc_fp8_value.restype = f64; L.orc_fp8_value.argtypes = [i32, ctypes.c_uint]
        L.orc_code_value.restype = f64; L.orc_code_value.argtypes = [i32, ctypes.c_uint]
        L.orc_encode_rtne.restype = ctypes.c_uint8; L.orc_encode_rtne.argtypes = [i32, f32]
        L.orc_encode_sr.restype = ctypes.c_uint8; L.orc_encode_sr.argtypes = [i32, f32, u32]
        L.orc_philox4x32_10.restype = None; L.orc_philox4x32_10.argtypes = [vp, vp, vp]
        L.orc_sr_bits.restype = u32; L.orc_sr_bits.argtypes = [u64, u64]
        L.orc_bf16_round.restype = f32; L.orc_bf16_round.argtypes = [f32]
        L.orc_scale.restype = None
        L.orc_scale.argtypes = [vp, i64, i64, i64, i32, i32, i32, i64, i64, vp]
        L.orc_quantize.restype = None
        L.orc_quantize.argtypes = [vp, i64, i64, i64, i32, i32, i32, i64, i64, vp, i32, u64, u64, vp]
        L.orc_gemm_codes.restype = None
        L.orc_gemm_codes.argtypes = [vp, i32, vp, i32, i64, i64, i64, i64, vp, vp]
        L.orc_gemm_codes_rows.restype = None
        L.orc_gemm_codes_rows.argtypes = [vp, i32, vp, i32, i64, i64, vp, i64, vp, vp]
        L.orc_gemm_int8.restype = i64
        L.orc_gemm_int8.argtypes = [vp, vp, i64, i64, i64, i64, vp]
        L.orc_dequant.restype = None
        L.orc_dequant.argtypes = [vp, i64, i64, i64, vp, i32, i64, i64, vp, i32, i64, i64, i32, vp]
        L.orc_ref_gemm.restype = None
        L.orc_ref_gemm.argtypes = [vp, vp, i64, i64, i64, i64, vp]
        L.orc_metric.restype = None
        L.orc_metric.argtypes = [vp, vp, vp, i64, vp]
        L.orc_dequantize_codes.restype = None
        L.orc_dequantize_codes.argtypes = [vp, i64, i64, i64, i32, i32, i64, i64, vp, vp]
        L.orc_moments.restype = None
        L.orc_moments.argtypes = [vp, i64, vp]
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f32_3d(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.ndim == 2:
        x = x[None]
    assert x.ndim == 3
    return x


def num_threads():
    return lib().orc_num_threads()


def qmax(fmt):
    return lib().orc_qmax(fmt)


def fp8_value(fmt, code):
    return lib().orc_fp8_value(fmt, int(code))


def code_value(fmt, code):
    return lib().orc_code_value(fmt, int(code))


def decode(fmt, codes):
    """Values (float64) of an array of uint8 codes."""
    table = np.array([code_value(fmt, c) for c in range(256)], dtype=np.float64)
    return table[np.asarray(codes, dtype=np.uint8)]


def encode_rtne(fmt, t):
    """Element-wise RTNE encode of float32 values (scalar calls; for tests)."""
    t = np.asarray(t, dtype=np.float32)
    out = np.empty(t.shape, dtype=np.uint8)
    f = lib().orc_encode_rtne
    flat_in, flat_out = t.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = f(fmt, ctypes.c_float(flat_in[i]))
    return out


def encode_sr(fmt, t, u24):
    return lib().orc_encode_sr(fmt, ctypes.c_float(np.float32(t)), int(u24))


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32); k = np.asarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def sr_bits(seed, g):
    return lib().orc_sr_bits(int(seed), int(g))


def bf16_round(v):
    v = np.asarray(v, dtype=np.float32)
    f = lib().orc_bf16_round
    return np.array([f(ctypes.c_float(a)) for a in v.reshape(-1)], dtype=np.float32).reshape(v.shape)


def n_scales(shape3, contract_axis, per_channel, batch_groups):
    _, rows, cols = shape3
    c = (rows if contract_axis == 1 else cols) if per_channel else 1
    return batch_groups * c


def scale(x, contract_axis, fmt, per_channel=False, batch_groups=1, batch_inner=1):
    x = _f32_3d(x)
    b, r, c = x.shape
    delta = np.empty(n_scales(x.shape, contract_axis, per_channel, batch_groups), dtype=np.float32)
    lib().orc_scale(_p(x), b, r, c, contract_axis, fmt, int(per_channel), batch_groups, batch_inner, _p(delta))
    return delta


def quantize(x, contract_axis, fmt, delta, per_channel=False, batch_groups=1, mode=RTNE, seed=0, offset=0, batch_inner=1):
    x = _f32_3d(x)
    b, r, c = x.shape
    delta = np.ascontiguousarray(delta, dtype=np.float32)
    assert delta.size == n_scales(x.shape, contract_axis, per_channel, batch_groups)
    nc, kc = (r, c) if contract_axis == 1 else (c, r)
    codes = np.empty((b, nc, kc), dtype=np.uint8)
    lib().orc_quantize(_p(x), b, r, c, contract_axis, fmt, int(per_channel), batch_groups, batch_inner, _p(delta),
                       mode, int(seed), int(offset), _p(codes))
    return codes


def gemm_codes(a, a_fmt, b, b_fmt, want_sabs=True):
    a = np.ascontiguousarray(a, dtype=np.uint8); b = np.ascontiguousarray(b, dtype=np.uint8)
    if a.ndim == 2:
        a = a[None]; b = b[None]
    bt, m, k = a.shape
    n = b.shape[1]
    assert b.shape == (bt, n, k)
    acc = np.empty((bt, m, n), dtype=np.float64)
    sabs = np.empty((bt, m, n), dtype=np.float64) if want_sabs else None
    lib().orc_gemm_codes(_p(a), a_fmt, _p(b), b_fmt, bt, m, n, k, _p(acc), _p(sabs) if want_sabs else None)
    return (acc, sabs) if want_sabs else acc


def gemm_codes_rows(a, a_fmt, b, b_fmt, rows):
    """Rows `rows` of a single (un-batched) product: returns (acc, sabs) of shape [len(rows), N]."""
    a = np.ascontiguousarray(a, dtype=np.uint8); b = np.ascontiguousarray(b, dtype=np.uint8)
    assert a.ndim == 2 and b.ndim == 2 and a.shape[1] == b.shape[1]
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    n, k = b.shape
    acc = np.empty((rows.size, n), dtype=np.float64); sabs = np.empty_like(acc)
    lib().orc_gemm_codes_rows(_p(a), a_fmt, _p(b), b_fmt, n, k, _p(rows), rows.size, _p(acc), _p(sabs))
    return acc, sabs


def gemm_int8(a, b):
    a = np.ascontiguousarray(a).view(np.int8); b = np.ascontiguousarray(b).view(np.int8)
    if a.ndim == 2:
        a = a[None]; b = b[None]
    bt, m, k = a.shape
    n = b.shape[1]
    acc = np.empty((bt, m, n), dtype=np.int64)
    bad = lib().orc_gemm_int8(_p(a), _p(b), bt, m, n, k, _p(acc))
    assert bad == 0, "accumulator does not fit 32 bits"
    return acc


def dequant(acc, dl, dr, l_per_channel=False, l_groups=1, r_per_channel=False, r_groups=1, out_bf16=False,
            l_inner=1, r_inner=1):
    acc = np.ascontiguousarray(acc, dtype=np.float64)
    if acc.ndim == 2:
        acc = acc[None]
    bt, m, n = acc.shape
    dl = np.ascontiguousarray(dl, dtype=np.float32); dr = np.ascontiguousarray(dr, dtype=np.float32)
    assert dl.size == l_groups * (m if l_per_channel else 1)
    assert dr.size == r_groups * (n if r_per_channel else 1)
    y = np.empty((bt, m, n), dtype=np.float32)
    lib().orc_dequant(_p(acc), bt, m, n, _p(dl), int(l_per_channel), l_groups, l_inner, _p(dr), int(r_per_channel),
                      r_groups, r_inner, int(out_bf16), _p(y))
    return y


def ref_gemm(x, w):
    x = _f32_3d(x); w = _f32_3d(w)
    bt, m, k = x.shape
    n = w.shape[1]
    assert w.shape == (bt, n, k)
    r = np.empty((bt, m, n), dtype=np.float32)
    lib().orc_ref_gemm(_p(x), _p(w), bt, m, n, k, _p(r))
    return r


def metric(y, r, d=None):
    y = np.ascontiguousarray(y, dtype=np.float32).reshape(-1)
    r = np.ascontiguousarray(r, dtype=np.float32).reshape(-1)
    assert y.size == r.size
    if d is not None:
        d = np.ascontiguousarray(d, dtype=np.float32).reshape(-1)
        assert d.size == y.size
    out = np.empty(16, dtype=np.float64)
    lib().orc_metric(_p(y), _p(r), _p(d) if d is not None else None, y.size, _p(out))
    return out


def dequantize_codes(codes, fmt, delta, per_channel=False, batch_groups=1, batch_inner=1):
    """Values (float32) of codes [batch, nc, kc] (or [nc, kc]) as laid out by quantize: code value times step size."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    shape = codes.shape
    if codes.ndim == 2:
        codes = codes[None]
    b, nc, kc = codes.shape
    delta = np.ascontiguousarray(delta, dtype=np.float32)
    assert delta.size == batch_groups * (nc if per_channel else 1)
    out = np.empty(codes.shape, dtype=np.float32)
    lib().orc_dequantize_codes(_p(codes), b, nc, kc, fmt, int(per_channel), batch_groups, batch_inner, _p(delta), _p(out))
    return out.reshape(shape)


MOMENT_FIELDS = ("n", "mean", "m2", "m3", "m4", "absmax", "nan_cnt", "rsv")


def moments(x):
    """Population moments about the mean of all elements of x (two passes, binary64): 8 doubles, MOMENT_FIELDS."""
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    out = np.empty(8, dtype=np.float64)
    lib().orc_moments(_p(x), x.size, _p(out))
    return out


def metric_dict(out):
    d = dict(zip(METRIC_FIELDS, [float(v) for v in out]))
    d["NSR"] = d["S_ee"] / d["S_rr"] if d["S_rr"] > 0 else float("nan")
    return d


def quantized_matmul(x, w, fmt_x, fmt_w, per_channel=False, out_bf16=False):
    """Whole path on un-batched operands x [M,K], w [N,K] (K contracting): scale, quantize,
    product, descale.  Returns (y, acc, sabs, dx, dw, cx, cw)."""
    dx = scale(x, 1, fmt_x, per_channel); dw = scale(w, 1, fmt_w, per_channel)
    cx = quantize(x, 1, fmt_x, dx, per_channel); cw = quantize(w, 1, fmt_w, dw, per_channel)
    acc, sabs = gemm_codes(cx, fmt_x, cw, fmt_w)
    y = dequant(acc, dx, dw, per_channel, 1, per_channel, 1, out_bf16)
    return y, acc, sabs, dx, dw, cx, cw


def encode_bulk(fmt, t, mode=RTNE, seed=0, offset=0):
    """Encode an array of float32 values t directly (step size 1, so x * (1/1) = x exactly)."""
    t = np.ascontiguousarray(t, dtype=np.float32)
    one = np.ones(1, dtype=np.float32)
    return quantize(t.reshape(1, 1, -1), 1, fmt, one, mode=mode, seed=seed, offset=offset).reshape(t.shape)
