"""The device's FP8 accumulators against the written-down arithmetic of tests/fp8_mfma_model.py, bit for bit, through
every kernel the FP8 product can take (Methodology, third implementation bullet: the 8-bit product held in the wider
accumulator of the multiply-accumulate unit):
  * kernels that return accumulators (LDS-tiled, both tile sizes; split-K; register-direct): acc == model;
  * kernels that only write y (short contractions on resident workgroups, the streaming kernel): y == the oracle's
    descale of the model's accumulators, binary32 and bfloat16, step sizes per tensor / channel / head.
Codes: quantized from the distribution families of the paper's tensors (all four format pairs) -- equality required
everywhere -- and uniformly random E4M3 codes on the tile shapes (equal as well).  Codes drawn uniformly over a
format's whole exponent range (34 binades of products for E4M3, 60 for E5M2 inside one dot product: nothing a scaled
tensor produces) are the one case where the model is known to be incomplete: about one dot product in a million
differs in the last bit (a step in which the accumulator exceeds the step's products by 2^8..2^13 and the aligned
products end in exactly half a grid step); there the tests allow a 2e-5 fraction of accumulators to differ by at
most 2 ulps (fp8_mfma_model.nearly_equal).  The exact sums of the oracle bound both (tests/test_fp8_mfma_model.py).
"""
import ctypes

import numpy as np
import pytest
import torch

import fp8_mfma_model as model
from oracle import oracle as O
from paper_2408_02897_amd import qmm, workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
PAIRS = [(qmm.E4M3, qmm.E4M3), (qmm.E5M2, qmm.E4M3), (qmm.E4M3, qmm.E5M2), (qmm.E5M2, qmm.E5M2)]


def finite_codes(fmt, shape, seed):
    rng = np.random.default_rng(seed)
    c = np.arange(256, dtype=np.uint8)
    c = c[np.isfinite(O.decode(fmt, c))]
    return c[rng.integers(0, c.size, shape)]


def quantized_codes(x, fmt, groups=1):
    """scale + quantize on the device (step size per batch group), codes back as numpy."""
    xd = x.to(DEV)
    d = qmm.scale(xd, 1, fmt, False, groups)
    return qmm.quantize(xd, 1, fmt, d, False, groups).cpu().numpy()


def device(a, fa, b, fb, da=None, db=None, a_pc=False, b_pc=False, a_groups=1, b_groups=1, out=torch.float32, want_acc=True):
    ta, tb = torch.from_numpy(a).to(DEV), torch.from_numpy(b).to(DEV)
    one = torch.ones(1, device=DEV)
    tda = one if da is None else torch.from_numpy(da).to(DEV)
    tdb = one if db is None else torch.from_numpy(db).to(DEV)
    oa = qmm.operand(ta, fa, tda, a_pc, a_groups); ob = qmm.operand(tb, fb, tdb, b_pc, b_groups)
    r = qmm.gemm((ta, oa), (tb, ob), out, want_acc=want_acc)
    return (r[0].float().cpu().numpy(), r[1].cpu().numpy()) if want_acc else r.float().cpu().numpy()


def model_acc(a, fa, b, fb, matrices=None, rows=None, splits=1):
    out = {}
    for m in (range(a.shape[0]) if matrices is None else matrices):
        am = a[m] if rows is None else a[m][rows]
        out[m] = model.accumulate(fa, am, fb, b[m]) if splits == 1 else model.accumulate_split(fa, am, fb, b[m], splits)
    return out


def assert_same_bits(got, want, what=""):
    bad = np.argwhere(got.view(np.uint32) != want.view(np.uint32))
    assert bad.shape[0] == 0, f"{what}: {bad.shape[0]} of {got.size} differ, first at {bad[0]}: {got[tuple(bad[0])]!r} vs {want[tuple(bad[0])]!r}"


TILE_SHAPES = [(1, 16, 16, 16), (1, 128, 128, 128), (1, 200, 136, 400), (1, 300, 272, 144), (3, 130, 80, 64),
               (1, 256, 768, 1040), (2, 257, 512, 272), (1, 64, 1000, 48)]


@pytest.mark.parametrize("shape", TILE_SHAPES)
def test_uniform_e4m3_codes_equal_the_model(shape):
    bt, M, N, K = shape
    a, b = finite_codes(O.E4M3, (bt, M, K), 31), finite_codes(O.E4M3, (bt, N, K), 32)
    _, acc = device(a, qmm.E4M3, b, qmm.E4M3)
    want = model_acc(a, O.E4M3, b, O.E4M3)
    for m in range(bt):
        assert_same_bits(acc[m], want[m], f"matrix {m}")


@pytest.mark.parametrize("fa,fb", PAIRS)
@pytest.mark.parametrize("kind", ["normal", "t4", "lognormal"])
def test_paper_shaped_operands_equal_the_model(fa, fb, kind):
    """A quantized from N(0,1), Student-t(4) or sign * exp(N(-8, 2^2)) (the gradient family), B from N(0, 0.02^2), by
    the library's own scale and quantize; 2 matrices of 320 x 272 x 1040 (ragged tiles, ragged last slab)."""
    bt, M, N, K = 2, 320, 272, 1040
    x = {"normal": W.normal((bt, M, K), 1.0, 41), "t4": W.student_t((bt, M, K), 4, 42),
         "lognormal": W.lognormal_signed((bt, M, K), -8.0, 2.0, 43)}[kind]
    w = W.normal((bt, N, K), 0.02, 44)
    a, b = quantized_codes(x, fa), quantized_codes(w, fb)
    _, acc = device(a, fa, b, fb)
    want = model_acc(a, fa, b, fb)
    exact, sabs = O.gemm_codes(a, fa, b, fb)
    for m in range(bt):
        assert_same_bits(acc[m], want[m], f"matrix {m}")
    err = np.abs(acc.astype(np.float64) - exact)
    print(f"{kind} {fa}x{fb}: max |acc - exact| / S = {np.max(err / sabs):.2e}")
    assert np.all(err <= {"normal": 1e-5, "t4": 5e-5, "lognormal": 4e-4}[kind] * sabs)


@pytest.mark.parametrize("fa,fb", PAIRS[1:])
def test_codes_over_the_whole_e5m2_range_nearly_equal_the_model(fa, fb):
    bt, M, N, K = 1, 256, 256, 512
    a, b = finite_codes(fa, (bt, M, K), 51), finite_codes(fb, (bt, N, K), 52)
    _, acc = device(a, fa, b, fb)
    want = model_acc(a, fa, b, fb)[0]
    assert model.nearly_equal(acc[0], want), np.count_nonzero(model.ulp_distance(acc[0], want))
    exact, sabs = O.gemm_codes(a, fa, b, fb)
    assert np.all(np.abs(acc.astype(np.float64) - exact)[0] <= model.error_bound(fa, a[0], fb, b[0], sabs[0]))


@pytest.mark.parametrize("shape", [(1, 64, 96, 4096), (2, 100, 72, 2064), (1, 300, 272, 2048)])
@pytest.mark.parametrize("fa,fb", PAIRS[:2])
def test_split_contractions_equal_the_model(shape, fa, fb):
    """Small outputs with a long K: ranges of whole slabs summed from zero, partial sums added in ascending order."""
    bt, M, N, K = shape
    x, w = W.student_t((bt, M, K), 4, 61), W.normal((bt, N, K), 0.02, 62)
    a, b = quantized_codes(x, fa), quantized_codes(w, fb)
    ta, tb = torch.from_numpy(a).to(DEV), torch.from_numpy(b).to(DEV)
    one = torch.ones(1, device=DEV)
    oa, ob = qmm.operand(ta, fa, one), qmm.operand(tb, fb, one)
    ws = qmm.lib().qmm_gemm_workspace_size(ctypes.byref(oa), ctypes.byref(ob), bt, M, N, K)
    assert ws > 0 and ws % (bt * M * N * 4) == 0, "this shape is meant to take the split path"
    splits = ws // (bt * M * N * 4)
    _, acc = device(a, fa, b, fb)
    want = model_acc(a, fa, b, fb, splits=splits)
    for m in range(bt):
        assert_same_bits(acc[m], want[m], f"matrix {m}, {splits} ranges")


@pytest.mark.parametrize("shape", [(36, 250, 250, 64), (66, 500, 40, 144), (66, 40, 500, 144), (40, 512, 64, 128)])
def test_register_direct_kernel_equals_the_model(shape):
    bt, M, N, K = shape
    x, w = W.normal((bt, M, K), 1.0, 71), W.normal((bt, N, K), 1.0, 72)
    a, b = quantized_codes(x, qmm.E4M3), quantized_codes(w, qmm.E4M3)
    _, acc = device(a, qmm.E4M3, b, qmm.E4M3)
    pick = [0, bt // 2, bt - 1]
    want = model_acc(a, O.E4M3, b, O.E4M3, matrices=pick)
    for m in pick:
        assert_same_bits(acc[m], want[m], f"matrix {m}")


# ------------------------------------------------------------------ kernels that write y only
# one slab of K at most, whole 256 x 256 tiles, at least 512 of them: the resident-workgroup kernel of the attention scores
SHORTK_SHAPES = [(128, 512, 512, 64), (70, 1024, 512, 48), (64, 768, 768, 128)]


def _y_only_case(shape, fa, fb, gran, out_dtype, data, pick, rows=None):
    bt, M, N, K = shape
    heads = 8 if bt % 8 == 0 else 1
    if data == "uniform":
        a, b = finite_codes(fa, (bt, M, K), 81), finite_codes(fb, (bt, N, K), 82)
    else:
        a = quantized_codes(W.normal((bt, M, K), 1.0, 83), fa, heads)
        b = quantized_codes(W.normal((bt, N, K), 1.0, 84), fb, heads)
    rng = np.random.default_rng(bt + M)
    a_pc = b_pc = gran == "channel"
    ga = gb = heads if gran == "head" else 1
    da = rng.uniform(1e-3, 1e-2, ga * (M if a_pc else 1)).astype(np.float32)
    db = rng.uniform(1e-3, 1e-2, gb * (N if b_pc else 1)).astype(np.float32)
    y = device(a, fa, b, fb, da, db, a_pc, b_pc, ga, gb, out_dtype, want_acc=False)
    want_acc = model_acc(a, fa, b, fb, matrices=pick, rows=rows)
    for m in pick:
        # the oracle's descale wants the whole batch's group indexing: give it matrix m alone with its group's step sizes
        g = m % ga
        dam = da[g * (M if a_pc else 1):(g + 1) * (M if a_pc else 1)]
        dbm = db[(m % gb) * (N if b_pc else 1):((m % gb) + 1) * (N if b_pc else 1)]
        if rows is not None and a_pc:
            dam = dam[rows]
        want_y = O.dequant(want_acc[m][None].astype(np.float64), dam, dbm, a_pc, 1, b_pc, 1, out_dtype == torch.bfloat16)[0]
        got = y[m] if rows is None else y[m][rows]
        assert_same_bits(got, want_y, f"matrix {m}")


@pytest.mark.parametrize("shape", SHORTK_SHAPES)
@pytest.mark.parametrize("fa,fb", PAIRS)
@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_short_contraction_kernel_y_equals_descaled_model(shape, fa, fb, out_dtype):
    """Attention-score shapes, output in y alone (the path config 5's Q K^T takes at full batch): three whole matrices
    per case (first, middle, last: the first and last tiles a resident workgroup walks), quantized normal data."""
    bt = shape[0]
    _y_only_case(shape, fa, fb, "tensor", out_dtype, "quantized", [0, bt // 2, bt - 1])


@pytest.mark.parametrize("gran", ["channel", "head"])
@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_short_contraction_kernel_step_sizes_per_channel_and_head(gran, out_dtype):
    _y_only_case(SHORTK_SHAPES[0], qmm.E4M3, qmm.E4M3, gran, out_dtype, "uniform", [0, 63, 127])
    _y_only_case(SHORTK_SHAPES[2], qmm.E5M2, qmm.E4M3, gran, out_dtype, "quantized", [1, 62])


def test_short_contraction_kernel_exact_cases():
    """Powers of two and one-hot operands through the y-only kernel (step sizes 1, binary32 out): exact sums."""
    bt, M, N, K = 128, 512, 512, 64
    rng = np.random.default_rng(9)
    ea = rng.integers(5, 9, (bt, M, K)); eb = rng.integers(5, 9, (bt, N, K))
    a = ((ea << 3) | (rng.integers(0, 2, ea.shape) << 7)).astype(np.uint8)
    b = ((eb << 3) | (rng.integers(0, 2, eb.shape) << 7)).astype(np.uint8)
    y = device(a, qmm.E4M3, b, qmm.E4M3, want_acc=False)
    for m in (0, 77, 127):
        want = O.gemm_codes(a[m:m + 1], O.E4M3, b[m:m + 1], O.E4M3, want_sabs=False)[0]
        assert np.array_equal(y[m].astype(np.float64), want)
    a = np.zeros((bt, M, K), np.uint8); b = np.zeros((bt, N, K), np.uint8)
    hot = [(0, 0, 0, 0), (127, 511, 511, 63), (64, 255, 256, 31), (5, 300, 17, 32)]
    for (m, i, j, k) in hot:
        a[m, i, k] = 0x45; b[m, j, k] = 0xC2                          # E5M2 5.0 and -3.0
    y = device(a, qmm.E5M2, b, qmm.E5M2, want_acc=False)
    assert np.count_nonzero(y) == len(hot)
    for (m, i, j, k) in hot:
        assert y[m, i, j] == -15.0


@pytest.mark.parametrize("fa,fb", PAIRS)
@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_streaming_kernel_y_equals_descaled_model(fa, fb, out_dtype):
    """More whole tiles than CUs, several slabs, y alone: rows around tile borders and random rows of every matrix."""
    shape = (2, 2560, 3584, 640)             # 280 tiles for 256 workgroups, five slabs
    M = shape[1]
    rows = np.unique(np.concatenate([[0, 1, 255, 256, 257, M - 257, M - 256, M - 1],
                                     np.random.default_rng(5).choice(M, 24, replace=False)]))
    _y_only_case(shape, fa, fb, "tensor", out_dtype, "quantized", [0, 1], rows=rows)
