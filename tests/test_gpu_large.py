"""Sizes past 2^31 elements (element and byte offsets that do not fit 32 bits): the hot path at sizes no oracle run
finishes on, checked on slices the oracle computes one by one (quantize is element-wise once the step size is
fixed; a GEMM row depends on one row of A only) and on closed forms that hold at any size (metric sums of constant
arrays with planted errors)."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2408_02897_amd import qmm

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
COLS = 4096
ROWS = (1 << 19) + 3                      # ROWS * COLS = 2^31 + 12288


def np32(t):
    return t.detach().float().cpu().numpy()


def big_operand():
    g = torch.Generator(device="cpu"); g.manual_seed(2024)
    block = (torch.randn(1 << 20, generator=g) * 3.0).to(torch.bfloat16).to(DEV)
    reps = (ROWS * COLS + block.numel() - 1) // block.numel()
    x = block.repeat(reps)[: ROWS * COLS].reshape(1, ROWS, COLS)
    x[0, ROWS - 2, 17] = 1000.0           # the largest magnitude sits past element 2^31
    x[0, ROWS - 1, COLS - 1] = -7.25      # and the very last element is not part of the repeated block
    return x


@pytest.mark.parametrize("fmt", [qmm.E4M3, qmm.INT8])
def test_scale_and_quantize_past_2_31_elements(fmt):
    x = big_operand()
    qmax = {qmm.E4M3: 448.0, qmm.INT8: 127.0}[fmt]
    delta = qmm.scale(x, 1, fmt)
    assert delta.cpu().numpy()[0] == np.float32(np.float32(1000.0) / np.float32(qmax))
    codes = qmm.quantize(x, 1, fmt, delta)
    assert codes.shape == (1, ROWS, COLS)
    d = delta.cpu().numpy()
    for r0, r1 in ((0, 64), ((1 << 19) - 32, (1 << 19) + 3), (ROWS - 64, ROWS)):      # start, across 2^31, end
        want = O.quantize(np32(x[:, r0:r1]), 1, fmt, d)
        assert np.array_equal(codes[:, r0:r1].cpu().numpy(), want)
    # one step size per row: the rows past 2^31 elements get their own
    dr = qmm.scale(x, 1, fmt, per_channel=True)
    rows = np.array([0, 1, (1 << 19) - 1, 1 << 19, ROWS - 2, ROWS - 1])
    trows = torch.from_numpy(rows).to(DEV)
    want_dr = O.scale(np32(x[:, trows]), 1, fmt, True)
    assert np.array_equal(dr.cpu().numpy().reshape(-1)[rows], want_dr.reshape(-1))
    cr = qmm.quantize(x, 1, fmt, dr, per_channel=True)
    want_cr = O.quantize(np32(x[:, trows]), 1, fmt, want_dr, True)
    assert np.array_equal(cr[:, trows].cpu().numpy(), want_cr)
    del codes, cr, x
    torch.cuda.empty_cache()


def test_metric_past_2_31_elements():
    n = (1 << 31) + 12288 + 3
    r = torch.full((n,), 2.0, dtype=torch.float32, device=DEV)
    y = torch.full((n,), 2.0, dtype=torch.bfloat16, device=DEV)
    planted = {5: 3.0, (1 << 31) + 7: 1.0, n - 1: 2.5, n - 4: 4.0}       # y values; errors 1, -1, 0.5, 2
    for i, v in planted.items():
        y[i] = v
    m = qmm.metric(y, r).cpu().numpy()
    errs = np.array([abs(v - 2.0) for v in planted.values()])
    assert m[0] == np.sum(errs ** 2) and m[1] == 4.0 * n                  # S_ee, S_rr: exact in binary64
    assert m[2] == np.sum(errs) and m[3] == 2.0 * n                       # S_ae, S_ar
    assert m[4] == 2.0 and m[5] == 2.0                                    # maxima
    assert m[6] == np.sum(errs / 2.0) and m[7] == 1.0 and m[8] == n       # Eq. 2: sum, max, count
    assert m[12] == n and m[13] == 0
    del y, r
    torch.cuda.empty_cache()


@pytest.mark.parametrize("K", [32, 272])
def test_gemm_output_past_2_31_elements(K):
    """65536 x 33024 outputs (2^31 + 2^24 of them): rows sampled against the oracle.  K = 32 takes the kernel for short
    contractions, K = 272 the general one."""
    M, N = 65536, 33024
    rng = np.random.default_rng(11)
    a = rng.integers(-127, 128, (1, M, K), dtype=np.int8).view(np.uint8)
    b = rng.integers(-127, 128, (1, N, K), dtype=np.int8).view(np.uint8)
    da = np.array([0.015625], dtype=np.float32); db = np.array([0.03125], dtype=np.float32)
    ta, tb = torch.from_numpy(a).to(DEV), torch.from_numpy(b).to(DEV)
    oa = qmm.operand(ta, qmm.INT8, torch.from_numpy(da).to(DEV)); ob = qmm.operand(tb, qmm.INT8, torch.from_numpy(db).to(DEV))
    y = qmm.gemm((ta, oa), (tb, ob), torch.bfloat16)
    assert y.shape == (1, M, N)
    rows = np.array([0, 1, 255, 256, 32767, 32768, 65022, 65023, 65024, 65279, 65280, M - 2, M - 1])   # row 65024 starts past 2^31
    acc = O.gemm_int8(a[:, rows], b)
    want = O.dequant(acc.astype(np.float64), da, db, False, 1, False, 1, True)
    got = y[:, torch.from_numpy(rows).to(DEV)].float().cpu().numpy()
    assert np.array_equal(got.view(np.uint32), want.astype(np.float32).view(np.uint32))
    del y
    torch.cuda.empty_cache()


def test_moments_and_dequantize_past_2_31_elements():
    n = (1 << 31) + 12288 + 5
    x = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    a = 6.0
    x[3] = a; x[n - 2] = -a                      # symmetric about 0: odd moments vanish, even ones are 2 a^k / n
    m = qmm.moments(x).cpu().numpy()
    assert m[0] == n and m[5] == a and m[6] == 0
    assert abs(m[1]) <= 1e-18
    assert abs(m[2] - 2 * a ** 2 / n) <= 1e-12 * (2 * a ** 2 / n)
    assert abs(m[3]) <= 1e-12 * (2 * a ** 3 / n)
    assert abs(m[4] - 2 * a ** 4 / n) <= 1e-12 * (2 * a ** 4 / n)
    del x
    torch.cuda.empty_cache()
    rows = (1 << 19) + 3
    g = torch.Generator(device="cpu"); g.manual_seed(7)
    block = torch.randint(0, 256, (1 << 20,), generator=g, dtype=torch.int32).to(torch.uint8)
    block[block == 0x7F] = 0x31; block[block == 0xFF] = 0x31         # no E4M3 NaN codes
    block = block.to(DEV)
    codes = block.repeat((rows * COLS + block.numel() - 1) // block.numel())[: rows * COLS].reshape(1, rows, COLS)
    delta = torch.tensor([0.0078125], dtype=torch.float32, device=DEV)
    v = qmm.dequantize(codes, qmm.E4M3, delta, out_dtype=torch.bfloat16)
    for r0, r1 in ((0, 16), ((1 << 19) - 8, (1 << 19) + 3), (rows - 16, rows)):
        want = O.dequantize_codes(codes[:, r0:r1].cpu().numpy(), O.E4M3, delta.cpu().numpy())
        got = v[:, r0:r1].float().cpu().numpy()
        want_bf16 = torch.from_numpy(want).to(torch.bfloat16).float().numpy()
        assert np.array_equal(got.view(np.uint32), want_bf16.view(np.uint32))
    del v, codes
    torch.cuda.empty_cache()
