"""GPU parity on the paper-shaped workloads (BERT-base / BERT-large GEMM shapes, attention batched GEMMs) with
the distributions the paper reports for BERT tensors (Student-t activations, normal weights, log-normal
upstream gradients).  Step sizes and codes are compared in full (bit-exact); products are compared on seeded
sample rows the oracle can afford, in the launch configuration the benchmark times (bfloat16 output, 256 x 256
tiles), and the metric pass on the full-size outputs via sums that must agree with the oracle's on the same data.

FP8 accumulators: always within the bound the matrix instruction's arithmetic gives (hw_fp8_bound, see
test_gpu_parity.py).  In units of S = sum_k |a||b| the observed error is ~1e-6 on normal data, ~1.3e-5 on
Student-t(4) activations (a few large products per group of 8 truncate the small ones) and larger on log-normal
gradients; the tests with heavy-tailed inputs assert 5e-5 * S, the normal-data test 1e-5 * S.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2408_02897_amd import qmm, workloads as W
from test_gpu_parity import hw_fp8_bound, np32

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _check_rows(a_bf16, b_bf16, fa, fb, per_channel, rows, out_dtype=torch.bfloat16, tight=None):
    """Full path on device for A [M,K], B [N,K]; oracle on the sample `rows` of A (scale/quantize in full)."""
    ad, bd = a_bf16.to(DEV), b_bf16.to(DEV)
    (ca, oa), da = qmm.quantized_operand(ad, 1, fa, per_channel)
    (cb, ob), db = qmm.quantized_operand(bd, 1, fb, per_channel)
    an, bn = np32(a_bf16), np32(b_bf16)
    da_o = O.scale(an, 1, fa, per_channel); db_o = O.scale(bn, 1, fb, per_channel)
    assert np.array_equal(da.cpu().numpy(), da_o) and np.array_equal(db.cpu().numpy(), db_o)
    cb_o = O.quantize(bn, 1, fb, db_o, per_channel)
    assert np.array_equal(cb.cpu().numpy(), cb_o)
    ca_dev = ca.cpu().numpy()
    ca_rows_o = O.quantize(an[rows], 1, fa, da_o[rows] if per_channel else da_o, per_channel)
    assert np.array_equal(ca_dev[0][rows], ca_rows_o[0])
    y, acc = qmm.gemm((ca, oa), (cb, ob), out_dtype, want_acc=True)
    acc_o, sabs = O.gemm_codes_rows(ca_dev[0], fa, cb_o[0], fb, rows)
    acc_d = acc.cpu().numpy()[0][rows].astype(np.float64)
    if fa == O.INT8:
        assert np.array_equal(acc_d, acc_o)
    else:
        err = np.abs(acc_d - acc_o)
        bound = hw_fp8_bound(ca_dev[:, rows], fa, cb_o, fb, sabs[None])[0]
        assert np.all(err <= bound), f"err/bound {np.max(err / (bound + 1e-300)):.3f}"
        ratio = float(np.max(err / (sabs + 1e-300)))
        if tight is not None:
            assert ratio <= tight, f"err/S {ratio:.3e}"
    y_o = O.dequant(acc_d, da_o[rows] if per_channel else da_o, db_o, per_channel, 1, per_channel, 1,
                    out_bf16=(out_dtype == torch.bfloat16))
    assert np.array_equal(np32(y)[0][rows].view(np.uint32), y_o[0].view(np.uint32))
    # the call without accumulators out (the benchmark's; large per-tensor shapes take the streaming kernel): same bits
    assert torch.equal(qmm.gemm((ca, oa), (cb, ob), out_dtype), y)
    return y, ad, bd


@pytest.mark.parametrize("name", ["qkv", "attn_out", "ffn1", "ffn2"])
def test_bert_base_forward_e4m3(name):
    """BERT-base layer forward GEMMs (4096 tokens, hidden 768): E4M3 per-tensor, full metric vs oracle on sampled rows."""
    op = {o.name: o for o in W.bert_forward_ops(**W.BERT_BASE)}[name]
    x, w = W.forward_operands(op, 2)
    rows = np.sort(np.random.default_rng(op.N).choice(op.M, 48, replace=False))
    y, xd, wd = _check_rows(x, w, O.E4M3, O.E4M3, False, rows, tight=5e-5)
    r = qmm.reference_gemm(xd.unsqueeze(0), wd.unsqueeze(0))
    r_o = O.ref_gemm(np32(x)[rows], np32(w))
    sab = np.abs(np32(x)[rows]).astype(np.float64) @ np.abs(np32(w)).astype(np.float64).T
    assert np.all(np.abs(r.cpu().numpy()[0][rows] - r_o[0]) <= 1e-5 * sab)
    m = qmm.metric(y, r).cpu().numpy()
    m_o = O.metric(np32(y), r.cpu().numpy())
    assert np.allclose(m, m_o, rtol=1e-10, atol=0)
    nsr = m[0] / m[1]
    assert 1.0e-3 < nsr < 2.0e-3            # two E4M3 operands: about 2 x 7e-4


@pytest.mark.parametrize("name", ["qkv", "ffn2"])
@pytest.mark.parametrize("kind", ["dgrad", "wgrad"])
def test_bert_base_backward_e5m2_gradients(name, kind):
    """dgrad dX = dY . W^T and wgrad dW = X^T . dY with dY in E5M2 (log-normal magnitudes) and the other operand in
    E4M3; the contraction over tokens goes through the transposing quantize path."""
    op = {o.name: o for o in W.bert_forward_ops(**W.BERT_BASE)}[name]
    x, w = W.forward_operands(op, 3)
    dy = W.upstream_gradient(op, 3)
    rng = np.random.default_rng(7)
    if kind == "dgrad":       # A = dY [M, N] contract over N ; B = W^T given as [K, N]: rows K, contract over N
        a, b = dy, w.t().contiguous()            # B[k][n] = W[n][k]
        fa, fb = O.E5M2, O.E4M3
        rows = np.sort(rng.choice(op.M, 32, replace=False))
        _check_rows(a, b, fa, fb, False, rows, out_dtype=torch.float32)
    else:                     # dW[k][n] = sum_t X[t][k] dY[t][n]: both operands contract over their rows
        xd, dyd = x.to(DEV), dy.to(DEV)
        (ca, oa), da = qmm.quantized_operand(xd, 0, qmm.E4M3)
        (cb, ob), db = qmm.quantized_operand(dyd, 0, qmm.E5M2)
        da_o = O.scale(np32(x), 0, O.E4M3); db_o = O.scale(np32(dy), 0, O.E5M2)
        assert np.array_equal(da.cpu().numpy(), da_o) and np.array_equal(db.cpu().numpy(), db_o)
        ca_o = O.quantize(np32(x), 0, O.E4M3, da_o); cb_o = O.quantize(np32(dy), 0, O.E5M2, db_o)
        assert np.array_equal(ca.cpu().numpy(), ca_o) and np.array_equal(cb.cpu().numpy(), cb_o)
        y, acc = qmm.gemm((ca, oa), (cb, ob), torch.float32, want_acc=True)
        rows = np.sort(rng.choice(op.K, 16, replace=False))
        acc_o, sabs = O.gemm_codes_rows(ca_o[0], O.E4M3, cb_o[0], O.E5M2, rows)
        err = np.abs(acc.cpu().numpy()[0][rows] - acc_o)
        bound = hw_fp8_bound(ca_o[:, rows], O.E4M3, cb_o, O.E5M2, sabs[None])[0]
        assert np.all(err <= bound), f"err/bound {np.max(err / (bound + 1e-300)):.3f}"


@pytest.mark.parametrize("fmt", [O.E4M3, O.INT8, O.E5M2])
@pytest.mark.parametrize("per_channel", [False, True])
def test_bert_large_ffn1_full_size_sampled(fmt, per_channel):
    """BERT-large FFN1 (16384 x 4096 x 1024) in the benchmark's launch configuration, sampled rows vs the oracle."""
    op = W.bert_forward_ops(**W.BERT_LARGE)[2]
    x, w = W.forward_operands(op, 4)
    rows = np.sort(np.random.default_rng(11).choice(op.M, 24, replace=False))
    rows[0], rows[-1] = 0, op.M - 1
    y, xd, wd = _check_rows(x, w, fmt, fmt, per_channel, rows, tight=5e-5 if fmt != O.INT8 else None)
    r = qmm.reference_gemm(xd.unsqueeze(0), wd.unsqueeze(0))
    m = qmm.metric(y, r).cpu().numpy()
    # properties that hold at any size
    assert m[12] == op.M * op.N and m[13] == 0
    nsr = m[0] / m[1]
    if fmt == O.INT8 and not per_channel:
        assert nsr > 5e-3                      # heavy-tailed activations: one step size for the tensor is too coarse
    if fmt == O.E4M3:
        assert 1.0e-3 < nsr < 2.0e-3


def test_attention_batched_per_head():
    """QK^T and P.V for 4 examples x 16 heads, seq 512, dim 64 (the same kernels as the 32-example case),
    E4M3 with one step size per head shared by the examples; outlier channels x20."""
    batch, heads, seq, dim = 4, 16, 512, 64
    q, k, v = W.attention_operands(batch, heads, seq, dim)
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    (cq, oq), dq = qmm.quantized_operand(qd, 1, qmm.E4M3, False, heads)
    (ck, ok), dk = qmm.quantized_operand(kd, 1, qmm.E4M3, False, heads)
    dq_o = O.scale(np32(q), 1, O.E4M3, False, heads); dk_o = O.scale(np32(k), 1, O.E4M3, False, heads)
    assert np.array_equal(dq.cpu().numpy(), dq_o) and np.array_equal(dk.cpu().numpy(), dk_o)
    cq_o = O.quantize(np32(q), 1, O.E4M3, dq_o, False, heads); ck_o = O.quantize(np32(k), 1, O.E4M3, dk_o, False, heads)
    assert np.array_equal(cq.cpu().numpy(), cq_o) and np.array_equal(ck.cpu().numpy(), ck_o)
    s, acc = qmm.gemm((cq, oq), (ck, ok), torch.float32, want_acc=True)
    sel = [0, 17, 63]
    acc_o, sabs = O.gemm_codes(cq_o[sel], O.E4M3, ck_o[sel], O.E4M3)
    err = np.abs(acc.cpu().numpy()[sel] - acc_o)
    assert np.all(err <= hw_fp8_bound(cq_o[sel], O.E4M3, ck_o[sel], O.E4M3, sabs))
    s_o = O.dequant(acc.cpu().numpy()[sel].astype(np.float64), dq_o, dk_o, False, heads, False, heads)
    # batch group of entry b is b % heads: check through entries of different heads
    for t, b in enumerate(sel):
        want = (acc.cpu().numpy()[b] * dq_o[b % heads]) * dk_o[b % heads]
        assert np.array_equal(s.cpu().numpy()[b], want.astype(np.float32))
    # P.V: P = softmax of the reference scores (harness), V contracts over the sequence -> transposing quantize
    s_ref = qmm.reference_gemm(qd, kd)
    p = W.softmax_probabilities(s_ref, dim).contiguous()
    assert torch.allclose(p.float().sum(-1), torch.ones(batch * heads, seq, device=DEV), atol=2e-2)
    (cp, op_), dp = qmm.quantized_operand(p, 1, qmm.E4M3, False, heads)
    (cv, ov), dv = qmm.quantized_operand(vd, 0, qmm.E4M3, False, heads)       # V [seq, dim] contracts over rows
    dv_o = O.scale(np32(v), 0, O.E4M3, False, heads)
    cv_o = O.quantize(np32(v), 0, O.E4M3, dv_o, False, heads)
    assert np.array_equal(dv.cpu().numpy(), dv_o) and np.array_equal(cv.cpu().numpy(), cv_o)
    o, acc2 = qmm.gemm((cp, op_), (cv, ov), torch.float32, want_acc=True)
    cp_n = cp.cpu().numpy()
    acc2_o, sabs2 = O.gemm_codes(cp_n[sel], O.E4M3, cv_o[sel], O.E4M3)
    err2 = np.abs(acc2.cpu().numpy()[sel] - acc2_o)
    assert np.all(err2 <= hw_fp8_bound(cp_n[sel], O.E4M3, cv_o[sel], O.E4M3, sabs2))
    o_ref = qmm.reference_gemm(p, vd.transpose(1, 2).contiguous())
    m = qmm.metric(o, o_ref).cpu().numpy()
    assert m[13] == 0 and m[0] / m[1] < 5e-2
