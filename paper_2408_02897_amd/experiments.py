"""The paper's illustrative example (section "Quantized matrix multiplication: An illustrative example", Eq. 3):
element-wise backward error |L R - Q(L, R)| / (|L| |R|) of the quantized product of two 512 x 512 Student-t
matrices with per-vector (per-row / per-column) step sizes, for INT8, E4M3 and E5M2 over a range of degrees of
freedom.  Every step runs in the library's kernels (scale, quantize, GEMM, reference GEMM, metric); this module
only draws the inputs and strings the calls together.

    python -m paper_2408_02897_amd.experiments
"""
import torch

from . import qmm, workloads as W


def backward_error_row(dof, fmt, n=512, device="cuda:0"):
    """One cell of the sweep: returns a dict with max / mean backward error and the noise-to-signal ratio."""
    L, R = W.backward_error_operands(dof, n)
    ld, rd = L.to(device), R.to(device)
    (cl, ol), _ = qmm.quantized_operand(ld, 1, fmt, per_channel=True)
    (cr, orr), _ = qmm.quantized_operand(rd, 1, fmt, per_channel=True)
    y = qmm.gemm((cl, ol), (cr, orr), torch.float32)
    ref = qmm.reference_gemm(ld.unsqueeze(0), rd.unsqueeze(0))
    denom = qmm.reference_gemm(ld.abs().unsqueeze(0), rd.abs().unsqueeze(0))      # |L| |R|: inputs of the metric
    m = qmm.metric(y, ref, denom).cpu().tolist()
    f = dict(zip(qmm.METRIC_FIELDS, m))
    return {"dof": dof, "format": fmt, "be_max": f["BE_max"], "be_mean": f["BE_sum"] / max(f["BE_cnt"], 1.0),
            "nsr": f["S_ee"] / f["S_rr"], "fields": f, "y": y, "ref": ref, "denom": denom}


def backward_error_sweep(dofs=W.BACKWARD_ERROR_DOFS, formats=(qmm.INT8, qmm.E4M3, qmm.E5M2), n=512, device="cuda:0"):
    return [backward_error_row(d, f, n, device) for d in dofs for f in formats]


def relative_error_profile(fmt, points_per_decade=384, decades=11, device="cuda:0"):
    """Relative error of Eq. 2 over magnitudes (the figure comparing the three formats under RTNE): positive bfloat16
    magnitudes log-spaced over `decades` decades below the largest one, 1.0, which the step size maps onto the
    format's largest code.  Library calls only: scale -> quantize -> dequantize, then qmm_metric over each decade's
    slice, whose Eq. 2 fields are the profile.  Returns one dict per decade d (magnitudes in (10^-(d+1), 10^-d]):
    re_max, re_mean (a value quantized to zero has relative error 1) and the number of magnitudes."""
    n = points_per_decade * decades
    x = torch.logspace(-float(decades), 0.0, n + 1, dtype=torch.float32)[1:].to(torch.bfloat16).to(device).reshape(1, -1)
    delta = qmm.scale(x, 1, fmt)
    codes = qmm.quantize(x, 1, fmt, delta)
    v = qmm.dequantize(codes, fmt, delta).reshape(-1)
    xf = x.float().reshape(-1)
    rows = []
    for d in range(decades):
        lo, hi = n - (d + 1) * points_per_decade, n - d * points_per_decade
        f = dict(zip(qmm.METRIC_FIELDS, qmm.metric(v[lo:hi].contiguous(), xf[lo:hi].contiguous()).cpu().tolist()))
        rows.append({"decade": d, "re_max": f["RE_max"], "re_mean": f["RE_sum"] / max(f["RE_cnt"], 1.0), "n": int(f["RE_cnt"])})
    return rows


# Candidates of the per-op choice, cheapest scaling first: one step size per tensor before one per channel.  The
# three 8-bit formats cost the same matrix rate on this part, so within a granularity the order is by typical error
# on near-normal operands (E4M3, INT8, E5M2).
CANDIDATES = ((qmm.E4M3, False), (qmm.INT8, False), (qmm.E5M2, False),
              (qmm.E4M3, True), (qmm.INT8, True), (qmm.E5M2, True))


def op_error(x, w, fmt_x, fmt_w, per_channel, ref=None):
    """Quantized product X W^T of one op (x: [M, K], w: [N, K], device bfloat16) against the high-precision product:
    dict with the noise-to-signal ratio and the mean / max relative error of Eq. 2.  Library calls only."""
    (cx, ox), _ = qmm.quantized_operand(x, 1, fmt_x, per_channel=per_channel)
    (cw, ow), _ = qmm.quantized_operand(w, 1, fmt_w, per_channel=per_channel)
    y = qmm.gemm((cx, ox), (cw, ow), torch.float32)
    if ref is None:
        ref = qmm.reference_gemm(x.unsqueeze(0), w.unsqueeze(0))
    f = dict(zip(qmm.METRIC_FIELDS, qmm.metric(y, ref).cpu().tolist()))
    return {"nsr": f["S_ee"] / f["S_rr"] if f["S_rr"] > 0 else float("inf"),
            "re_mean": f["RE_sum"] / max(f["RE_cnt"], 1.0), "re_max": f["RE_max"], "fields": f}


def format_sweep(x, w, candidates=CANDIDATES):
    """Error of every candidate (format, per_channel) on one op; the same format on both operands."""
    ref = qmm.reference_gemm(x.unsqueeze(0), w.unsqueeze(0))
    return [dict(format=fmt, per_channel=pc, **op_error(x, w, fmt, fmt, pc, ref)) for fmt, pc in candidates]


def choose_format(x, w, nsr_max, candidates=CANDIDATES):
    """The error metric applied to the mapping of one op onto a format (the mapping the Conclusion calls the crucial
    step; an extension: the paper chooses by training runs, not per op): the first candidate, in the order given,
    whose noise-to-signal ratio against the high-precision product is at most `nsr_max`; None if there is none (the
    op stays in bfloat16).  Returns (choice or None, the rows evaluated so far)."""
    ref = qmm.reference_gemm(x.unsqueeze(0), w.unsqueeze(0))
    rows = []
    for fmt, pc in candidates:
        rows.append(dict(format=fmt, per_channel=pc, **op_error(x, w, fmt, fmt, pc, ref)))
        if rows[-1]["nsr"] <= nsr_max:
            return (fmt, pc), rows
    return None, rows


def main():
    names = {v: k for k, v in qmm.FORMATS.items()}
    rows = backward_error_sweep()
    print(f"{'dof':>6s} {'format':>6s} {'BE max':>11s} {'BE mean':>11s} {'NSR':>11s}")
    for r in rows:
        dof = "normal" if r["dof"] is None else str(r["dof"])
        print(f"{dof:>6s} {names[r['format']]:>6s} {r['be_max']:11.3e} {r['be_mean']:11.3e} {r['nsr']:11.3e}")
    print("\nworst relative error of a value (Eq. 2) per decade of magnitude below the tensor's largest one")
    print(f"{'decade':>10s} " + " ".join(f"{n:>10s}" for n in ("int8", "e4m3", "e5m2")))
    prof = {f: relative_error_profile(f) for f in (qmm.INT8, qmm.E4M3, qmm.E5M2)}
    for d in range(0, 11):
        print(f"  1e-{d + 1:<2d}..1e-{d:<2d}" + " ".join(f"{prof[f][d]['re_max']:10.3e}" for f in (qmm.INT8, qmm.E4M3, qmm.E5M2)))
    print("\nnoise-to-signal ratio per op, BERT-large forward shapes (synthetic operands), format x granularity;"
          " choice = first candidate with NSR <= 1e-3")
    print(f"{'op':>9s} " + " ".join(f"{names[f] + ('/ch' if pc else '/t'):>10s}" for f, pc in CANDIDATES) + "  choice")
    for op in W.bert_forward_ops(**W.BERT_LARGE):
        x, w = W.forward_operands(op, 4, layer=0)
        xd, wd = x.to("cuda:0"), w.to("cuda:0")
        rows = format_sweep(xd, wd)
        choice = next(((r["format"], r["per_channel"]) for r in rows if r["nsr"] <= 1e-3), None)
        label = "bf16" if choice is None else names[choice[0]] + ("/ch" if choice[1] else "/t")
        print(f"{op.name:>9s} " + " ".join(f"{r['nsr']:10.3e}" for r in rows) + f"  {label}")


if __name__ == "__main__":
    main()
