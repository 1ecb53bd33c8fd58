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


def main():
    names = {v: k for k, v in qmm.FORMATS.items()}
    rows = backward_error_sweep()
    print(f"{'dof':>6s} {'format':>6s} {'BE max':>11s} {'BE mean':>11s} {'NSR':>11s}")
    for r in rows:
        dof = "normal" if r["dof"] is None else str(r["dof"])
        print(f"{dof:>6s} {names[r['format']]:>6s} {r['be_max']:11.3e} {r['be_mean']:11.3e} {r['nsr']:11.3e}")


if __name__ == "__main__":
    main()
