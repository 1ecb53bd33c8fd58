#!/usr/bin/env python3
"""Benchmark of the quantized-matmul hot path on one MI355X.

One "step" = one pass of the whole path over the forward GEMMs of one BERT-large encoder layer
(16384 tokens, hidden 1024, FFN 4096: QKV, attention output, FFN1, FFN2): for every op
    qmm_scale(X), qmm_scale(W), qmm_quantize(X), qmm_quantize(W), qmm_gemm (+descale, bf16 out), qmm_metric(Y, Y_ref)
with E4M3 operands, per-tensor step sizes, synthetic seeded inputs already resident in HBM.  The
high-precision reference product Y_ref is an input of the metric pass and is computed once, outside
the timed region (it is the un-quantized baseline the method compares against, not part of the
quantized path).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload bert_large_fwd|bert_base_fwd]
                    [--format e4m3|e5m2|int8] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per GEMM launch (mean of the four launches of a step) from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this
# very command, scaled by what the same counters read for a plain 256 MiB copy (factors 2.00 and 1.00); the summary
# with the commands is profiles/bench_bert_large_fwd_e4m3.md.  Other workloads / formats: not collected (null).
GEMM_TRAFFIC = {("bert_large_fwd", "e4m3"): {"read_bytes": 56.6e6, "write_bytes": 75.6e6,
                                             "algorithmic_read_bytes": 32.4e6, "algorithmic_write_bytes": 75.4e6}}
PEAK = {"e4m3": 5000.0, "e5m2": 5000.0, "int8": 5000.0}   # dense MFMA TFLOP/s (TOP/s), MI355X
HBM_PEAK_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="bert_large_fwd", choices=["bert_large_fwd", "bert_base_fwd"])
    ap.add_argument("--format", default="e4m3", choices=["e4m3", "e5m2", "int8"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run ten plain device copies of 256 MiB (to scale the FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2408_02897_amd import qmm, workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = 256 << 20
        src = torch.ones(n, dtype=torch.uint8, device=dev); dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_copy": n, "bytes_written_per_copy": n, "copies": 10}}))
        return
    fmt = qmm.FORMATS[args.format]
    cfg_no, dims = (4, W.BERT_LARGE) if args.workload == "bert_large_fwd" else (2, W.BERT_BASE)
    ops = W.bert_forward_ops(**dims)

    # ---- inputs, resident in HBM; reference products (untimed)
    state = []
    for op in ops:
        x, w = W.forward_operands(op, cfg_no, layer=0)
        xd, wd = x.to(dev), w.to(dev)
        st = dict(op=op, x=xd, w=wd)
        st["y_ref"] = qmm.reference_gemm(xd.unsqueeze(0), wd.unsqueeze(0))
        st["dx"] = torch.empty(1, dtype=torch.float32, device=dev); st["dw"] = torch.empty(1, dtype=torch.float32, device=dev)
        st["cx"] = torch.empty((1, op.M, op.K), dtype=torch.uint8, device=dev)
        st["cw"] = torch.empty((1, op.N, op.K), dtype=torch.uint8, device=dev)
        st["y"] = torch.empty((1, op.M, op.N), dtype=torch.bfloat16, device=dev)
        st["m"] = torch.empty(16, dtype=torch.float64, device=dev)
        st["ws"] = torch.empty(1 << 20, dtype=torch.uint8, device=dev)
        st["host_x"], st["host_w"] = x, w
        state.append(st)
    torch.cuda.synchronize()

    kinds = ("scale", "quantize", "gemm", "metric")
    events = {k: [] for k in kinds}

    def timed(kind, record, fn):
        if kind in record:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); fn(); e1.record()
            events[kind].append((e0, e1))
        else:
            fn()

    for st in state:
        st["oa"] = qmm.operand(st["cx"], fmt, st["dx"]); st["ob"] = qmm.operand(st["cw"], fmt, st["dw"])
        # activations and weights of a product go through scale and quantize together (qmm_scale_multi /
        # qmm_quantize_multi: the tensor index is a grid dimension, so the 2-8 MB weight matrix, latency-bound on its
        # own, rides in the activations' launches); argument arrays built once
        st["xw"] = qmm.MultiDesc([st["x"], st["w"]])
        st["d_ptrs"] = qmm.MultiDesc.pointers([st["dx"], st["dw"]])
        st["c_ptrs"] = qmm.MultiDesc.pointers([st["cx"], st["cw"]])

    def step(record):
        for st in state:
            timed("scale", record, lambda: qmm.scale_multi(st["xw"], fmt, outs=[st["dx"], st["dw"]], workspace=st["ws"],
                                                           out_ptrs=st["d_ptrs"]))
            timed("quantize", record, lambda: qmm.quantize_multi(st["xw"], fmt, [st["dx"], st["dw"]],
                                                                 outs=[st["cx"], st["cw"]], delta_ptrs=st["d_ptrs"],
                                                                 out_ptrs=st["c_ptrs"]))
            timed("gemm", record, lambda: qmm.gemm((st["cx"], st["oa"]), (st["cw"], st["ob"]), out=st["y"]))
            timed("metric", record, lambda: qmm.metric(st["y"], st["y_ref"], out=st["m"], workspace=st["ws"]))

    # Timed region: K whole steps, with a pair of HIP events around every launch of the dominant kernel only (an
    # event pair costs about 4 us of stream time; around all 24 launches of a step it would add a sixth to the step).
    for _ in range(args.warmup):
        step(())
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(("gemm",))
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # The other kernel classes are timed the same way in K further steps, outside the timed region.
    for _ in range(args.steps):
        step(("scale", "quantize", "metric"))
    torch.cuda.synchronize()
    # The tensor-moments pass (not a step of the quantized product: it characterises the operands beforehand) over
    # the same X and W, timed the same way.
    events["moments"] = []
    mom = torch.empty(8, dtype=torch.float64, device=dev)
    for _ in range(args.steps):
        for st in state:
            timed("moments", ("moments",), lambda: (qmm.moments(st["x"], out=mom, workspace=st["ws"]),
                                                    qmm.moments(st["w"], out=mom, workspace=st["ws"])))
    torch.cuda.synchronize()

    flops = sum(op.flops for op in ops)
    ms_per_step = dt / args.steps * 1e3
    value = flops / (dt / args.steps) / 1e12

    # ---- per-kernel-class device time from HIP events on the launch stream
    per_kind_ms = {k: sum(a.elapsed_time(b) for a, b in v) / args.steps for k, v in events.items()}
    elems_x = sum(op.M * op.K for op in ops); elems_w = sum(op.N * op.K for op in ops); elems_y = sum(op.M * op.N for op in ops)
    algo_bytes = {"scale": 2 * (elems_x + elems_w), "quantize": 3 * (elems_x + elems_w),
                  "metric": (2 + 4) * elems_y, "moments": 2 * (elems_x + elems_w)}
    gemm_ms_per_launch = per_kind_ms["gemm"] / len(ops)
    gemm_tflops = flops / (per_kind_ms["gemm"] * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "gemm_stream_kernel (QKV, FFN1) + gemm_kernel (attn_out, FFN2): fp8/int8 MFMA, 4 launches per step",
                "achieved": round(gemm_tflops, 1), "peak": PEAK[args.format], "unit": "TFLOP/s",
                "frac": round(gemm_tflops / PEAK[args.format], 4),
                "traffic": GEMM_TRAFFIC.get((args.workload, args.format)),
                "avg_launch_ms": round(gemm_ms_per_launch, 4)}
    g_ms = [a.elapsed_time(b) for a, b in events["gemm"]]       # launch order: step-major, op-minor
    roofline["median_launch_ms_by_op"] = {st["op"].name: round(sorted(g_ms[i::len(ops)])[args.steps // 2], 4)
                                          for i, st in enumerate(state)}
    # ---- what the matrix units sustain on these very codes with no memory traffic (and on constant codes): the
    #      chip's clock under matrix load is set by power, which depends on the operand bytes
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(n_cu * 256, dtype=torch.float32, device=dev)

    def mfma_only(codes):
        ts = []
        for _ in range(4):       # about 1 ms each, so that dispatch latency does not count
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); _, fl = qmm.mfma_rate(codes, fmt, fmt, rounds=1000, workgroups=n_cu, sink=sink); e1.record()
            torch.cuda.synchronize(); ts.append(e0.elapsed_time(e1))
        return fl / (sorted(ts[1:])[1] * 1e-3) / 1e12
    big = max(state, key=lambda st: st["cx"].numel())
    const_code = 0x38 if fmt != qmm.INT8 else 0x40
    mfma_codes = mfma_only(big["cx"].view(-1))
    mfma_const = mfma_only(torch.full((1 << 20,), const_code, dtype=torch.uint8, device=dev))
    # stream time an event pair adds around a launch (dispatch latency): a pair around a one-element kernel
    tiny = torch.zeros(1, device=dev)
    ov = []
    for _ in range(20):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); tiny.add_(1.0); e1.record(); torch.cuda.synchronize(); ov.append(e0.elapsed_time(e1))
    roofline["event_pair_around_one_element_kernel_ms"] = round(sorted(ov)[len(ov) // 2], 4)
    roofline["mfma_only_tflops"] = {"workload_codes": round(mfma_codes, 1), "constant_codes": round(mfma_const, 1)}
    roofline["frac_of_mfma_only_on_workload_codes"] = round(gemm_tflops / mfma_codes, 4)
    # ---- context only, no part of the path: the vendor library's FP8 GEMM (torch._scaled_mm, i.e. hipBLASLt) on this
    #      step's own code matrices with unit scales and bf16 output.  Ten launches back to back per op between one
    #      event pair: its dispatch through torch costs more host time than ours, and timed launch by launch that
    #      would be charged to its kernel (its kernel time by rocprofv3 is in profiles/).
    def library_context():
        if fmt == qmm.INT8:
            return None
        try:
            dt8 = torch.float8_e4m3fn if fmt == qmm.E4M3 else torch.float8_e5m2
            one = torch.ones((), device=dev)
            total_ms, per_op = 0.0, {}
            for st in state:
                a, b = st["cx"][0].view(dt8), st["cw"][0].view(dt8)
                ts = []
                for it in range(4):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(10):
                        torch._scaled_mm(a, b.t(), scale_a=one, scale_b=one, out_dtype=torch.bfloat16)
                    e1.record()
                    torch.cuda.synchronize()
                    if it >= 1:
                        ts.append(e0.elapsed_time(e1) / 10)
                per_op[st["op"].name] = round(sorted(ts)[len(ts) // 2], 4)
                total_ms += per_op[st["op"].name]
            return {"what": "torch._scaled_mm (hipBLASLt) on the same codes, 10 launches back to back per event pair",
                    "tflops": round(flops / (total_ms * 1e-3) / 1e12, 1), "ms_per_launch": per_op}
        except Exception as e:          # the library may lack the call: the context line is then left out
            return {"error": str(e)[:120]}
    roofline["vendor_library_gemm"] = library_context()

    def own_back_to_back():
        total_ms, per_op = 0.0, {}
        for st in state:
            ts = []
            for it in range(4):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(10):
                    qmm.gemm((st["cx"], st["oa"]), (st["cw"], st["ob"]), out=st["y"])
                e1.record()
                torch.cuda.synchronize()
                if it >= 1:
                    ts.append(e0.elapsed_time(e1) / 10)
            per_op[st["op"].name] = round(sorted(ts)[len(ts) // 2], 4)
            total_ms += per_op[st["op"].name]
        return {"what": "qmm_gemm timed the same way (10 launches back to back per event pair)",
                "tflops": round(flops / (total_ms * 1e-3) / 1e12, 1), "ms_per_launch": per_op}
    roofline["gemm_back_to_back"] = own_back_to_back()

    # the same product with the noise-to-signal sums taken in its epilogue (qmm_gemm_nsr), next to the product
    # followed by the full metric pass, both ten launches back to back per event pair
    def fused_nsr_context():
        def ms_of(fn):
            ts = []
            for it in range(4):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(10):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                if it >= 1:
                    ts.append(e0.elapsed_time(e1) / 10)
            return sorted(ts)[len(ts) // 2]
        o2 = torch.empty(2, dtype=torch.float64, device=dev)
        ws = torch.empty(4 << 20, dtype=torch.uint8, device=dev)
        fused, separate = {}, {}
        for st in state:
            fused[st["op"].name] = round(ms_of(lambda: qmm.gemm_nsr((st["cx"], st["oa"]), (st["cw"], st["ob"]), st["y_ref"][0],
                                                                    out=st["y"], out2=o2, workspace=ws)), 4)
            separate[st["op"].name] = round(ms_of(lambda: (qmm.gemm((st["cx"], st["oa"]), (st["cw"], st["ob"]), out=st["y"]),
                                                           qmm.metric(st["y"], st["y_ref"], out=st["m"], workspace=st["ws"]))), 4)
        return {"what": "qmm_gemm_nsr (two sums of the noise-to-signal ratio in the epilogue) against qmm_gemm + qmm_metric "
                        "(all 16 fields), ms per op", "gemm_nsr": fused, "gemm_then_metric": separate}
    roofline["fused_nsr"] = fused_nsr_context()
    passes = {k: {"ms_per_step": round(per_kind_ms[k], 4),
                  "GBps": round(algo_bytes[k] / (per_kind_ms[k] * 1e-3) / 1e9, 1),
                  "frac_hbm": round(algo_bytes[k] / (per_kind_ms[k] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
              for k in ("scale", "quantize", "metric", "moments")}
    nsr = {st["op"].name: float(st["m"][0].item() / st["m"][1].item()) for st in state}

    # ---- the memory-bound passes on the step's largest tensors alone, free of launch latency: ten launches back to
    #      back per event pair, rotating over three copies of the operand (more bytes than the 256 MB memory-side
    #      cache holds, so every launch reads HBM); the metric's inputs are larger than that cache by themselves
    def passes_on_largest():
        big_x = max(state, key=lambda st: st["x"].numel())
        xs = [big_x["x"]] + [big_x["x"].clone() for _ in range(2)]
        cs = [torch.empty_like(big_x["cx"]) for _ in range(3)]
        big_y = max(state, key=lambda st: st["y"].numel())
        nx, ny = big_x["x"].numel(), big_y["y"].numel()
        ws, dx, m = big_x["ws"], big_x["dx"], big_y["m"]
        qmm.scale(xs[0], 1, fmt, out=dx, workspace=ws)

        def rate(nbytes, fn):
            ts = []
            for it in range(4):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for k in range(10):
                    fn(k % 3)
                e1.record()
                torch.cuda.synchronize()
                if it >= 1:
                    ts.append(e0.elapsed_time(e1) / 10)
            ms = sorted(ts)[len(ts) // 2]
            return {"bytes_per_launch": nbytes, "ms_per_launch": round(ms, 4), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                    "frac_hbm": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        return {"what": "largest X of the step (scale, quantize, moments) and largest Y (metric), 10 launches back to back per "
                        "event pair, operands rotated over 3 copies",
                "scale": rate(2 * nx, lambda k: qmm.scale(xs[k], 1, fmt, out=dx, workspace=ws)),
                "quantize": rate(3 * nx, lambda k: qmm.quantize(xs[k], 1, fmt, dx, out=cs[k])),
                "metric": rate(6 * ny, lambda k: qmm.metric(big_y["y"], big_y["y_ref"], out=m, workspace=ws)),
                "moments": rate(2 * nx, lambda k: qmm.moments(xs[k], out=mom, workspace=ws))}
    passes["largest_tensors"] = passes_on_largest()

    # ---- the oracle timed on the host cores, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(state, args.format)

    out = {"metric": "quantized GEMM TFLOP/s (e4m3/int8) + metric-pass GB/s, % of MI355X peak",
           "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": {"e4m3": "fp8_e4m3", "e5m2": "fp8_e5m2", "int8": "int8"}[args.format], "data": "synthetic",
           "config": {"workload": f"{args.workload}: scale+quantize+gemm+descale+metric over QKV, attn_out, FFN1, FFN2 "
                                  f"(tokens {dims['tokens']}, hidden {dims['hidden']}, ffn {dims['ffn']}), "
                                  f"{args.format} per-tensor, bf16 out, reference product precomputed",
                      "flops_per_step": flops},
           "roofline": roofline, "passes": passes, "gemm_tflops": round(gemm_tflops, 1), "nsr": nsr,
           "cpu_baseline": cpu}
    print(json.dumps(out))


def cpu_baseline(state, fmt_name, rows_per_op=8192):
    """Time the oracle (as it stands) on `rows_per_op` seeded rows of every op: scale and quantize of those rows of X
    and of all of W, the product of those rows with all of W, descale and metric."""
    import numpy as np
    from oracle import oracle as O
    fmt = O.FORMATS[fmt_name]
    O.lib()
    flops = 0
    t0 = time.perf_counter()
    for st in state:
        op = st["op"]
        rng = np.random.default_rng(op.M + op.N)
        rows = np.sort(rng.choice(op.M, size=min(rows_per_op, op.M), replace=False))
        xs = st["host_x"][torch_index(rows)].float().numpy()
        w = st["host_w"].float().numpy()
        dx = O.scale(xs, 1, fmt); dw = O.scale(w, 1, fmt)
        cx = O.quantize(xs, 1, fmt, dx); cw = O.quantize(w, 1, fmt, dw)
        acc = O.gemm_codes(cx, fmt, cw, fmt, want_sabs=False)
        y = O.dequant(acc, dx, dw, out_bf16=True)
        r = O.ref_gemm(xs, w)
        O.metric(y, r)
        flops += 2 * len(rows) * op.N * op.K
    dt = time.perf_counter() - t0
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": O.num_threads(), "kind": "oracle",
            "sample": f"{rows_per_op} seeded rows of X per op against all of W (4 ops), full path incl. reference product; "
                      f"{dt:.1f} s of CPU work"}


def torch_index(rows):
    import torch
    return torch.from_numpy(rows)


if __name__ == "__main__":
    main()
