#!/usr/bin/env python3
"""Benchmark of the quantized-matmul hot path on one MI355X.

One "step" = one pass of the whole path over the forward GEMMs of one BERT-large encoder layer
(16384 tokens, hidden 1024, FFN 4096: QKV, attention output, FFN1, FFN2): for every op
    qmm_scale(X, W), qmm_quantize(X, W), qmm_gemm (+descale, bf16 out), qmm_metric(Y, Y_ref)
with per-tensor step sizes, synthetic seeded inputs already resident in HBM.  The high-precision reference product
Y_ref is an input of the metric pass and is computed once, outside the timed region (it is the un-quantized baseline
the method compares against, not part of the quantized path).  The headline (`value`, `roofline`, `passes`) is that
step in E4M3; the same line carries, measured after the timed region:
    int8        the same step in INT8 (the metric names both types)
    ops         every product of the layer -- forward, dgrad, wgrad; E4M3 (gradients E5M2) and INT8; step sizes per
                tensor and per channel -- as GEMM time, TFLOP/s and fraction of the 5.0 PFLOP/s peak
    attention   the batched products of BERT-large attention (32 x 16 heads, 512 x 512 x 64), bound by their output
                stream: GB/s of codes in + Y out
    ceilings    what plain streaming kernels reach on buffers larger than the caches (read, copy)
Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload bert_large_fwd|bert_base_fwd]
                    [--format e4m3|e5m2|int8] [--settle-ms T] [--no-cpu-baseline] [--no-extras] [--full]
The line on stdout is compact (numbers per section); every table goes to a JSON file whose path the line gives as `detail`.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per GEMM launch by format, from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this very command: written by
# `python -m paper_2408_02897_amd.traffic` from the counter files (the commands are in profiles/).
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gemm_traffic.json")
PEAK = {"e4m3": 5000.0, "e5m2": 5000.0, "int8": 5000.0}   # dense MFMA TFLOP/s (TOP/s), MI355X
HBM_PEAK_GBS = 8000.0
GEMM_EVENT_EVERY = 4       # timed region: HIP events around the GEMM launches of every fourth step
DTYPE = {"e4m3": "fp8_e4m3", "e5m2": "fp8_e5m2", "int8": "int8"}


def load_traffic(workload, fmt_name):
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f).get(f"{workload}/{fmt_name}")
    except (OSError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="bert_large_fwd", choices=["bert_large_fwd", "bert_base_fwd"])
    ap.add_argument("--format", default="e4m3", choices=["e4m3", "e5m2", "int8"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--settle-ms", type=float, default=15.0,
                    help="run the step untimed for this long before the warm-up steps, so that the clock has settled (0: off)")
    ap.add_argument("--no-extras", action="store_true", help="only the timed step (what the profiling commands run)")
    ap.add_argument("--full", action="store_true", help="print every table in the line instead of the compact form")
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
    cfg_no, dims = (4, W.BERT_LARGE) if args.workload == "bert_large_fwd" else (2, W.BERT_BASE)
    ops = W.bert_forward_ops(**dims)
    flops = sum(op.flops for op in ops)

    def event_pair():
        return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def back_to_back_ms(fn, launches=10, repeats=5, settle_ms=12.0):
        """median over `repeats` of (time of `launches` calls between one event pair) / launches, after the same calls have
        kept the GPU busy for `settle_ms`: a measurement taken right behind set-up work (allocation, the quantize
        kernels, a host synchronisation) runs at whatever clock the part is ramping through and read up to 20 % off
        either way; once the same launches have run for some 10 ms the figure repeats to 2-3 %."""
        spent, k = 0.0, 0
        while spent < settle_ms and k < 2000:
            e0, e1 = event_pair()
            e0.record()
            for i in range(launches):
                fn(k + i)
            e1.record()
            torch.cuda.synchronize()
            spent += e0.elapsed_time(e1); k += launches
        ts = []
        for it in range(repeats):
            e0, e1 = event_pair()
            e0.record()
            for k in range(launches):
                fn(k)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) / launches)
        return sorted(ts)[len(ts) // 2]

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
        # activations and weights of a product go through scale and quantize together (qmm_scale_multi /
        # qmm_quantize_multi: the tensor index is a grid dimension, so the 2-8 MB weight matrix, latency-bound on its
        # own, rides in the activations' launches); argument arrays built once
        st["xw"] = qmm.MultiDesc([st["x"], st["w"]])
        st["d_ptrs"] = qmm.MultiDesc.pointers([st["dx"], st["dw"]])
        st["c_ptrs"] = qmm.MultiDesc.pointers([st["cx"], st["cw"]])
        state.append(st)
    torch.cuda.synchronize()
    elems_x = sum(op.M * op.K for op in ops); elems_w = sum(op.N * op.K for op in ops); elems_y = sum(op.M * op.N for op in ops)
    algo_bytes = {"scale": 2 * (elems_x + elems_w), "quantize": 3 * (elems_x + elems_w),
                  "metric": (2 + 4) * elems_y, "moments": 2 * (elems_x + elems_w)}

    def run_steps(fmt_name, steps, warmup):
        """The step in one format: wall clock around `steps` steps with an event pair around every GEMM launch, then
        `steps` further steps with event pairs around the other kernel classes."""
        fmt = qmm.FORMATS[fmt_name]
        kinds = ("scale", "quantize", "gemm", "metric")
        events = {k: [] for k in kinds}
        for st in state:
            st["oa"] = qmm.operand(st["cx"], fmt, st["dx"]); st["ob"] = qmm.operand(st["cw"], fmt, st["dw"])

        def timed(kind, record, fn):
            if kind in record:
                e0, e1 = event_pair()
                e0.record(); fn(); e1.record()
                events[kind].append((e0, e1))
            else:
                fn()

        def step(record):
            for st in state:
                timed("scale", record, lambda: qmm.scale_multi(st["xw"], fmt, outs=[st["dx"], st["dw"]], workspace=st["ws"],
                                                               out_ptrs=st["d_ptrs"]))
                timed("quantize", record, lambda: qmm.quantize_multi(st["xw"], fmt, [st["dx"], st["dw"]],
                                                                     outs=[st["cx"], st["cw"]], delta_ptrs=st["d_ptrs"],
                                                                     out_ptrs=st["c_ptrs"]))
                timed("gemm", record, lambda: qmm.gemm((st["cx"], st["oa"]), (st["cw"], st["ob"]), out=st["y"]))
                timed("metric", record, lambda: qmm.metric(st["y"], st["y_ref"], out=st["m"], workspace=st["ws"]))

        # Timed region: whole steps, with a pair of HIP events around the launches of the dominant kernel only, in every
        # fourth step (an event pair costs several us of stream time: around all 16 launches of every step it would add a
        # tenth to the step, around the four GEMM launches of every step still 4 %).
        # Set-up, untimed: the step runs until the GPU has been busy for `--settle-ms` (the part's clock under this load
        # takes some 10 ms to settle; a step is half a millisecond, so a handful of warm-up steps end while it still
        # ramps and the steps timed behind them read 5 % low).  Then the W warm-up steps, then exactly K timed steps.
        t_settle = time.perf_counter()
        while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
            for _ in range(4):
                step(())
            torch.cuda.synchronize()
        for _ in range(warmup):
            step(())
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(("gemm",) if i % GEMM_EVENT_EVERY == 0 else ())
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        for _ in range(steps):
            step(("scale", "quantize", "metric"))
        torch.cuda.synchronize()
        n_gemm_steps = (steps + GEMM_EVENT_EVERY - 1) // GEMM_EVENT_EVERY
        per_kind_ms = {k: sum(a.elapsed_time(b) for a, b in v) / (n_gemm_steps if k == "gemm" else steps) for k, v in events.items()}
        g_ms = [a.elapsed_time(b) for a, b in events["gemm"]]       # launch order: step-major, op-minor
        gemm_tflops = flops / (per_kind_ms["gemm"] * 1e-3) / 1e12
        res = {"ms_per_step": dt / steps * 1e3, "value": flops / (dt / steps) / 1e12, "gemm_tflops": gemm_tflops,
               "gemm_ms_per_launch": per_kind_ms["gemm"] / len(ops), "per_kind_ms": per_kind_ms,
               "median_launch_ms_by_op": {st["op"].name: round(sorted(g_ms[i::len(ops)])[n_gemm_steps // 2], 4)
                                          for i, st in enumerate(state)},
               "nsr": {st["op"].name: float(st["m"][0].item() / st["m"][1].item()) for st in state}}
        res["passes"] = {k: {"ms_per_step": round(per_kind_ms[k], 4),
                             "GBps": round(algo_bytes[k] / (per_kind_ms[k] * 1e-3) / 1e9, 1),
                             "frac_hbm": round(algo_bytes[k] / (per_kind_ms[k] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
                         for k in ("scale", "quantize", "metric")}
        return res

    main_res = run_steps(args.format, args.steps, args.warmup)
    fmt = qmm.FORMATS[args.format]
    passes = main_res["passes"]
    traffic = load_traffic(args.workload, args.format)
    roofline = {"bound": "mfma", "kernel": "gemm_stream_kernel (QKV, FFN1) + gemm_kernel (attn_out, FFN2): fp8/int8 MFMA, 4 launches per step",
                "achieved": round(main_res["gemm_tflops"], 1), "peak": PEAK[args.format], "unit": "TFLOP/s",
                "frac": round(main_res["gemm_tflops"] / PEAK[args.format], 4),
                "traffic": traffic, "avg_launch_ms": round(main_res["gemm_ms_per_launch"], 4),
                "median_launch_ms_by_op": main_res["median_launch_ms_by_op"]}
    out = {"metric": "quantized GEMM TFLOP/s (e4m3/int8) + metric-pass GB/s, % of MI355X peak",
           "value": round(main_res["value"], 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(main_res["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": DTYPE[args.format], "data": "synthetic",
           "config": {"workload": f"{args.workload} ({args.format}, per-tensor, bf16 out): scale+quantize+gemm+metric of QKV, "
                                  f"attn_out, FFN1, FFN2; tokens {dims['tokens']}, hidden {dims['hidden']}, ffn {dims['ffn']}",
                      "flops_per_step": flops, "settle_ms_before_warmup": args.settle_ms},
           "roofline": roofline, "passes": passes, "gemm_tflops": round(main_res["gemm_tflops"], 1), "nsr": main_res["nsr"]}
    if args.no_extras:
        out["cpu_baseline"] = None
        if traffic:
            roofline["traffic"] = traffic["read_bytes"] + traffic["write_bytes"]
            roofline["traffic_detail"] = traffic
        print(json.dumps(out))
        return

    # ---- the tensor-moments pass (not a step of the quantized product: it characterises the operands beforehand) over
    #      the same X and W, an event pair around the two calls of an op
    mom = torch.empty(8, dtype=torch.float64, device=dev)
    mom_ev = []
    for _ in range(args.steps):
        for st in state:
            e0, e1 = event_pair()
            e0.record(); qmm.moments(st["x"], out=mom, workspace=st["ws"]); qmm.moments(st["w"], out=mom, workspace=st["ws"]); e1.record()
            mom_ev.append((e0, e1))
    torch.cuda.synchronize()
    mom_ms = sum(a.elapsed_time(b) for a, b in mom_ev) / args.steps
    passes["moments"] = {"ms_per_step": round(mom_ms, 4), "GBps": round(algo_bytes["moments"] / (mom_ms * 1e-3) / 1e9, 1),
                         "frac_hbm": round(algo_bytes["moments"] / (mom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    # ---- what the matrix units sustain on these very codes with no memory traffic (and on constant codes): the
    #      chip's clock under matrix load is set by power, which depends on the operand bytes
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(n_cu * 256, dtype=torch.float32, device=dev)

    def mfma_only(codes, f=None):
        f = fmt if f is None else f
        ts = []
        for it in range(16):     # about 1 ms each, so that dispatch latency does not count; the first ten let the clock settle
            e0, e1 = event_pair()
            e0.record(); _, fl = qmm.mfma_rate(codes, f, f, rounds=1000, workgroups=n_cu, sink=sink); e1.record()
            torch.cuda.synchronize()
            if it >= 10: ts.append(e0.elapsed_time(e1))
        return fl / (sorted(ts)[len(ts) // 2] * 1e-3) / 1e12
    big = max(state, key=lambda st: st["cx"].numel())
    const_code = 0x38 if fmt != qmm.INT8 else 0x40
    mfma_codes = mfma_only(big["cx"].view(-1))
    mfma_const = mfma_only(torch.full((1 << 20,), const_code, dtype=torch.uint8, device=dev))
    # stream time an event pair adds around a launch (dispatch latency): a pair around a one-element kernel
    tiny = torch.zeros(1, device=dev)
    ov = []
    for _ in range(20):
        e0, e1 = event_pair()
        e0.record(); tiny.add_(1.0); e1.record(); torch.cuda.synchronize(); ov.append(e0.elapsed_time(e1))
    roofline["event_pair_around_one_element_kernel_ms"] = round(sorted(ov)[len(ov) // 2], 4)
    roofline["mfma_only_tflops"] = {"workload_codes": round(mfma_codes, 1), "constant_codes": round(mfma_const, 1)}
    roofline["frac_of_mfma_only_on_workload_codes"] = round(main_res["gemm_tflops"] / mfma_codes, 4)

    # ---- context only, no part of the path: the vendor library's FP8 GEMM (torch._scaled_mm, i.e. hipBLASLt) on this
    #      step's own code matrices with unit scales and bf16 output, ten launches back to back per event pair
    def library_context():
        if fmt == qmm.INT8:
            return None
        try:
            dt8 = torch.float8_e4m3fn if fmt == qmm.E4M3 else torch.float8_e5m2
            one = torch.ones((), device=dev)
            total_ms, per_op = 0.0, {}
            for st in state:
                a, b = st["cx"][0].view(dt8), st["cw"][0].view(dt8)
                ms = back_to_back_ms(lambda k: torch._scaled_mm(a, b.t(), scale_a=one, scale_b=one, out_dtype=torch.bfloat16))
                per_op[st["op"].name] = round(ms, 4)
                total_ms += ms
            return {"what": "torch._scaled_mm (hipBLASLt) on the same codes, 10 launches back to back per event pair",
                    "tflops": round(flops / (total_ms * 1e-3) / 1e12, 1), "ms_per_launch": per_op}
        except Exception as e:          # the library may lack the call: the context line is then left out
            return {"error": str(e)[:120]}
    roofline["vendor_library_gemm"] = library_context()

    def own_back_to_back():
        total_ms, per_op = 0.0, {}
        for st in state:
            ms = back_to_back_ms(lambda k: qmm.gemm((st["cx"], st["oa"]), (st["cw"], st["ob"]), out=st["y"]))
            per_op[st["op"].name] = round(ms, 4)
            total_ms += ms
        return {"what": "qmm_gemm timed the same way (10 launches back to back per event pair)",
                "tflops": round(flops / (total_ms * 1e-3) / 1e12, 1), "ms_per_launch": per_op}
    roofline["gemm_back_to_back"] = own_back_to_back()

    # the same product with the noise-to-signal sums taken in its epilogue (qmm_gemm_nsr), next to the product
    # followed by the full metric pass, both ten launches back to back per event pair
    def fused_nsr_context():
        o2 = torch.empty(2, dtype=torch.float64, device=dev)
        ws = torch.empty(4 << 20, dtype=torch.uint8, device=dev)
        fused, separate = {}, {}
        for st in state:
            fused[st["op"].name] = round(back_to_back_ms(lambda k: qmm.gemm_nsr((st["cx"], st["oa"]), (st["cw"], st["ob"]), st["y_ref"][0],
                                                                                out=st["y"], out2=o2, workspace=ws)), 4)
            separate[st["op"].name] = round(back_to_back_ms(lambda k: (qmm.gemm((st["cx"], st["oa"]), (st["cw"], st["ob"]), out=st["y"]),
                                                                       qmm.metric(st["y"], st["y_ref"], out=st["m"], workspace=st["ws"]))), 4)
        return {"what": "qmm_gemm_nsr (two sums of the noise-to-signal ratio in the epilogue) against qmm_gemm + qmm_metric "
                        "(all 16 fields), ms per op", "gemm_nsr": fused, "gemm_then_metric": separate}
    roofline["fused_nsr"] = fused_nsr_context()

    # ---- the memory-bound passes on the step's largest tensors alone, free of launch latency: ten launches back to
    #      back per event pair, rotating over three copies of the operand (more bytes than the 256 MB memory-side
    #      cache holds, so every launch reads HBM); the metric's inputs are larger than that cache by themselves.
    #      Next to them the ceilings: a plain read and a plain copy kernel (qmm_hbm_rate) over three rotating 256 MiB buffers.
    def rate(nbytes, fn, ceiling=None):
        ms = back_to_back_ms(lambda k: fn(k % 3))
        r = {"bytes_per_launch": nbytes, "ms_per_launch": round(ms, 4), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
             "frac_hbm": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        if ceiling:
            r["frac_of_measured_ceiling"] = round(r["GBps"] / ceiling, 4)
        return r

    def ceilings():
        sk = torch.empty(1024 * 256, dtype=torch.int32, device=dev)
        def bufs(nbytes, count):
            return [torch.full((nbytes,), i + 1, dtype=torch.uint8, device=dev) for i in range(count)]
        small = bufs(128 << 20, 3)                          # the size of the step's largest X
        dsts = [torch.empty(128 << 20, dtype=torch.uint8, device=dev) for _ in range(3)]
        rd128 = rate(128 << 20, lambda k: qmm.hbm_rate(small[k], None, 1024, sk))
        cp128 = rate(2 * (128 << 20), lambda k: qmm.hbm_rate(small[k], dsts[k], 1024, sk))
        del dsts
        large = bufs(384 << 20, 3)                          # the bytes one metric launch reads (Y bf16 + Y_ref)
        rd384 = rate(384 << 20, lambda k: qmm.hbm_rate(large[k], None, 1024, sk))
        return {"what": "plain streaming kernels (qmm_hbm_rate, 1024 workgroups, 16-byte streaming loads / stores) over three "
                        "rotating buffers of the passes' own sizes, 10 launches back to back per event pair; copy counts bytes "
                        "read + written", "read_128MiB": rd128, "read_384MiB": rd384, "copy_128MiB": cp128}
    ceil = ceilings()

    def passes_on_largest():
        big_x = max(state, key=lambda st: st["x"].numel())
        xs = [big_x["x"]] + [big_x["x"].clone() for _ in range(2)]
        cs = [torch.empty_like(big_x["cx"]) for _ in range(3)]
        big_y = max(state, key=lambda st: st["y"].numel())
        nx, ny = big_x["x"].numel(), big_y["y"].numel()
        ws, dx, m = big_x["ws"], big_x["dx"], big_y["m"]
        qmm.scale(xs[0], 1, fmt, out=dx, workspace=ws)
        return {"what": "largest X of the step (scale, quantize, moments) and largest Y (metric), 10 launches back to back per "
                        "event pair, operands rotated over 3 copies; frac_of_measured_ceiling is against the plain read kernel on "
                        "buffers of the same size (quantize: against the plain copy kernel)",
                "scale": rate(2 * nx, lambda k: qmm.scale(xs[k], 1, fmt, out=dx, workspace=ws), ceil["read_128MiB"]["GBps"]),
                "quantize": rate(3 * nx, lambda k: qmm.quantize(xs[k], 1, fmt, dx, out=cs[k]), ceil["copy_128MiB"]["GBps"]),
                "metric": rate(6 * ny, lambda k: qmm.metric(big_y["y"], big_y["y_ref"], out=m, workspace=ws), ceil["read_384MiB"]["GBps"]),
                "moments": rate(2 * nx, lambda k: qmm.moments(xs[k], out=mom, workspace=ws), ceil["read_128MiB"]["GBps"])}
    passes["largest_tensors"] = passes_on_largest()
    out["ceilings"] = ceil

    # ---- the same step in INT8 (the metric names e4m3 and int8)
    if args.format == "e4m3" and args.workload == "bert_large_fwd":
        r8 = run_steps("int8", max(5, args.steps // 2), 2)
        out["int8"] = {"what": "the same step with INT8 operands (one step size per tensor), timed the same way",
                       "value": round(r8["value"], 2), "unit": "TOP/s", "ms_per_step": round(r8["ms_per_step"], 4),
                       "roofline": {"bound": "mfma", "achieved": round(r8["gemm_tflops"], 1), "peak": PEAK["int8"], "unit": "TOP/s",
                                    "frac": round(r8["gemm_tflops"] / PEAK["int8"], 4), "traffic": load_traffic(args.workload, "int8"),
                                    "avg_launch_ms": round(r8["gemm_ms_per_launch"], 4),
                                    "median_launch_ms_by_op": r8["median_launch_ms_by_op"]},
                       "passes": r8["passes"], "nsr": r8["nsr"]}
        # the state now holds INT8 codes: what the matrix units sustain on them with no memory traffic
        out["int8"]["roofline"]["mfma_only_tops_workload_codes"] = round(mfma_only(big["cx"].view(-1), qmm.INT8), 1)
        out["ops"] = ops_table(torch, qmm, W, state, ops, cfg_no, back_to_back_ms, dev)
        out["attention"] = attention_products(torch, qmm, W, back_to_back_ms, dev)

    # ---- the oracle timed on the host cores, on a bounded sample of the same workload
    out["cpu_baseline"] = None if args.no_cpu_baseline else cpu_baseline(state, args.format)
    if args.full:
        print(json.dumps(out))
        return
    # Everything measured goes to a file; the ONE line on stdout carries the contract keys and the figures of each section
    # as plain numbers (a few KB).
    try:
        os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(ROOT, "gpurun_out", "bench_detail.json"), "w") as f:
            json.dump(out, f, indent=1)
    except OSError:
        pass
    print(json.dumps(compact_line(out)))


def compact_line(out):
    """The printed line: contract keys unchanged; nested tables flattened to numbers."""
    r = out["roofline"]
    t = r.get("traffic") or {}
    roof = {k: r[k] for k in ("bound", "kernel", "achieved", "peak", "unit", "frac", "avg_launch_ms")}
    roof["traffic"] = (t["read_bytes"] + t["write_bytes"]) if t else None        # HBM bytes per launch, by counters
    if t:
        roof.update({"traffic_read_bytes": t["read_bytes"], "traffic_write_bytes": t["write_bytes"],
                     "algorithmic_bytes": t["algorithmic_read_bytes"] + t["algorithmic_write_bytes"],
                     "operand_reread_ratio": t.get("reread_ratio")})
    roof["ms_by_op"] = r["median_launch_ms_by_op"]
    roof.update({"event_pair_overhead_ms": r["event_pair_around_one_element_kernel_ms"],
                 "mfma_only_tflops_workload_codes": r["mfma_only_tflops"]["workload_codes"],
                 "mfma_only_tflops_constant_codes": r["mfma_only_tflops"]["constant_codes"],
                 "frac_of_mfma_only_on_workload_codes": r["frac_of_mfma_only_on_workload_codes"],
                 "gemm_back_to_back_tflops": r["gemm_back_to_back"]["tflops"],
                 "vendor_library_gemm_tflops": (r["vendor_library_gemm"] or {}).get("tflops")})
    line = {k: out[k] for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                                "scaling", "vs_baseline", "dtype", "data", "config")}
    if "int8" in out:
        i8 = out["int8"]
        roof.update({"int8_achieved": i8["roofline"]["achieved"], "int8_frac": i8["roofline"]["frac"],
                     "int8_step_value": i8["value"], "int8_ms_per_step": i8["ms_per_step"],
                     "int8_mfma_only_tops_workload_codes": i8["roofline"].get("mfma_only_tops_workload_codes")})
        t8 = i8["roofline"].get("traffic") or {}
        if t8:
            roof["int8_traffic"] = t8["read_bytes"] + t8["write_bytes"]
    c = out["ceilings"]
    roof.update({"hbm_read_ceiling_GBps": c["read_128MiB"]["GBps"], "hbm_read_ceiling_384MiB_GBps": c["read_384MiB"]["GBps"],
                 "hbm_copy_ceiling_GBps": c["copy_128MiB"]["GBps"]})
    line["roofline"] = roof
    ps = out["passes"]
    big = ps["largest_tensors"]
    line["passes"] = {k: {"in_step_GBps": ps[k]["GBps"], "in_step_frac_hbm": ps[k]["frac_hbm"],
                          "largest_tensor_GBps": big[k]["GBps"], "largest_tensor_frac_hbm": big[k]["frac_hbm"],
                          "frac_of_measured_ceiling": big[k]["frac_of_measured_ceiling"]}
                      for k in ("scale", "quantize", "metric", "moments")}
    if "ops" in out:
        line["layer_gemm_tflops"] = out["ops"]["layer_tflops"]       # product / formats / step sizes -> TFLOP/s of one layer
        a = out["attention"]
        line["attention"] = {k: {"ms": v["ms"], "GBps": v["GBps"], "frac_hbm": v["frac_hbm"]} for k, v in a.items() if k != "what"}
    if "int8" in out:
        line["int8_passes"] = {k: v["frac_hbm"] for k, v in out["int8"]["passes"].items()}
    line["fused_nsr_ms"] = {"gemm_nsr": r["fused_nsr"]["gemm_nsr"], "gemm_then_metric": r["fused_nsr"]["gemm_then_metric"]}
    line["nsr"] = {k: round(v, 6) for k, v in out["nsr"].items()}
    line["detail"] = "gpurun_out/bench_detail.json (every table; --full prints it instead)"
    line["cpu_baseline"] = out["cpu_baseline"]
    return line


def ops_table(torch, qmm, W, state, ops, cfg_no, back_to_back_ms, dev):
    """Every product of the layer as the GEMM alone (codes in, bf16 out, 10 launches back to back per event pair):
    forward Y = X W^T, dgrad dX = dY W, wgrad dW^T = dY^T X (both operands contract over the token axis: codes from the
    transposing quantize); E4M3 with E5M2 gradients, and INT8; one step size per tensor / per channel."""
    rows = []
    for st in state:
        op = st["op"]
        dy = W.upstream_gradient(op, cfg_no).to(dev)
        wt = st["w"].t().contiguous()
        products = {"fwd": ((st["x"], 1), (st["w"], 1), False), "dgrad": ((dy, 1), (wt, 1), True), "wgrad": ((dy, 0), (st["x"], 0), True)}
        for pname, ((a, a_axis), (b, b_axis), a_is_grad) in products.items():
            for family in ("e4m3", "int8"):
                fa = qmm.INT8 if family == "int8" else (qmm.E5M2 if a_is_grad else qmm.E4M3)
                fb = qmm.INT8 if family == "int8" else qmm.E4M3
                for per_channel in (False, True):
                    (ca, oa), _ = qmm.quantized_operand(a, a_axis, fa, per_channel)
                    (cb, ob), _ = qmm.quantized_operand(b, b_axis, fb, per_channel)
                    M, K = ca.shape[1:]; N = cb.shape[1]
                    y = torch.empty((1, M, N), dtype=torch.bfloat16, device=dev)
                    ms = back_to_back_ms(lambda k: qmm.gemm((ca, oa), (cb, ob), out=y))
                    tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
                    rows.append({"op": op.name, "product": pname, "M": M, "N": N, "K": K,
                                 "formats": ("int8" if family == "int8" else ("e5m2xe4m3" if a_is_grad else "e4m3")),
                                 "step_sizes": "channel" if per_channel else "tensor", "ms": round(ms, 4),
                                 "tflops": round(tf, 1), "frac_mfma_peak": round(tf / 5000.0, 4)})
                    del ca, cb, y
        del dy, wt
    agg = {}
    for r in rows:
        key = f"{r['product']}/{r['formats']}/{r['step_sizes']}"
        a = agg.setdefault(key, [0.0, 0.0])
        a[0] += 2.0 * r["M"] * r["N"] * r["K"]; a[1] += r["ms"]
    # compact: one list per product (the JSON line stays a few KB)
    return {"what": "GEMM alone per product of one BERT-large layer, codes in, bf16 out, 10 launches back to back per event pair; "
                    "rows = [op, product, formats, step sizes, ms, TFLOP/s, fraction of 5.0 PFLOP/s]",
            "rows": [[r["op"], r["product"], r["formats"], r["step_sizes"], r["ms"], r["tflops"], r["frac_mfma_peak"]] for r in rows],
            "layer_tflops": {k: round(v[0] / (v[1] * 1e-3) / 1e12, 1) for k, v in agg.items()}}


def attention_products(torch, qmm, W, back_to_back_ms, dev):
    """BERT-large attention (32 examples x 16 heads, sequence 512, head dimension 64), E4M3 with one step size per head:
    Q K^T (512 matrices of 512 x 512 x 64) and P V (512 x 64 x 512).  Both are bound by their operand and output
    streams, not by the matrix units: GB/s of codes in + Y out against 8 TB/s."""
    batch, heads, seq, dim = 32, 16, 512, 64
    q, k, v = W.attention_operands(batch, heads, seq, dim)
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    (cq, oq), _ = qmm.quantized_operand(qd, 1, qmm.E4M3, False, heads)
    (ck, ok), _ = qmm.quantized_operand(kd, 1, qmm.E4M3, False, heads)
    p = W.softmax_probabilities(qmm.reference_gemm(qd, kd), dim).contiguous()
    (cp, op_), _ = qmm.quantized_operand(p, 1, qmm.E4M3, False, heads)
    (cv, ov), _ = qmm.quantized_operand(vd, 0, qmm.E4M3, False, heads)
    res = {"what": "GEMM alone, codes in, 10 launches back to back per event pair; bytes = codes of both operands + Y"}
    nb = batch * heads
    for name, a, b, m, n, kk, dts in (("qk_t", (cq, oq), (ck, ok), seq, seq, dim, (torch.bfloat16, torch.float32)),
                                      ("p_v", (cp, op_), (cv, ov), seq, dim, seq, (torch.bfloat16,))):
        for dt in dts:
            y = torch.empty((nb, m, n), dtype=dt, device=dev)
            ms = back_to_back_ms(lambda i: qmm.gemm(a, b, out=y))
            nbytes = nb * ((m + n) * kk + m * n * y.element_size())
            res[f"{name}_{'bf16' if dt == torch.bfloat16 else 'f32'}_out"] = {
                "ms": round(ms, 4), "bytes": nbytes, "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                "frac_hbm": round(nbytes / (ms * 1e-3) / 1e9 / 8000.0, 4),
                "tflops": round(2.0 * nb * m * n * kk / (ms * 1e-3) / 1e12, 1)}
            del y
    return res


def cpu_baseline(state, fmt_name, rows_per_op=8192):
    """Time the oracle (as it stands) on `rows_per_op` seeded rows of every op: scale and quantize of those rows of X
    and of all of W, the product of those rows with all of W, descale and metric."""
    import numpy as np
    import torch
    from oracle import oracle as O
    fmt = O.FORMATS[fmt_name]
    O.lib()
    flops = 0
    t0 = time.perf_counter()
    for st in state:
        op = st["op"]
        rng = np.random.default_rng(op.M + op.N)
        rows = np.sort(rng.choice(op.M, size=min(rows_per_op, op.M), replace=False))
        xs = st["host_x"][torch.from_numpy(rows)].float().numpy()
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


if __name__ == "__main__":
    main()
