"""HBM traffic of the GEMM launches of bench.py's step from rocprofv3 counter files -> profiles/gemm_traffic.json.

The counters FETCH_SIZE and WRITE_SIZE (KiB per dispatch, one rocprofv3 --pmc run each: the tool does not split
counters over passes) are scaled by what the same counter reads for a plain device copy of known size
(`bench.py --copy-calibration`), then averaged per op over the dispatches of `bench.py --no-extras --format F`, whose
only quantized-GEMM launches are the four of each step, in the order QKV, attn_out, FFN1, FFN2.

    python -m paper_2408_02897_amd.traffic --format e4m3 --fetch DIR --write DIR --copy-fetch DIR --copy-write DIR
                                           [--workload bert_large_fwd] [--out profiles/gemm_traffic.json]

DIR = the -d directory given to rocprofv3 (searched recursively for *counter_collection.csv).  The entry of the given
workload / format in the JSON file is replaced, the others are kept.  bench.py reads the file for `roofline.traffic`.
"""
import argparse
import csv
import glob
import json
import os

from . import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_BYTES = 256 << 20


def _rows(directory, counter):
    out = []
    for f in sorted(glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)):
        with open(f, newline="") as fh:
            for i, r in enumerate(csv.DictReader(fh)):
                if r.get("Counter_Name") == counter:
                    out.append((int(r.get("Dispatch_Id", i)), r["Kernel_Name"], float(r["Counter_Value"])))
    out.sort()
    return out


def _copy_factor(directory, counter):
    vals = [v for _, name, v in _rows(directory, counter) if "copyBuffer" in name]
    if not vals:
        raise SystemExit(f"no copy kernel dispatches with {counter} under {directory}")
    return COPY_BYTES / 1024.0 / (sum(vals) / len(vals))


def _is_quantized_gemm(name):
    if "gemm_" not in name or "splitk_reduce" in name:
        return False
    return not any(tag in name for tag in ("gemm_kernel<2,", "gemm_direct_kernel<2,", "gemm_shortk_kernel<2,"))   # KIND 2 = bf16 reference


def per_op_bytes(directory, counter, factor, n_ops):
    vals = [v * 1024.0 * factor for _, name, v in _rows(directory, counter) if _is_quantized_gemm(name)]
    if not vals or len(vals) % n_ops:
        raise SystemExit(f"{len(vals)} quantized GEMM dispatches under {directory}: not a multiple of {n_ops}")
    return [sum(vals[i::n_ops]) / len(vals[i::n_ops]) for i in range(n_ops)]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--format", required=True, choices=["e4m3", "e5m2", "int8"])
    ap.add_argument("--workload", default="bert_large_fwd", choices=["bert_large_fwd", "bert_base_fwd"])
    ap.add_argument("--fetch", required=True); ap.add_argument("--write", required=True)
    ap.add_argument("--copy-fetch", required=True); ap.add_argument("--copy-write", required=True)
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles", "gemm_traffic.json"))
    a = ap.parse_args()
    ops = W.bert_forward_ops(**(W.BERT_LARGE if a.workload == "bert_large_fwd" else W.BERT_BASE))
    ff, fw = _copy_factor(a.copy_fetch, "FETCH_SIZE"), _copy_factor(a.copy_write, "WRITE_SIZE")
    rd = per_op_bytes(a.fetch, "FETCH_SIZE", ff, len(ops))
    wr = per_op_bytes(a.write, "WRITE_SIZE", fw, len(ops))
    algo_rd = [(op.M + op.N) * op.K for op in ops]
    algo_wr = [2 * op.M * op.N for op in ops]
    entry = {"what": "HBM bytes per GEMM launch (mean over the step's four launches) by rocprofv3 FETCH_SIZE / WRITE_SIZE, "
                     "each scaled by the same counter's reading for a plain 256 MiB device copy",
             "counter_scale": {"FETCH_SIZE": round(ff, 4), "WRITE_SIZE": round(fw, 4)},
             "read_bytes": round(sum(rd) / len(ops)), "write_bytes": round(sum(wr) / len(ops)),
             "algorithmic_read_bytes": round(sum(algo_rd) / len(ops)), "algorithmic_write_bytes": round(sum(algo_wr) / len(ops)),
             "reread_ratio": round(sum(rd) / sum(algo_rd), 3),
             "per_op": {op.name: {"read_bytes": round(r), "write_bytes": round(w), "algorithmic_read_bytes": ar,
                                  "algorithmic_write_bytes": aw, "reread_ratio": round(r / ar, 3)}
                        for op, r, w, ar, aw in zip(ops, rd, wr, algo_rd, algo_wr)}}
    table = {}
    if os.path.exists(a.out):
        with open(a.out) as f:
            table = json.load(f)
    table[f"{a.workload}/{a.format}"] = entry
    with open(a.out, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")
    print(json.dumps(entry))


if __name__ == "__main__":
    main()
