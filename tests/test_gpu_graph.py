"""The hot path recorded once as a HIP graph and replayed: every replay must give what the eager calls give on the same
inputs.  What this guards: the library's own arrays (the ring of arrival counters of the single-launch step-size
reductions) are left at zero by every call, so a recorded call can run any number of times; nothing in a call depends
on values a previous call left in a workspace; no call allocates.  The inputs change between replays (written into
the recorded buffers), the program's own eager calls and synchronisations run in between, and three replays are
checked, not one.  Eq. 1 (scale, quantize), the Methodology's 8-bit product and descale, the error sums of the Results
section: one product with the large-tensor single-launch qmm_scale, one with the several-tensors calls."""
import pytest
import torch

from paper_2408_02897_amd import qmm, workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _buffers(M, N, K, fmt):
    b = {"x": torch.empty((1, M, K), dtype=torch.bfloat16, device=DEV), "w": torch.empty((1, N, K), dtype=torch.bfloat16, device=DEV),
         "dx": torch.empty(1, device=DEV), "dw": torch.empty(1, device=DEV),
         "cx": torch.empty((1, M, K), dtype=torch.uint8, device=DEV), "cw": torch.empty((1, N, K), dtype=torch.uint8, device=DEV),
         "y": torch.empty((1, M, N), dtype=torch.bfloat16, device=DEV), "ref": torch.empty((1, M, N), dtype=torch.float32, device=DEV),
         "m": torch.empty(16, dtype=torch.float64, device=DEV), "ws": torch.empty(1 << 20, dtype=torch.uint8, device=DEV)}
    b["oa"] = qmm.operand(b["cx"], fmt, b["dx"]); b["ob"] = qmm.operand(b["cw"], fmt, b["dw"])
    return b


def _step_single(b, fmt):
    """qmm_scale / qmm_quantize tensor by tensor (x has 2^24 elements: the single-launch reduction)."""
    qmm.scale(b["x"], 1, fmt, out=b["dx"], workspace=b["ws"]); qmm.scale(b["w"], 1, fmt, out=b["dw"], workspace=b["ws"])
    qmm.quantize(b["x"], 1, fmt, b["dx"], out=b["cx"]); qmm.quantize(b["w"], 1, fmt, b["dw"], out=b["cw"])
    qmm.gemm((b["cx"], b["oa"]), (b["cw"], b["ob"]), out=b["y"])
    qmm.metric(b["y"], b["ref"], out=b["m"], workspace=b["ws"])


def _step_multi(b, fmt):
    qmm.scale_multi(b["xw"], fmt, outs=[b["dx"], b["dw"]], workspace=b["ws"], out_ptrs=b["dp"])
    qmm.quantize_multi(b["xw"], fmt, [b["dx"], b["dw"]], outs=[b["cx"], b["cw"]], delta_ptrs=b["dp"], out_ptrs=b["cp"])
    qmm.gemm((b["cx"], b["oa"]), (b["cw"], b["ob"]), out=b["y"])
    qmm.metric(b["y"], b["ref"], out=b["m"], workspace=b["ws"])


@pytest.mark.parametrize("kind,fmt", [("single", qmm.E4M3), ("multi", qmm.E4M3), ("multi", qmm.INT8)])
def test_recorded_step_replays_like_eager(kind, fmt):
    M, N, K = (4096, 512, 4096) if kind == "single" else (2048, 768, 1024)
    rec, eag = _buffers(M, N, K, fmt), _buffers(M, N, K, fmt)
    for b in (rec, eag):
        b["xw"] = qmm.MultiDesc([b["x"], b["w"]])
        b["dp"] = qmm.MultiDesc.pointers([b["dx"], b["dw"]]); b["cp"] = qmm.MultiDesc.pointers([b["cx"], b["cw"]])
    step = _step_single if kind == "single" else _step_multi

    def load(b, seed):
        b["x"].copy_(W.student_t((1, M, K), 4, seed).to(DEV) * (1.0 + seed % 3)); b["w"].copy_(W.normal((1, N, K), 0.02, seed + 1).to(DEV))
        b["ref"].copy_(qmm.reference_gemm(b["x"], b["w"]))

    load(rec, 100)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                    # first use of every kernel outside the recording
        step(rec, fmt)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(rec, fmt)
    torch.cuda.synchronize()
    for rep, seed in enumerate((200, 300, 400)):
        load(rec, seed); load(eag, seed)
        step(eag, fmt)                                   # the program's own eager work between the replays
        torch.cuda.synchronize()
        for key in ("dx", "dw", "cx", "cw", "y", "m"):   # nothing of the previous replay may survive unnoticed
            rec[key].fill_(0 if key != "m" else -1.0)
        graph.replay()
        torch.cuda.synchronize()
        for key in ("dx", "dw", "cx", "cw", "y"):
            assert torch.equal(rec[key], eag[key]), (rep, key)
        assert torch.equal(rec["m"], eag["m"]), (rep, rec["m"], eag["m"])
