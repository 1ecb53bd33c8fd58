"""MI355X-native quantized matrix multiply with per-op error metrics (arXiv 2408.02897).

`paper_2408_02897_amd.qmm` binds the C-ABI HIP library (qmm_scale, qmm_quantize, qmm_gemm,
qmm_metric); `paper_2408_02897_amd.workloads` draws the seeded synthetic inputs.  Importing
the package loads nothing native; the library is opened on first use of `qmm` and its
absence is an error, never a fallback.
"""
__all__ = ["qmm", "workloads"]
