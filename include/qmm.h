/*
 * qmm.h -- C ABI of the MI355X (gfx950) quantized-matmul library.
 *
 * The library implements the hot path of "A Metric Driven Approach to Mixed
 * Precision Training" (arXiv 2408.02897): for one matrix multiply,
 *   qmm_scale     step size delta = max|X| / qmax per scale group   (Eq. 1, right half)
 *   qmm_quantize  codes = round(X / delta) onto INT8 / E4M3 / E5M2  (Eq. 1, left half;
 *                 Methodology bullets on saturation, underflow and rounding)
 *   qmm_gemm      8-bit x 8-bit product in a wide accumulator, then
 *                 descale by deltaL * deltaR                        (Methodology, scaling bullet)
 *   qmm_metric    error sums of the result against the high-precision
 *                 product: noise-to-signal ratio, Eq. 2, Eq. 3      (Results, Eq. 2 and Eq. 3)
 *
 * General rules
 *  - Every pointer named "device" is GPU memory owned by the caller; the
 *    library allocates nothing and frees nothing.  What it keeps between calls:
 *    per GPU, the addresses of two arrays of its own device image (the scratch
 *    of qmm_scale_static, and a ring of arrival counters that the single-launch
 *    reductions of qmm_scale / qmm_scale_multi use and leave at zero; a call
 *    takes the next slot of the ring, 1024 calls would have to be in flight for
 *    two of them to meet on one), and which GPUs have had the kernels' LDS limit set.
 *    Descriptor structs (qmm_tensor, qmm_operand, qmm_granularity) are host memory
 *    and are read before the call returns.
 *  - Calls validate their arguments on the host, enqueue kernels on `stream`
 *    (a hipStream_t passed as void*; NULL = the default stream) and return
 *    without synchronising.  Results stay on the device.
 *  - Argument errors are reported before anything is launched and leave the
 *    outputs untouched.  A launch failure returns QMM_ERR_LAUNCH.
 *  - NaN / inf inputs and all-zero groups are not errors; their results are
 *    defined below.
 *  - Arithmetic is IEEE binary32 unless stated, round-to-nearest-even,
 *    subnormals kept.
 *
 * Scale groups.  A tensor is a batch of matrices [batch][rows][cols].  Matrix b
 * belongs to batch group g = (b / batch_inner) % batch_groups (batch_groups = 1:
 * one group for the whole batch, "tensor"/"channel" level; batch_groups = H with
 * the batch laid out [example][head]: one group per head, shared by the
 * examples -- the fine-grained level of the Results section, which adds batch
 * dimensions other than the examples' to the scale's index).  With the batch
 * laid out [outer][mid][inner], batch_groups = mid and batch_inner = inner give
 * one group per index of the middle dimensions, shared over outer and inner:
 * any run of neighbouring batch dimensions can carry the scales.  With
 * per_channel = 1 every index c of the non-contracting axis has its own step
 * size, shared by the matrices of the group: delta[g * C + c], C = extent of
 * the non-contracting axis.  With per_channel = 0: delta[g].
 */
#ifndef QMM_H
#define QMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QMM_OK = 0,
    QMM_ERR_NULL = 1,        /* a required pointer is NULL                        */
    QMM_ERR_SHAPE = 2,       /* negative extent, stride smaller than extent, ...  */
    QMM_ERR_ENUM = 3,        /* unknown format / dtype / rounding / axis value    */
    QMM_ERR_ALIGN = 4,       /* pointer or extent alignment rule violated         */
    QMM_ERR_UNSUPPORTED = 5, /* valid request this build does not implement       */
    QMM_ERR_WORKSPACE = 6,   /* workspace missing or too small                    */
    QMM_ERR_LAUNCH = 7,      /* the HIP runtime refused a launch                  */
    QMM_ERR_LIMIT = 8        /* input larger than a fixed, documented capacity    */
} qmm_status;

/* 8-bit formats of the paper, plus the un-quantized pass-through used for the
 * high-precision reference product.  Largest magnitudes: 127, 448, 57344. */
typedef enum { QMM_FMT_INT8 = 0, QMM_FMT_E4M3 = 1, QMM_FMT_E5M2 = 2, QMM_FMT_BF16 = 3 } qmm_format;
typedef enum { QMM_DT_BF16 = 0, QMM_DT_F32 = 1 } qmm_dtype;
typedef enum { QMM_ROUND_RTNE = 0, QMM_ROUND_STOCHASTIC = 1 } qmm_round;

/* A batch of row-major matrices in device memory.  Element (b, r, c) is at
 * data[b*batch_stride + r*row_stride + c] (strides in elements, columns are
 * contiguous).  contract_axis names the axis the matrix multiply sums over:
 * 1 = columns (an [M][K] operand), 0 = rows (a [K][M] operand, e.g. the
 * activations and the upstream gradient in a weight-gradient product). */
typedef struct {
    const void* data;        /* device */
    int32_t dtype;           /* qmm_dtype */
    int32_t contract_axis;   /* 0 or 1 */
    int64_t batch, rows, cols;
    int64_t batch_stride, row_stride;
} qmm_tensor;

typedef struct {
    int32_t per_channel;     /* 0: one step size per batch group; 1: one per non-contracting index */
    int32_t batch_inner;     /* >= 0; 0 means 1: consecutive matrices that share a group            */
    int64_t batch_groups;    /* >= 1: group = (b / batch_inner) % batch_groups                      */
} qmm_granularity;

/* Number of step sizes qmm_scale writes / qmm_quantize reads for this tensor. */
int64_t qmm_num_scales(const qmm_tensor* x, const qmm_granularity* g);

/*
 * Step 1 -- step size (Eq. 1: delta = max|X| / (2^(n-1)-1); for FP8 the
 * denominator is the format maximum, last Methodology bullet).
 *   delta_out  device, qmm_num_scales() floats.
 *   workspace  device scratch of at least qmm_scale_workspace_size() bytes,
 *              16-byte aligned; contents on entry are irrelevant.
 * Defined results: the maximum is taken over magnitude bit patterns, so an
 * inf or NaN element makes its group's delta inf / NaN; an all-zero (or
 * empty) group gets delta = 1; a quotient below 2^-126 is raised to 2^-126.
 * fmt must be one of the three 8-bit formats.  batch above 65535: QMM_ERR_UNSUPPORTED.
 */
size_t qmm_scale_workspace_size(const qmm_tensor* x, const qmm_granularity* g);
qmm_status qmm_scale(const qmm_tensor* x, qmm_format fmt, const qmm_granularity* g,
                     float* delta_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * qmm_scale_static -- qmm_scale for callers that cannot allocate device memory or hand over a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same arguments, results and errors as
 * qmm_scale without the workspace: the partial maxima go to a scratch array of QMM_SCALE_STATIC_BYTES that is part
 * of the library's device image (one copy per GPU, held until the process ends; its address is looked up once per
 * device on the first call there).  The call allocates and frees nothing.
 *   Limit: qmm_scale_workspace_size(x, g) must not exceed QMM_SCALE_STATIC_BYTES, else QMM_ERR_LIMIT (checked on
 *   the host before anything is launched; 1 MiB covers one step size per tensor for any size, and e.g. one step
 *   size per row for 262144 rows).
 *   Nothing in the array has to be cleared between calls (every word read by the second kernel has been written by
 *   the first of the same call), but all calls on one GPU share it: calls that may overlap on one GPU -- different
 *   streams, or graphs replayed concurrently -- race on it and must be serialised by the caller.
 */
#define QMM_SCALE_STATIC_BYTES (1u << 20)
qmm_status qmm_scale_static(const qmm_tensor* x, qmm_format fmt, const qmm_granularity* g,
                            float* delta_out, void* stream);

/*
 * Step 2 -- quantize (Eq. 1: code = round(X / delta)).  The quotient is formed
 * as t = fl(x * fl(1/delta)): one correctly rounded reciprocal per group, one
 * correctly rounded product per element.
 *   INT8: round half to even, keep [-127, 127], two's complement byte; NaN -> 0.
 *   E4M3 / E5M2 (OCP FP8 value sets): nearest finite value, ties to the even
 *   mantissa, |t| above the maximum (and inf) -> +-maximum, sign of t kept
 *   (negative underflow -> 0x80), NaN -> 0x7F.
 *   QMM_ROUND_STOCHASTIC: with lo <= |t| < hi the neighbouring grid values, the
 *   result is hi iff u < (|t|-lo)/(hi-lo), u = (24 random bits)/2^24.  The bits
 *   of output element p (linear index in codes_out) are the top 24 bits of word
 *   (p+offset)%4 of Philox4x32-10 with counter ((p+offset)/4, 0) as two 32-bit
 *   halves followed by two zero words, and key = seed as two 32-bit halves, so
 *   a tensor quantized in pieces with matching offsets equals the whole.
 *   codes_out  device, [batch][non-contracting][contracting] bytes, dense: the
 *              contracting axis is contiguous whatever contract_axis is.
 *   delta      device, as written by qmm_scale (or supplied by the caller).
 * Uses no workspace.  batch above 65535: QMM_ERR_UNSUPPORTED.
 */
qmm_status qmm_quantize(const qmm_tensor* x, qmm_format fmt, const qmm_granularity* g,
                        const float* delta, qmm_round mode, uint64_t seed, uint64_t offset,
                        uint8_t* codes_out, void* stream);

/*
 * qmm_scale_multi / qmm_quantize_multi -- steps 1 and 2 (Eq. 1) for `count` tensors in one call each, e.g. the
 * activations and the weights of one product: the results are those of `count` calls of qmm_scale / qmm_quantize.
 *   x, g        host arrays of `count` descriptors / granularities.
 *   delta_out, delta, codes_out   host arrays of `count` device pointers, each as the single-tensor call takes it.
 *   offsets     host array of `count` stream offsets for stochastic rounding, or NULL for zeros.
 *   workspace   device scratch, qmm_scale_multi_workspace_size() bytes (the tensors' own sizes, each rounded up to 16),
 *               16-byte aligned.
 * When all tensors (at most 8) are single dense bfloat16 matrices in 16-byte aligned whole vectors with one step size
 * each (and, for quantize: contract_axis 1, cols a multiple of 16, round to nearest even), each call is one launch
 * (for scale too: each tensor's workgroup that finishes last folds its partial maxima) with the tensor index as a grid dimension, so that the
 * small tensors' latency-bound kernels run inside the large tensors' launches.  Otherwise the tensors are processed
 * one after the other by the single-tensor code, after every tensor's arguments have been checked (an argument
 * error in any of them is returned before anything is launched).  Errors as for the single-tensor calls; count = 0
 * is a no-op, count < 0 QMM_ERR_SHAPE.
 */
size_t qmm_scale_multi_workspace_size(int32_t count, const qmm_tensor* x, const qmm_granularity* g);
qmm_status qmm_scale_multi(int32_t count, const qmm_tensor* x, qmm_format fmt, const qmm_granularity* g,
                           float* const* delta_out, void* workspace, size_t workspace_bytes, void* stream);
qmm_status qmm_quantize_multi(int32_t count, const qmm_tensor* x, qmm_format fmt, const qmm_granularity* g,
                              const float* const* delta, qmm_round mode, uint64_t seed, const uint64_t* offsets,
                              uint8_t* const* codes_out, void* stream);

/* One operand of qmm_gemm: a dense batch [batch][rows][K] with K contiguous. */
typedef struct {
    const void* data;        /* device; 8-bit codes, or bfloat16 values (see is_codes)          */
    int32_t format;          /* qmm_format the operand is multiplied in                          */
    int32_t is_codes;        /* 1: data holds 8-bit codes of `format`.
                                0: data holds bfloat16; with an 8-bit `format` the values are
                                   quantized with `delta` (RTNE) while they are staged for the
                                   multiply; with QMM_FMT_BF16 they are multiplied as they are. */
    const float* delta;      /* device step sizes (ignored for QMM_FMT_BF16)                     */
    qmm_granularity gran;    /* how delta is indexed; per_channel refers to the operand's rows   */
} qmm_operand;

/*
 * Steps 3 and 4 -- Y[b][i][j] = (acc * deltaA[i]) * deltaB[j],
 * acc = sum_k value(A[b][i][k]) * value(B[b][j][k])   (third Methodology bullet:
 * scaling before and after the multiply, result held in a wider accumulator).
 *   INT8 x INT8 accumulates exactly in int32 (|acc| must stay below 2^31);
 *   FP8 x FP8 (E4M3 and E5M2 may be mixed) accumulates in binary32; the
 *   summation order is unspecified;  BF16 x BF16 accumulates in binary32 and
 *   is not descaled (the high-precision reference product).
 *   Both operands must be 8-bit formats of the same family (both INT8 or both
 *   FP8) or both BF16.  INT8 code 0x80 (-128) is outside the format: undefined.
 *   y          device [batch][M][N], y_dtype F32 or BF16 (RNE).  May be NULL if
 *              acc_out is given.
 *   acc_out    device [batch][M][N] raw accumulators (int32 for INT8, else
 *              binary32) or NULL.
 *   K must be a multiple of 16 bytes' worth of elements (16 codes / 8 bf16)
 *   and all data pointers 16-byte aligned, else QMM_ERR_ALIGN.
 *   K in bytes (K codes, or 2 K for BF16) must not exceed 2^22, else
 *   QMM_ERR_UNSUPPORTED.
 *   workspace  device scratch of at least qmm_gemm_workspace_size() bytes,
 *              16-byte aligned (may be 0, then NULL is accepted).  It is non-zero
 *              for small outputs with a long K (weight-gradient shapes): K is
 *              then split into ranges whose partial accumulators are kept there
 *              and added in ascending order by a second kernel, so results do
 *              not depend on timing.  Too small: QMM_ERR_WORKSPACE.
 */
size_t qmm_gemm_workspace_size(const qmm_operand* a, const qmm_operand* b,
                               int64_t batch, int64_t M, int64_t N, int64_t K);
qmm_status qmm_gemm(const qmm_operand* a, const qmm_operand* b,
                    int64_t batch, int64_t M, int64_t N, int64_t K,
                    void* y, qmm_dtype y_dtype, void* acc_out,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * qmm_gemm_nsr -- qmm_gemm with the noise-to-signal sums taken in its epilogue (the error metric the path reduces
 * for every op, here without a second pass over Y; an extension: the paper measures, it does not say where).
 * Computes Y exactly as qmm_gemm does and, over the values it stores (rounded to y_dtype),
 *     out2[0] = sum (y - y_ref)^2      out2[1] = sum y_ref^2
 * in binary64, elements whose error is NaN left out of both sums -- fields 0 and 1 of qmm_metric(Y, y_ref).  The
 * order of additions is fixed by the shapes (per-wavefront sums folded by a second kernel), so results are
 * reproducible run to run; it differs from qmm_metric's order, so the sums agree with it to rounding only.
 *   a, b       8-bit operands given as codes (is_codes = 1); BF16 and quantize-on-load operands: QMM_ERR_UNSUPPORTED.
 *   y          device [batch][M][N], required.      y_ref  device [batch][M][N] binary32, 16-byte aligned.
 *   out2       device, 2 doubles, 8-byte aligned.
 *   workspace  device scratch of at least qmm_gemm_nsr_workspace_size() bytes, 16-byte aligned: QMM_ERR_WORKSPACE
 *              if missing or too small.  K is never split here.
 * Other argument rules and errors as for qmm_gemm.  An empty output writes two zeros.
 */
size_t qmm_gemm_nsr_workspace_size(int64_t batch, int64_t M, int64_t N);
qmm_status qmm_gemm_nsr(const qmm_operand* a, const qmm_operand* b,
                        int64_t batch, int64_t M, int64_t N, int64_t K,
                        void* y, qmm_dtype y_dtype, const float* y_ref, double* out2,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Step 6 -- error metrics of y against the high-precision result y_ref, one
 * pass, binary64 accumulation, e = y - y_ref.  out16 (device, 16 doubles):
 *   [0] sum e^2          [1] sum ref^2        (noise-to-signal ratio = [0]/[1])
 *   [2] sum |e|          [3] sum |ref|
 *   [4] max |e|          [5] max |ref|
 *   [6] sum over ref != 0 of |e|/|ref|   [7] its max   [8] its term count   (Eq. 2)
 *   [9] sum over d > 0 of |e|/d          [10] its max  [11] its term count  (Eq. 3, element-wise;
 *        d = (|L|.|R|)_ij supplied by the caller in denom, or NULL: [9..11] = 0)
 *   [12] elements counted   [13] elements skipped because e is NaN   [14],[15] = 0
 * Elements whose error is NaN are left out of every sum and maximum.
 *   y          device, n elements of y_dtype;  y_ref, denom: device, n floats.
 *   workspace  device scratch, qmm_metric_workspace_size(n) bytes, 16-byte aligned.
 * n = 0 writes sixteen zeros.
 */
size_t qmm_metric_workspace_size(int64_t n);
qmm_status qmm_metric(const void* y, qmm_dtype y_dtype, const float* y_ref, const float* denom,
                      int64_t n, double* out16, void* workspace, size_t workspace_bytes, void* stream);

/*
 * qmm_dequantize -- the reduced-precision value of every quantized element (the v-tilde of Eq. 2), for looking at
 * the quantization error of a tensor itself rather than of a product:
 *     out[b][r][k] = fl32( value(codes[b][r][k]) * delta[group(b) * C + (per_channel ? r : 0)] )
 * with codes and delta exactly as qmm_quantize takes / writes them (C = rows if per_channel, else 1); the code's
 * value is exact in binary32, so this is one rounding; bfloat16 output rounds that once more (RNE).
 * An FP8 NaN code gives NaN, an E5M2 infinity code gives infinity, the INT8 code 0x80 gives -128 delta.
 *   codes  device [batch][rows][K] uint8;  out  device [batch][rows][K] of out_dtype; caller-owned.
 * Asynchronous on `stream`, uses no workspace.  Empty tensors return QMM_OK.
 * Errors: QMM_ERR_NULL, QMM_ERR_ENUM, QMM_ERR_SHAPE, QMM_ERR_ALIGN (out not aligned to its element), QMM_ERR_LAUNCH.
 */
qmm_status qmm_dequantize(const uint8_t* codes, int64_t batch, int64_t rows, int64_t K, qmm_format fmt,
                          const qmm_granularity* g, const float* delta, void* out, qmm_dtype out_dtype, void* stream);

/*
 * qmm_moments -- statistics of a tensor the method looks at before choosing a format (Results section, first
 * paragraph: mean, variance, skew and kurtosis of the matrix-multiply inputs).  Estimators (the paper names none):
 * population moments about the mean,  mean = sum x / n,  m_k = sum (x - mean)^k / n  for k = 2, 3, 4;
 * skew = m3 / m2^1.5 and kurtosis = m4 / m2^2 (3 for a normal distribution) are left to the caller.
 *   x        device, n contiguous elements (bfloat16 or binary32), 16-byte aligned; not modified
 *   center   finite value the power sums are taken about in the single pass over x (binary64).  0 is right for
 *            tensors whose mean lies within a few standard deviations of 0; otherwise pass an estimate of the
 *            mean: the relative error of m_k grows like (1 + ((mean - center) / sigma)^2)^(k/2) * 1e-15.
 *   out8     device, 8 doubles: n (non-NaN count), mean, m2, m3, m4, max |x|, NaN count, 0.
 *            NaN elements are counted and otherwise ignored; n = 0 gives zeros.  Infinite elements propagate.
 *   workspace  device scratch, qmm_moments_workspace_size(n) bytes, 16-byte aligned.
 * Asynchronous on `stream`; deterministic (fixed order of additions for a given n).
 * Errors: QMM_ERR_NULL, QMM_ERR_ENUM, QMM_ERR_SHAPE (n < 0 or center not finite), QMM_ERR_ALIGN,
 * QMM_ERR_WORKSPACE, QMM_ERR_LAUNCH.
 */
size_t qmm_moments_workspace_size(int64_t n);
qmm_status qmm_moments(const void* x, qmm_dtype dtype, int64_t n, double center, double* out8,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * qmm_mfma_rate -- measurement aid, not a step of the method: the rate the matrix units sustain on given operand
 * bytes with no memory traffic, against which the GEMM's rate is read (next to the datasheet peak, which is quoted
 * at the top clock; under matrix load the clock is set by power, and that depends on the operand bytes).
 *   operand_bytes device, 32-byte aligned, nbytes >= 32: 8-bit codes in the given formats (e.g. the codes
 *                 qmm_quantize wrote); every lane takes ten fragments from it.  Not modified.
 *   rounds        every wavefront issues rounds * 64 (FP8) or rounds * 16 (INT8) matrix instructions
 *   workgroups    number of workgroups of four wavefronts (one per CU fills the chip)
 *   sink          device, workgroups * 256 floats, written (keeps the work alive); caller-owned
 *   flops_out     host: operations the launch performs (2 per multiply-add)
 * Asynchronous on `stream`; the caller times it.  Formats: both INT8, or any pair of E4M3 / E5M2.
 * Errors: QMM_ERR_NULL, QMM_ERR_ENUM, QMM_ERR_UNSUPPORTED, QMM_ERR_SHAPE, QMM_ERR_ALIGN, QMM_ERR_LAUNCH.
 */
qmm_status qmm_mfma_rate(qmm_format a_format, qmm_format b_format, const void* operand_bytes, int64_t nbytes,
                         int64_t rounds, int32_t workgroups, float* sink, double* flops_out, void* stream);

/*
 * qmm_hbm_rate -- measurement aid, not a step of the method: a plain streaming kernel over `nbytes` of device memory,
 * the ceiling the memory-bound passes (steps 1, 2 and 6) are read against next to the datasheet bandwidth.
 *   src     device, nbytes (a multiple of 16), 16-byte aligned; read once with streaming loads
 *   dst     device, nbytes, 16-byte aligned: the bytes are copied there; or NULL: read only, folded into `sink`
 *   sink    device, workgroups * 256 words, written when dst is NULL (keeps the loads alive); caller-owned
 *   workgroups  grid size (1024 = four workgroups per CU, as the passes use)
 * Asynchronous on `stream`; the caller times it and rotates buffers larger than the caches.
 * Errors: QMM_ERR_NULL, QMM_ERR_SHAPE, QMM_ERR_ALIGN, QMM_ERR_LAUNCH.
 */
qmm_status qmm_hbm_rate(const void* src, void* dst, int64_t nbytes, int32_t workgroups, uint32_t* sink, void* stream);

const char* qmm_status_string(qmm_status s);
/* Version of this ABI (major*100 + minor). */
int qmm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QMM_H */
