// qmm_metric: one pass over (y, y_ref[, denom]) accumulating in binary64 the
// sums behind the noise-to-signal ratio, the relative error of Eq. 2 and the
// element-wise backward error of Eq. 3.  HBM-bound: 8 B per element for a
// binary32 y (6 B for bfloat16 y, +4 B with denominators).  Every thread keeps
// private sums, wavefronts fold them by shuffles, workgroups through LDS, and a
// small second kernel (one workgroup per field) folds the per-workgroup partials in a fixed order:
// no atomics, so the result is reproducible run to run.
#include <algorithm>
#include "qmm_device.h"

namespace qmm {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxBlocks = 1024;   // 4 workgroups per CU (what 126 registers keep resident); also 4 partials per thread in the final fold
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// Quotients n / d in binary64 for finite n >= 0 and finite d > 0 where d was converted from binary32 (24 significant
// bits) and n is such a value or the difference of two (exponents within +-150 or so).
//
// reciprocals4: the four reciprocals from ONE hardware estimate: p = d0 d1 d2 d3 (within 2^-596 .. 2^512), two Newton
// steps on rcp(p), then multiplied back by the other factors.  Each x[i] is 1 / d[i] to a few 2^-53.
// quotient_with: q0 = n x, r = n - d q0 (exact in one fused multiply-add: d q0 has 77 bits of which all but 25 cancel),
// q = fl(q0 + r x).  q0 + r x differs from n / d by |r / d| * |x d - 1| < 2^-100 relative, and a quotient with a 24-bit
// divisor is either representable or at least 2^-78 relative away from the nearest rounding boundary (n - m d is a
// multiple of 2^(e_m + e_d - 76) for a 54-bit midpoint m), so the single rounding of the last operation lands on the
// IEEE quotient: same bits as `/`, for 7.25 instructions per quotient (one quarter-rate) instead of 11 with the
// compiler's sequence.  (The metric pass is as much ALU- as HBM-bound; the divisions are its largest single cost.)
// A zero, infinite or NaN operand anywhere in the four gives NaN or infinity in the affected quotients, never a wrong
// finite value passed as right for them: the caller tests the quotients and takes the general path then.
QMM_DEV void reciprocals4(const double* d, double* x)
{
    const double p01 = d[0] * d[1], p23 = d[2] * d[3];
    const double p = p01 * p23;
    const double x0 = __builtin_amdgcn_rcp(p);
    const double x1 = fma(x0, fma(-p, x0, 1.0), x0);
    const double x2 = fma(x1, fma(-p, x1, 1.0), x1);
    const double x01 = x2 * p23, x23 = x2 * p01;
    x[0] = x01 * d[1]; x[1] = x01 * d[0]; x[2] = x23 * d[3]; x[3] = x23 * d[2];
}
// m = max(m, |v|) for values that are not NaN, as the one instruction.  (fmax() first quiets each operand that the
// compiler cannot prove canonical -- a converted, negated or loaded value -- with an instruction of its own, which
// doubled the cost of the running maxima.)
QMM_DEV void max_abs_plain(double& m, double v)
{
    asm("v_max_f64 %0, %0, |%1|" : "+v"(m) : "v"(v));
}
QMM_DEV double quotient_with(double n, double d, double x)
{
    const double q0 = n * x;
    return fma(fma(-d, q0, n), x, q0);
}

// Running sums of one thread.  Branch-free: an element whose error is NaN contributes zeros and bumps nan_cnt.
struct Acc {
    double s_ee = 0, s_rr = 0, s_ae = 0, s_ar = 0, m_e = 0, m_r = 0;
    double re_sum = 0, re_max = 0, be_sum = 0, be_max = 0;
    unsigned re_cnt = 0, be_cnt = 0, n = 0, nan_cnt = 0;     // a thread sees far fewer than 2^32 elements

    // The common case, taken when the whole wavefront's elements are ordinary (no NaN or infinite error, r != 0 and
    // d > 0 everywhere): |e|, |r| and the quotients come in computed.  Same sums as add(), without its selects.
    // re_sum and be_sum are taken by the caller (it adds the quotients itself, to test them).
    // e and r come in signed.
    template <bool HAS_D> QMM_DEV void add_plain(double e, double r, double q, double qb)
    {
        const double ae = e, ar = r;
        s_ee = fma(e, e, s_ee);
        s_rr = fma(r, r, s_rr);
        s_ae += fabs(e);
        s_ar += fabs(r);
        max_abs_plain(m_e, ae);
        max_abs_plain(m_r, ar);
        max_abs_plain(re_max, q);
        if constexpr (HAS_D) max_abs_plain(be_max, qb);
    }
    // counts of a run of `k` plain elements
    template <bool HAS_D> QMM_DEV void count_plain(unsigned k)
    {
        re_cnt += k; n += k;
        if constexpr (HAS_D) be_cnt += k;
    }
    template <bool HAS_D> QMM_DEV void add(float yf, float rf, float df)
    {
        const double e = (double)yf - (double)rf;
        const bool ok = (e == e);
        const double ae = ok ? fabs(e) : 0.0;
        const double ar = ok ? fabs((double)rf) : 0.0;
        s_ee = fma(ae, ae, s_ee);
        s_rr = fma(ar, ar, s_rr);
        s_ae += ae;
        s_ar += ar;
        m_e = fmax(m_e, ae);
        m_r = fmax(m_r, ar);
        const bool rnz = ar != 0.0;
        const double q = rnz ? ae / ar : 0.0;                 // Eq. 2 with |v| in the denominator
        re_sum += q;
        re_max = fmax(re_max, q);
        re_cnt += rnz ? 1u : 0u;
        if constexpr (HAS_D) {
            const double d = (double)df;
            const bool dpos = ok && d > 0.0;
            const double qb = dpos ? ae / d : 0.0;            // Eq. 3, element-wise
            be_sum += qb;
            be_max = fmax(be_max, qb);
            be_cnt += dpos ? 1u : 0u;
        }
        n += ok ? 1u : 0u;
        nan_cnt += ok ? 0u : 1u;
    }
};

// Workgroup partials are stored field-major: partial[field * nblocks + block].
QMM_DEV void store_partial(const Acc& a, double* partial, int nblocks)
{
    __shared__ double s[kThreads / kWave][16];
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
    double v[16];
    v[0] = wave_sum_f64(a.s_ee); v[1] = wave_sum_f64(a.s_rr); v[2] = wave_sum_f64(a.s_ae); v[3] = wave_sum_f64(a.s_ar);
    v[4] = wave_max_f64(a.m_e); v[5] = wave_max_f64(a.m_r);
    v[6] = wave_sum_f64(a.re_sum); v[7] = wave_max_f64(a.re_max); v[8] = wave_sum_f64((double)a.re_cnt);
    v[9] = wave_sum_f64(a.be_sum); v[10] = wave_max_f64(a.be_max); v[11] = wave_sum_f64((double)a.be_cnt);
    v[12] = wave_sum_f64((double)a.n); v[13] = wave_sum_f64((double)a.nan_cnt);
    v[14] = 0.0; v[15] = 0.0;
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < 16; ++i) s[w][i] = v[i];
    }
    __syncthreads();
    if (threadIdx.x < 16) {
        const int i = threadIdx.x;
        const bool is_max = (i == 4 || i == 5 || i == 7 || i == 10);
        double r = s[0][i];
        for (int k = 1; k < kThreads / kWave; ++k) r = is_max ? fmax(r, s[k][i]) : r + s[k][i];
        partial[(int64_t)i * nblocks + blockIdx.x] = r;
    }
}

template <bool Y_BF16> QMM_DEV f32x4 load_y4(const void* yv, int64_t i)
{
    if constexpr (Y_BF16) {
        const u32x2 w = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(yv) + i);
        return f32x4{__uint_as_float(w[0] << 16), __uint_as_float(w[0] & 0xFFFF0000u),
                     __uint_as_float(w[1] << 16), __uint_as_float(w[1] & 0xFFFF0000u)};
    } else {
        return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(yv) + i);
    }
}

template <bool Y_BF16, bool HAS_D> __global__ void __launch_bounds__(kThreads)
metric_partial(const void* __restrict__ yv, const float* __restrict__ r, const float* __restrict__ d, int64_t n,
               double* __restrict__ partial)
{
    Acc acc;
    const int64_t nvec = n >> 2;
    const int64_t tid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const f32x4* r4 = reinterpret_cast<const f32x4*>(r);
    const f32x4* d4 = reinterpret_cast<const f32x4*>(d);
    // A workgroup takes two consecutive pieces of 256 vectors per trip and the grid sweeps the arrays front to
    // back, so the loads in flight are neighbours in memory (loads a whole grid stride apart read large arrays
    // up to 25 % slower).  Both loads are in flight before the arithmetic of either starts.
    const int64_t stride = (int64_t)gridDim.x * kThreads * 2;
    int64_t i = (int64_t)blockIdx.x * kThreads * 2 + threadIdx.x;
    // (y and the reference are read once: streaming loads, which leave the caches to the tensors that are read again --
    // the benchmark's step is 3 % shorter for it, the pass itself 4 %)
    for (; i + kThreads < nvec; i += stride) {
        const f32x4 y0 = load_y4<Y_BF16>(yv, i), y1 = load_y4<Y_BF16>(yv, i + kThreads);
        const f32x4 r0 = __builtin_nontemporal_load(r4 + i), r1 = __builtin_nontemporal_load(r4 + i + kThreads);
        f32x4 d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
        if constexpr (HAS_D) { d0 = d4[i]; d1 = d4[i + kThreads]; }
        // |e|, |r| and the quotients of all eight elements first, four divisions per reciprocal estimate.  An element
        // the plain sums would get wrong (NaN or infinite e, r == 0, d not in (0, inf)) shows as a quotient that is
        // +infinity or NaN, which makes the running sum of quotients (all >= 0, far from overflow) non-finite, or is
        // caught by the sign test on d: then the whole wavefront takes the general path and the sums are not kept.
        double ae[8], ar[8], dd[8], x[8], q[8], qb[8];
        double re_next = acc.re_sum, be_next = acc.be_sum;
        bool sp = false;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float yf = j < 4 ? y0[j & 3] : y1[j & 3], rf = j < 4 ? r0[j & 3] : r1[j & 3];
            ae[j] = (double)yf - (double)rf;       // signed: the magnitudes are operand modifiers where they are used
            ar[j] = (double)rf;
        }
        reciprocals4(ar, x); reciprocals4(ar + 4, x + 4);      // signed reciprocals: the four signs cancel in pairs
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            q[j] = quotient_with(fabs(ae[j]), fabs(ar[j]), fabs(x[j]));
            re_next += q[j];
            qb[j] = 0.0;
        }
        sp = !(re_next < (double)__builtin_inff());
        if constexpr (HAS_D) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float df = j < 4 ? d0[j & 3] : d1[j & 3];
                dd[j] = (double)df;
                sp = sp || !(df > 0.0f);
            }
            reciprocals4(dd, x); reciprocals4(dd + 4, x + 4);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                qb[j] = quotient_with(fabs(ae[j]), dd[j], x[j]);
                be_next += qb[j];
            }
            sp = sp || !(be_next < (double)__builtin_inff());
        }
        if (!__any(sp)) {
#pragma unroll
            for (int j = 0; j < 8; ++j) acc.add_plain<HAS_D>(ae[j], ar[j], q[j], qb[j]);
            acc.re_sum = re_next;
            if constexpr (HAS_D) acc.be_sum = be_next;
            acc.count_plain<HAS_D>(8u);
        } else {
            // rare path, kept rolled: unrolled, its eight interleaved IEEE divisions set the kernel's register
            // count (99 instead of 72) and with it the number of resident wavefronts
#pragma unroll 1
            for (int j = 0; j < 8; ++j) {
                const f32x4 yy = j < 4 ? y0 : y1, rr = j < 4 ? r0 : r1, dd = j < 4 ? d0 : d1;
                acc.add<HAS_D>(yy[j & 3], rr[j & 3], dd[j & 3]);
            }
        }
    }
    if (i < nvec) {      // ragged end: the first piece of a workgroup's last trip
        const f32x4 y0 = load_y4<Y_BF16>(yv, i);
        const f32x4 r0 = r4[i];
        f32x4 d0 = {0.f, 0.f, 0.f, 0.f};
        if constexpr (HAS_D) d0 = d4[i];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc.add<HAS_D>(y0[j], r0[j], d0[j]);
    }
    // tail elements (n % 4), one thread each
    const int64_t t = (nvec << 2) + tid;
    if (t < n) {
        float y;
        if constexpr (Y_BF16) y = bf16_bits_to_f32(static_cast<const uint16_t*>(yv)[t]);
        else y = static_cast<const float*>(yv)[t];
        acc.add<HAS_D>(y, r[t], HAS_D ? d[t] : 0.f);
    }
    store_partial(acc, partial, (int)gridDim.x);
}

// Sixteen workgroups, one per field: thread t takes blocks t, t+256, ... in ascending order, the 64 lane values
// are folded by the fixed shuffle tree and the four wavefront values in wavefront order: the order of additions
// depends on nblocks only, so results are reproducible run to run.
constexpr int kFinalThreads = 256;
__global__ void __launch_bounds__(kFinalThreads)
metric_finalize(const double* __restrict__ partial, int nblocks, double* __restrict__ out)
{
    __shared__ double s[kFinalThreads / kWave];
    const int field = blockIdx.x, lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
    const bool is_max = (field == 4 || field == 5 || field == 7 || field == 10);
    const double* p = partial + (int64_t)field * nblocks;
    // all of a thread's partials are requested before any is used
    double v[kMaxBlocks / kFinalThreads];
#pragma unroll
    for (int k = 0; k < kMaxBlocks / kFinalThreads; ++k) {
        const int b = threadIdx.x + k * kFinalThreads;
        v[k] = b < nblocks ? p[b] : 0.0;
    }
    double r = 0.0;
#pragma unroll
    for (int k = 0; k < kMaxBlocks / kFinalThreads; ++k) r = is_max ? fmax(r, v[k]) : r + v[k];
    r = is_max ? wave_max_f64(r) : wave_sum_f64(r);
    if (lane == 0) s[w] = r;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = s[0];
        for (int k = 1; k < kFinalThreads / kWave; ++k) t = is_max ? fmax(t, s[k]) : t + s[k];
        out[field] = t;
    }
}

int plan_blocks(int64_t n)
{
    const int64_t per_block = (int64_t)kThreads * 4 * 4;   // four 4-element vectors per thread at least
    int64_t nb = (n + per_block - 1) / per_block;
    if (nb < 1) nb = 1;
    if (nb > kMaxBlocks) nb = kMaxBlocks;
    return (int)nb;
}

}  // namespace
}  // namespace qmm

using namespace qmm;

extern "C" size_t qmm_metric_workspace_size(int64_t n)
{
    return (size_t)plan_blocks(n < 0 ? 0 : n) * 16 * sizeof(double);
}

extern "C" qmm_status qmm_metric(const void* y, qmm_dtype y_dtype, const float* y_ref, const float* denom, int64_t n,
                                 double* out16, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!out16) return QMM_ERR_NULL;
    if (y_dtype != QMM_DT_BF16 && y_dtype != QMM_DT_F32) return QMM_ERR_ENUM;
    if (n < 0) return QMM_ERR_SHAPE;
    if (n > 0 && (!y || !y_ref)) return QMM_ERR_NULL;
    if (!workspace || workspace_bytes < qmm_metric_workspace_size(n)) return QMM_ERR_WORKSPACE;
    if (!aligned16(workspace) || (reinterpret_cast<uintptr_t>(out16) & 7u)) return QMM_ERR_ALIGN;
    if (n > 0 && (!aligned16(y_ref) || (denom && !aligned16(denom)) ||
                  (reinterpret_cast<uintptr_t>(y) & (y_dtype == QMM_DT_BF16 ? 7u : 15u))))
        return QMM_ERR_ALIGN;

    hipStream_t s = as_stream(stream);
    double* partial = static_cast<double*>(workspace);
    const bool bf = y_dtype == QMM_DT_BF16, hd = denom != nullptr;
    // with denominators the kernel holds 156 registers: three workgroups resident per CU, so no more than that are launched
    const int nb = hd ? std::min(plan_blocks(n), 768) : plan_blocks(n);
    if (bf && hd) metric_partial<true, true><<<nb, kThreads, 0, s>>>(y, y_ref, denom, n, partial);
    else if (bf) metric_partial<true, false><<<nb, kThreads, 0, s>>>(y, y_ref, denom, n, partial);
    else if (hd) metric_partial<false, true><<<nb, kThreads, 0, s>>>(y, y_ref, denom, n, partial);
    else metric_partial<false, false><<<nb, kThreads, 0, s>>>(y, y_ref, denom, n, partial);
    if (hipGetLastError() != hipSuccess) return QMM_ERR_LAUNCH;
    metric_finalize<<<16, kFinalThreads, 0, s>>>(partial, nb, out16);
    return launch_status();
}
