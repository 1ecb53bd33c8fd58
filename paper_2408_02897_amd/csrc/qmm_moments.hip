// qmm_moments: mean and the central moments of orders 2, 3, 4 of all elements of a tensor, plus max |x| (Results
// section, first paragraph: the inputs of the matrix multiplications are characterised by mean, variance, skew and
// kurtosis).  One pass over the data (HBM-bound, 2 B per bfloat16 element): every thread accumulates the power
// sums of d = x - center in binary64; workgroup partials are folded in a fixed order by a second small kernel,
// which also turns the power sums into moments about the mean.  No atomics: reproducible run to run.
#include "qmm_device.h"

namespace qmm {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxBlocks = 2048;
constexpr int kFields = 7;             // S1, S2, S3, S4, max |x|, count, NaN count
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct Sums {
    double s1 = 0, s2 = 0, s3 = 0, s4 = 0;
    float amax = 0.f;
    unsigned cnt = 0, nan_cnt = 0;

    QMM_DEV void add(float xf, double center)
    {
        if (xf != xf) { nan_cnt += 1u; return; }
        const double d = (double)xf - center, d2 = d * d;
        s1 += d; s2 += d2; s3 = fma(d2, d, s3); s4 = fma(d2, d2, s4);
        amax = fmaxf(amax, fabsf(xf));
        cnt += 1u;
    }
    // Eight elements none of which is NaN.  CENTERED = false: center == 0, the subtraction is left out (x - 0 = x).
    // The pass is ALU- as much as HBM-bound (a bfloat16 element brings 2 bytes and needs 8 instructions), so the
    // common case is kept to the conversions, one multiply and four accumulations per element.
    template <bool CENTERED> QMM_DEV void add8_plain(const double (&d)[8], const float (&e)[8])
    {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const double d2 = d[i] * d[i];
            s2 += d2; s3 = fma(d2, d[i], s3); s4 = fma(d2, d2, s4);
        }
#pragma unroll
        for (int i = 0; i < 8; i += 2) amax = fmaxf(fmaxf(amax, fabsf(e[i])), fabsf(e[i + 1]));    // one three-way maximum
        cnt += 8u;
    }
};

template <bool BF16> QMM_DEV void load8(const void* x, int64_t v, float (&out)[8])
{
    if constexpr (BF16) {
        const u32x4 w = reinterpret_cast<const u32x4*>(x)[v];
#pragma unroll
        for (int i = 0; i < 4; ++i) { out[2 * i] = __uint_as_float(w[i] << 16); out[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
    } else {
        const f32x4 a = reinterpret_cast<const f32x4*>(x)[2 * v], b = reinterpret_cast<const f32x4*>(x)[2 * v + 1];
#pragma unroll
        for (int i = 0; i < 4; ++i) { out[i] = a[i]; out[4 + i] = b[i]; }
    }
}

// partial[field * nblocks + block]
template <bool BF16, bool CENTERED> __global__ void __launch_bounds__(kThreads)
moments_partial(const void* __restrict__ x, int64_t n, double center, double* __restrict__ partial)
{
    Sums acc;
    const int64_t nvec = n >> 3;                       // vectors of eight elements
    const int64_t tid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    auto consume = [&](const float (&e)[8]) {
        // The eight deviations are summed first, as a tree: a NaN element makes that sum NaN (so do infinities of
        // both signs, for which the general path gives the same NaN sums), and one test replaces eight.
        double d[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) d[i] = CENTERED ? (double)e[i] - center : (double)e[i];
        const double t = ((d[0] + d[1]) + (d[2] + d[3])) + ((d[4] + d[5]) + (d[6] + d[7]));
        if (!__any(t != t)) {                          // the common case, without per-element tests
            acc.s1 += t;
            acc.template add8_plain<CENTERED>(d, e);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc.add(e[i], center);
        }
    };
    // Four consecutive pieces of 256 vectors per workgroup and trip, the grid sweeping the tensor front to back:
    // a thread's four loads in flight are neighbours in memory (a whole grid stride apart they read a large
    // tensor up to 25 % slower); all four are in flight before the arithmetic of the first starts.
    const int64_t sweep = (int64_t)gridDim.x * kThreads * 4;
    int64_t vi = (int64_t)blockIdx.x * kThreads * 4 + threadIdx.x;
    for (; vi + 3 * kThreads < nvec; vi += sweep) {
        float e0[8], e1[8], e2[8], e3[8];
        load8<BF16>(x, vi, e0); load8<BF16>(x, vi + kThreads, e1); load8<BF16>(x, vi + 2 * kThreads, e2); load8<BF16>(x, vi + 3 * kThreads, e3);
        consume(e0); consume(e1); consume(e2); consume(e3);
    }
    if (vi < nvec) {     // ragged end: at most three pieces of one workgroup
        for (int u = 0; u < 4; ++u)
            if (vi + u * kThreads < nvec) {
                float e[8];
                load8<BF16>(x, vi + u * kThreads, e);
                consume(e);
            }
    }
    const int64_t t = (nvec << 3) + tid;               // tail elements (n % 8), one thread each
    if (t < n) {
        float xf;
        if constexpr (BF16) xf = bf16_bits_to_f32(static_cast<const uint16_t*>(x)[t]);
        else xf = static_cast<const float*>(x)[t];
        acc.add(xf, center);
    }
    __shared__ double s[kThreads / kWave][kFields];
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
    double v[kFields];
    v[0] = wave_sum_f64(acc.s1); v[1] = wave_sum_f64(acc.s2); v[2] = wave_sum_f64(acc.s3); v[3] = wave_sum_f64(acc.s4);
    v[4] = wave_max_f64((double)acc.amax); v[5] = wave_sum_f64((double)acc.cnt); v[6] = wave_sum_f64((double)acc.nan_cnt);
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < kFields; ++i) s[w][i] = v[i];
    }
    __syncthreads();
    if (threadIdx.x < kFields) {
        const int i = threadIdx.x;
        double r = s[0][i];
        for (int k = 1; k < kThreads / kWave; ++k) r = (i == 4) ? fmax(r, s[k][i]) : r + s[k][i];
        partial[(int64_t)i * gridDim.x + blockIdx.x] = r;
    }
}

// One workgroup of kFields wavefronts: wavefront f folds field f (lane l takes blocks l, l+64, ... in ascending
// order, then the fixed shuffle tree); thread 0 then forms the moments about the mean from the power sums about
// `center`:  with a = S1/n (= mean - center):  m2 = S2/n - a^2,  m3 = S3/n - 3 a S2/n + 2 a^3,
// m4 = S4/n - 4 a S3/n + 6 a^2 S2/n - 3 a^4.
__global__ void __launch_bounds__(kFields * kWave)
moments_finalize(const double* __restrict__ partial, int nblocks, double center, double* __restrict__ out)
{
    __shared__ double f[kFields];
    const int field = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    const double* p = partial + (int64_t)field * nblocks;
    double v[kMaxBlocks / kWave];
#pragma unroll
    for (int k = 0; k < kMaxBlocks / kWave; ++k) {
        const int b = lane + k * kWave;
        v[k] = b < nblocks ? p[b] : 0.0;
    }
    double r = 0.0;
#pragma unroll
    for (int k = 0; k < kMaxBlocks / kWave; ++k) r = (field == 4) ? fmax(r, v[k]) : r + v[k];
    r = (field == 4) ? wave_max_f64(r) : wave_sum_f64(r);
    if (lane == 0) f[field] = r;
    __syncthreads();
    if (threadIdx.x == 0) {
        const double n = f[5];
        double mean = 0.0, m2 = 0.0, m3 = 0.0, m4 = 0.0;
        if (n > 0.0) {
            const double a = f[0] / n, q2 = f[1] / n, q3 = f[2] / n, q4 = f[3] / n;
            mean = center + a;
            m2 = q2 - a * a;
            m3 = q3 - 3.0 * a * q2 + 2.0 * a * a * a;
            m4 = q4 - 4.0 * a * q3 + 6.0 * a * a * q2 - 3.0 * a * a * a * a;
        }
        out[0] = n; out[1] = mean; out[2] = m2; out[3] = m3; out[4] = m4; out[5] = f[4]; out[6] = f[6]; out[7] = 0.0;
    }
}

int plan_blocks(int64_t n)
{
    const int64_t per_block = (int64_t)kThreads * 8 * 4;   // four vectors of eight elements per thread at least
    int64_t nb = (n + per_block - 1) / per_block;
    if (nb < 1) nb = 1;
    if (nb > kMaxBlocks) nb = kMaxBlocks;
    return (int)nb;
}

}  // namespace
}  // namespace qmm

using namespace qmm;

extern "C" size_t qmm_moments_workspace_size(int64_t n)
{
    return (size_t)plan_blocks(n < 0 ? 0 : n) * kFields * sizeof(double);
}

extern "C" qmm_status qmm_moments(const void* x, qmm_dtype dtype, int64_t n, double center, double* out8,
                                  void* workspace, size_t workspace_bytes, void* stream)
{
    if (!out8) return QMM_ERR_NULL;
    if (dtype != QMM_DT_BF16 && dtype != QMM_DT_F32) return QMM_ERR_ENUM;
    if (n < 0 || !(center == center) || center - center != 0.0) return QMM_ERR_SHAPE;   // center must be finite
    if (n > 0 && !x) return QMM_ERR_NULL;
    if (!workspace || workspace_bytes < qmm_moments_workspace_size(n)) return QMM_ERR_WORKSPACE;
    if (!aligned16(workspace) || (reinterpret_cast<uintptr_t>(out8) & 7u)) return QMM_ERR_ALIGN;
    if (n > 0 && !aligned16(x)) return QMM_ERR_ALIGN;
    hipStream_t s = as_stream(stream);
    double* partial = static_cast<double*>(workspace);
    const int nb = plan_blocks(n);
    const bool bf = dtype == QMM_DT_BF16, centered = center != 0.0;
    if (bf && centered) moments_partial<true, true><<<nb, kThreads, 0, s>>>(x, n, center, partial);
    else if (bf) moments_partial<true, false><<<nb, kThreads, 0, s>>>(x, n, center, partial);
    else if (centered) moments_partial<false, true><<<nb, kThreads, 0, s>>>(x, n, center, partial);
    else moments_partial<false, false><<<nb, kThreads, 0, s>>>(x, n, center, partial);
    if (hipGetLastError() != hipSuccess) return QMM_ERR_LAUNCH;
    moments_finalize<<<1, kFields * kWave, 0, s>>>(partial, nb, center, out8);
    return launch_status();
}
