/*
 * qmm_oracle.c -- slow, plain CPU definition of the metric-driven quantized
 * matrix multiply.  TEST INFRASTRUCTURE ONLY: it exists so that the GPU
 * library can be checked against something written straight from the paper.
 * It shares no source, header, table or helper with the HIP code, and only
 * the tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Every function cites the passage of "A Metric Driven Approach to Mixed
 * Precision Training" (arXiv 2408.02897) that it follows.  Where the paper is
 * silent the reading taken is stated next to the code.
 *
 * Conventions: matrices are dense row-major float (binary32) arrays
 * [batch][rows][cols]; a bfloat16 input is widened to binary32 by the caller
 * (that widening is exact).  "contract_axis" names the axis that the matrix
 * multiply sums over (0 = rows, 1 = cols).  Codes are written
 * [batch][non-contracting][contracting].  Scale groups: group g = (b /
 * batch_inner) % batch_groups (the Results section's granularity levels: one
 * group for the whole batch, or one per index of some of the batch dimensions;
 * with the batch laid out [outer][mid][inner] the groups follow mid); with
 * per_channel there is one step size for every index of the non-contracting
 * axis, delta[g*C + c]; otherwise one per group, delta[g].
 *
 * Parity pins (tests/test_oracle_*.py): closed-form value tables and the three
 * printed maxima; brute-force nearest-value search written separately in
 * numpy; torch's own float8 casts inside the finite range; Python integers and
 * Fractions for the products; numpy float64 for the metric sums; the published
 * known-answer vectors of Philox4x32-10.  The *choice* of Philox as the random
 * source of stochastic rounding is this build's (the paper names none):
 * parity unpinned for that choice, pinned for everything else.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_INT8 = 0, ORC_E4M3 = 1, ORC_E5M2 = 2 };
enum { ORC_RTNE = 0, ORC_STOCHASTIC = 1 };

/* Threads the row-parallel loops of the products use (for reporting). */
int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Formats                                                             */
/* ------------------------------------------------------------------ */

/* Largest expressible magnitude of each format (Methodology, last
 * implementation bullet: 448 for E4M3, 57344 for E5M2, 127 for INT8;
 * Eq. 1: 2^(n-1)-1 with n = 8). */
double orc_qmax(int fmt)
{
    if (fmt == ORC_INT8) return 127.0;
    if (fmt == ORC_E4M3) return 448.0;
    if (fmt == ORC_E5M2) return 57344.0;
    return NAN;
}

/* Value of an FP8 bit pattern.  Methodology: "EeMm" formats with one sign
 * bit and a biased exponent, following the FP8 formats paper the text cites:
 * E4M3 has bias 7, no infinities and a single NaN mantissa pattern
 * (S.1111.111); E5M2 has bias 15 and IEEE-style inf / NaN in the top
 * exponent.  Exponent field 0 holds the subnormals. */
double orc_fp8_value(int fmt, unsigned code)
{
    int ebits = (fmt == ORC_E4M3) ? 4 : 5;
    int mbits = (fmt == ORC_E4M3) ? 3 : 2;
    int bias = (fmt == ORC_E4M3) ? 7 : 15;
    unsigned s = (code >> 7) & 1u;
    unsigned e = (code >> mbits) & ((1u << ebits) - 1u);
    unsigned m = code & ((1u << mbits) - 1u);
    double v;
    if (fmt == ORC_E4M3) {
        if (e == 15u && m == 7u) return NAN;
    } else {
        if (e == 31u) return m == 0u ? (s ? -INFINITY : INFINITY) : NAN;
    }
    if (e == 0u)
        v = ldexp((double)m, 1 - bias - mbits);
    else
        v = ldexp((double)((1u << mbits) + m), (int)e - bias - mbits);
    return s ? -v : v;
}

/* Code of the largest finite magnitude. */
static unsigned fp8_max_code(int fmt) { return fmt == ORC_E4M3 ? 0x7Eu : 0x7Bu; }

/* Value of a stored 8-bit code in any of the three formats. */
double orc_code_value(int fmt, unsigned code)
{
    if (fmt == ORC_INT8) return (double)(int8_t)(uint8_t)code;
    return orc_fp8_value(fmt, code & 0xFFu);
}

/* Index i of the largest non-negative finite grid value <= a, for
 * 0 <= a < max.  Non-negative codes are ordered like their values. */
static unsigned fp8_floor_code(int fmt, double a)
{
    unsigned lo = 0, hi = fp8_max_code(fmt); /* value(lo) <= a < value(hi) */
    while (hi - lo > 1u) {
        unsigned mid = (lo + hi) / 2u;
        if (orc_fp8_value(fmt, mid) <= a) lo = mid; else hi = mid;
    }
    return lo;
}

/* Round-to-nearest-even onto the FP8 grid (Methodology: RTNE is the default
 * rounding; first implementation bullet: magnitudes above the maximum are
 * saturated at the maximum, and values too small for the smallest subnormal
 * become zero).  Reading taken: rounding is to the nearest of ALL finite grid
 * values including zero, so (minsub/2, minsub) rounds up to minsub and exactly
 * minsub/2 ties to zero; +-inf saturate; the sign of t is always kept (so a
 * negative underflow gives 0x80); NaN gives 0x7F in both formats whatever its
 * sign bit (the sign of a NaN produced by arithmetic differs between
 * machines, so it is not carried). */
uint8_t orc_fp8_encode_rtne(int fmt, float t)
{
    unsigned sign = signbit(t) ? 0x80u : 0u;
    if (isnan(t)) return (uint8_t)0x7Fu;
    double a = fabs((double)t);
    unsigned cmax = fp8_max_code(fmt);
    if (a >= orc_fp8_value(fmt, cmax)) return (uint8_t)(sign | cmax);
    unsigned i = fp8_floor_code(fmt, a);
    double below = a - orc_fp8_value(fmt, i);       /* exact in double */
    double above = orc_fp8_value(fmt, i + 1u) - a;  /* exact in double */
    unsigned c;
    if (below < above) c = i;
    else if (below > above) c = i + 1u;
    else c = (i & 1u) ? i + 1u : i;                 /* tie: even mantissa LSB */
    return (uint8_t)(sign | c);
}

/* Eq. 1 for INT8: round to the nearest integer, ties to even, then keep the
 * symmetric range [-127, 127] (2^(n-1)-1; saturation bullet).  -128 is never
 * produced.  NaN gives 0 (the paper is silent; reading taken). */
uint8_t orc_int8_encode_rtne(float t)
{
    if (isnan(t)) return 0;
    double x = (double)t;
    double f = floor(x);
    double d = x - f;
    double r;
    if (d < 0.5) r = f;
    else if (d > 0.5) r = f + 1.0;
    else r = (fmod(f, 2.0) == 0.0) ? f : f + 1.0;
    if (r > 127.0) r = 127.0;
    if (r < -127.0) r = -127.0;
    return (uint8_t)(int8_t)(int)r;
}

uint8_t orc_encode_rtne(int fmt, float t)
{
    return fmt == ORC_INT8 ? orc_int8_encode_rtne(t) : orc_fp8_encode_rtne(fmt, t);
}

/* Stochastic rounding (second implementation bullet).  |t| lies between two
 * neighbouring grid values lo <= |t| < hi; the result is hi with probability
 * (|t|-lo)/(hi-lo) and lo otherwise, which makes the rounding unbiased.
 * u24 is a uniform 24-bit integer; "up" is taken iff u24 / 2^24 is below that
 * probability.  Saturation and NaN as in RTNE. */
uint8_t orc_encode_sr(int fmt, float t, uint32_t u24)
{
    double u = (double)(u24 & 0xFFFFFFu);
    if (fmt == ORC_INT8) {
        if (isnan(t)) return 0;
        double a = fabs((double)t);
        double r;
        if (a >= 127.0) r = 127.0;
        else {
            double lo = floor(a);
            double p = a - lo;
            r = lo + ((u < p * 16777216.0) ? 1.0 : 0.0);
        }
        if (signbit(t)) r = -r;
        return (uint8_t)(int8_t)(int)r;
    }
    unsigned sign = signbit(t) ? 0x80u : 0u;
    if (isnan(t)) return (uint8_t)0x7Fu;
    double a = fabs((double)t);
    unsigned cmax = fp8_max_code(fmt);
    if (a >= orc_fp8_value(fmt, cmax)) return (uint8_t)(sign | cmax);
    unsigned i = fp8_floor_code(fmt, a);
    double lo = orc_fp8_value(fmt, i), hi = orc_fp8_value(fmt, i + 1u);
    double p = (a - lo) / (hi - lo);
    unsigned c = i + ((u < p * 16777216.0) ? 1u : 0u);
    return (uint8_t)(sign | c);
}

/* ------------------------------------------------------------------ */
/* Random source of stochastic rounding: Philox4x32-10 (Salmon, Moraes,  */
/* Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11).    */
/* The paper names no generator; this build fixes one so that both sides */
/* can reproduce the same draws from (seed, element index).              */
/* ------------------------------------------------------------------ */
void orc_philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4])
{
    uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
    uint32_t k0 = key_in[0], k1 = key_in[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 24 random bits of output element number g (g = linear index in the
 * code array + caller's offset): Philox block g/4 under key = seed, word
 * g%4, top 24 bits. */
uint32_t orc_sr_bits(uint64_t seed, uint64_t g)
{
    uint64_t blk = g >> 2;
    uint32_t ctr[4] = { (uint32_t)blk, (uint32_t)(blk >> 32), 0u, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return out[g & 3u] >> 8;
}

/* ------------------------------------------------------------------ */
/* Step 1: step size (Eq. 1, right half)                               */
/* ------------------------------------------------------------------ */

static int64_t n_channels(int64_t rows, int64_t cols, int contract_axis, int per_channel)
{
    if (!per_channel) return 1;
    return contract_axis == 1 ? rows : cols;
}

/* delta = max|X| / qmax over each scale group (Eq. 1; scaling bullets: tensor
 * level or finer on non-contracting dimensions; absmax aligned to the format
 * maximum).  Readings taken where the paper is silent: binary32 arithmetic,
 * one correctly rounded division; the maximum is taken over magnitude bit
 * patterns so an inf or NaN element dominates; an all-zero group gets
 * delta = 1; a quotient below 2^-126 is raised to 2^-126. */
static int64_t group_of(int64_t b, int64_t batch_groups, int64_t batch_inner)
{
    return (b / (batch_inner > 0 ? batch_inner : 1)) % batch_groups;
}

void orc_scale(const float* x, int64_t batch, int64_t rows, int64_t cols, int contract_axis,
               int fmt, int per_channel, int64_t batch_groups, int64_t batch_inner, float* delta)
{
    int64_t C = n_channels(rows, cols, contract_axis, per_channel);
    int64_t ng = batch_groups * C;
    uint32_t* amax = (uint32_t*)calloc((size_t)(ng > 0 ? ng : 1), sizeof(uint32_t));
    for (int64_t b = 0; b < batch; ++b)
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t c = 0; c < cols; ++c) {
                float v = x[(b * rows + r) * cols + c];
                uint32_t bits; memcpy(&bits, &v, 4);
                bits &= 0x7FFFFFFFu;
                int64_t ch = per_channel ? (contract_axis == 1 ? r : c) : 0;
                int64_t g = group_of(b, batch_groups, batch_inner) * C + ch;
                if (bits > amax[g]) amax[g] = bits;
            }
    float qmax = (float)orc_qmax(fmt);
    for (int64_t g = 0; g < ng; ++g) {
        float a; memcpy(&a, &amax[g], 4);
        float d;
        if (a == 0.0f) d = 1.0f;
        else {
            d = a / qmax;
            if (d < 0x1p-126f) d = 0x1p-126f;
        }
        delta[g] = d;
    }
    free(amax);
}

/* ------------------------------------------------------------------ */
/* Step 2: quantize (Eq. 1, left half)                                 */
/* ------------------------------------------------------------------ */

/* code = round(X / delta).  Reading taken for the arithmetic (the paper gives
 * none): binary32; the quotient is formed as x * (1/delta) with one correctly
 * rounded reciprocal per group and one correctly rounded product per element.
 * Output order [batch][non-contracting][contracting]. */
void orc_quantize(const float* x, int64_t batch, int64_t rows, int64_t cols, int contract_axis,
                  int fmt, int per_channel, int64_t batch_groups, int64_t batch_inner, const float* delta,
                  int mode, uint64_t seed, uint64_t offset, uint8_t* codes)
{
    int64_t NC = contract_axis == 1 ? rows : cols;   /* non-contracting extent */
    int64_t KC = contract_axis == 1 ? cols : rows;   /* contracting extent     */
    int64_t C = n_channels(rows, cols, contract_axis, per_channel);
    for (int64_t b = 0; b < batch; ++b)
        for (int64_t n = 0; n < NC; ++n) {
            float d = delta[group_of(b, batch_groups, batch_inner) * C + (per_channel ? n : 0)];
            volatile float rho = 1.0f / d;
            for (int64_t k = 0; k < KC; ++k) {
                int64_t r = contract_axis == 1 ? n : k;
                int64_t c = contract_axis == 1 ? k : n;
                volatile float t = x[(b * rows + r) * cols + c] * rho;
                int64_t p = (b * NC + n) * KC + k;
                if (mode == ORC_RTNE) codes[p] = orc_encode_rtne(fmt, t);
                else codes[p] = orc_encode_sr(fmt, t, orc_sr_bits(seed, (uint64_t)p + offset));
            }
        }
}

/* ------------------------------------------------------------------ */
/* Step 3: product of codes (third implementation bullet: the result   */
/* before re-scaling lives in a wider accumulator)                     */
/* ------------------------------------------------------------------ */

/* acc[b][i][j] = sum_k value(a[b][i][k]) * value(b[b][j][k]), summed in
 * double in ascending k.  Every product of two 8-bit values is exact in
 * double, and for INT8 the whole sum is exact.  sabs (may be NULL) receives
 * sum_k |value(a)|*|value(b)|, the scale of the rounding error bound. */
void orc_gemm_codes(const uint8_t* a, int a_fmt, const uint8_t* b, int b_fmt,
                    int64_t batch, int64_t M, int64_t N, int64_t K,
                    double* acc, double* sabs)
{
    double va[256], vb[256];
    for (unsigned c = 0; c < 256; ++c) { va[c] = orc_code_value(a_fmt, c); vb[c] = orc_code_value(b_fmt, c); }
    for (int64_t bb = 0; bb < batch; ++bb) {
        const uint8_t* A = a + bb * M * K;
        const uint8_t* B = b + bb * N * K;
        #pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < N; ++j) {
                double s = 0.0, sa = 0.0;
                for (int64_t k = 0; k < K; ++k) {
                    double p = va[A[i * K + k]] * vb[B[j * K + k]];
                    s += p;
                    sa += fabs(p);
                }
                acc[(bb * M + i) * N + j] = s;
                if (sabs) sabs[(bb * M + i) * N + j] = sa;
            }
    }
}

/* The same product for selected rows of A only: out row r is row rows[r]. */
void orc_gemm_codes_rows(const uint8_t* a, int a_fmt, const uint8_t* b, int b_fmt,
                         int64_t N, int64_t K, const int64_t* rows, int64_t nrows,
                         double* acc, double* sabs)
{
    double va[256], vb[256];
    for (unsigned c = 0; c < 256; ++c) { va[c] = orc_code_value(a_fmt, c); vb[c] = orc_code_value(b_fmt, c); }
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nrows; ++r)
        for (int64_t j = 0; j < N; ++j) {
            double s = 0.0, sa = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double p = va[a[rows[r] * K + k]] * vb[b[j * K + k]];
                s += p;
                sa += fabs(p);
            }
            acc[r * N + j] = s;
            if (sabs) sabs[r * N + j] = sa;
        }
}

/* INT8 x INT8 with a 64-bit integer accumulator.  Returns the number of
 * results that do not fit a 32-bit accumulator (expected 0). */
int64_t orc_gemm_int8(const int8_t* a, const int8_t* b, int64_t batch, int64_t M, int64_t N, int64_t K,
                      int64_t* acc)
{
    int64_t bad = 0;
    for (int64_t bb = 0; bb < batch; ++bb)
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < N; ++j) {
                int64_t s = 0;
                for (int64_t k = 0; k < K; ++k)
                    s += (int64_t)a[(bb * M + i) * K + k] * (int64_t)b[(bb * N + j) * K + k];
                acc[(bb * M + i) * N + j] = s;
                if (s > INT32_MAX || s < INT32_MIN) ++bad;
            }
    return bad;
}

/* ------------------------------------------------------------------ */
/* Step 4: descale (third implementation bullet; figure on the graph   */
/* modification)                                                       */
/* ------------------------------------------------------------------ */

/* Round a binary32 value to the nearest bfloat16 (ties to even); the result
 * is returned widened back to binary32. */
float orc_bf16_round(float v)
{
    uint32_t u; memcpy(&u, &v, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) { u |= 0x00400000u; u &= 0xFFFF0000u; }
    else { u += 0x7FFFu + ((u >> 16) & 1u); u &= 0xFFFF0000u; }
    float r; memcpy(&r, &u, 4);
    return r;
}

/* y = (acc * deltaL[row]) * deltaR[col] in binary32, in that order; acc is
 * first rounded once to binary32 (the accumulator type of the FP8 path; exact
 * for the integer path below 2^24 and correctly rounded above).  deltaL is
 * indexed by the row of the left operand, deltaR by the row of the right
 * operand (= output column) when per-channel; both by b % groups. */
void orc_dequant(const double* acc, int64_t batch, int64_t M, int64_t N,
                 const float* dl, int l_per_channel, int64_t l_groups, int64_t l_inner,
                 const float* dr, int r_per_channel, int64_t r_groups, int64_t r_inner,
                 int out_bf16, float* y)
{
    for (int64_t b = 0; b < batch; ++b)
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < N; ++j) {
                float sl = dl[group_of(b, l_groups, l_inner) * (l_per_channel ? M : 1) + (l_per_channel ? i : 0)];
                float sr = dr[group_of(b, r_groups, r_inner) * (r_per_channel ? N : 1) + (r_per_channel ? j : 0)];
                volatile float a = (float)acc[(b * M + i) * N + j];
                volatile float t = a * sl;
                volatile float v = t * sr;
                y[(b * M + i) * N + j] = out_bf16 ? orc_bf16_round(v) : v;
            }
}

/* ------------------------------------------------------------------ */
/* Step 5: the high-precision product the metric compares against      */
/* ------------------------------------------------------------------ */

/* r[b][i][j] = sum_k x[b][i][k] * w[b][j][k] on the un-quantized values
 * (Eq. 1 names bfloat16 as the high-precision type), summed in double and
 * rounded once to binary32. */
void orc_ref_gemm(const float* x, const float* w, int64_t batch, int64_t M, int64_t N, int64_t K, float* r)
{
    for (int64_t bb = 0; bb < batch; ++bb) {
        const float* X = x + bb * M * K;
        const float* W = w + bb * N * K;
        #pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < N; ++j) {
                double s = 0.0;
                for (int64_t k = 0; k < K; ++k) s += (double)X[i * K + k] * (double)W[j * K + k];
                r[(bb * M + i) * N + j] = (float)s;
            }
    }
}

/* ------------------------------------------------------------------ */
/* Step 6: error metrics                                               */
/* ------------------------------------------------------------------ */

/* One pass over (y, r[, d]) with e = y - r in double.
 *   out[0]  sum e^2            out[1]  sum r^2
 *   out[2]  sum |e|            out[3]  sum |r|
 *   out[4]  max |e|            out[5]  max |r|
 *   out[6]  sum_{r!=0} |e|/|r| (Eq. 2, taken with |v| in the denominator)
 *   out[7]  max of the same    out[8]  number of terms in it
 *   out[9]  sum_{d>0} |e|/d    (Eq. 3 element-wise, d = (|L|.|R|)_ij)
 *   out[10] max of the same    out[11] number of terms in it
 *   out[12] elements counted   out[13] elements skipped because e is NaN
 *   out[14], out[15] zero.
 * Noise-to-signal ratio of the op = out[0]/out[1] (named by the task, not by
 * the paper).  Elements whose error is NaN are counted in out[13] and left
 * out of everything else. */
void orc_metric(const float* y, const float* r, const float* d, int64_t n, double* out)
{
    for (int i = 0; i < 16; ++i) out[i] = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double e = (double)y[i] - (double)r[i];
        if (isnan(e)) { out[13] += 1.0; continue; }
        double ae = fabs(e), ar = fabs((double)r[i]);
        out[0] += e * e;
        out[1] += ar * ar;
        out[2] += ae;
        out[3] += ar;
        if (ae > out[4]) out[4] = ae;
        if (ar > out[5]) out[5] = ar;
        if (ar != 0.0) {
            double q = ae / ar;
            out[6] += q;
            if (q > out[7]) out[7] = q;
            out[8] += 1.0;
        }
        if (d && (double)d[i] > 0.0) {
            double q = ae / (double)d[i];
            out[9] += q;
            if (q > out[10]) out[10] = q;
            out[11] += 1.0;
        }
        out[12] += 1.0;
    }
}

/* ---- Tensor moments (Results section, first paragraph: inputs of the matrix multiplications are sampled "to
 * compute the mean, variance, skew and Kurtosis").  The paper does not say which estimators; reading: the plain
 * population moments about the mean,
 *     mean = sum x / n,   m_k = sum (x - mean)^k / n  for k = 2, 3, 4,
 * from which skew = m3 / m2^1.5 and (Pearson) kurtosis = m4 / m2^2 (3 for a normal distribution).
 * Two passes in binary64, exactly as written.  NaN elements are counted in out[6] and left out of everything
 * else.  out (8 doubles): n (non-NaN count), mean, m2, m3, m4, max |x|, NaN count, 0. */
void orc_moments(const float* x, int64_t n, double* out)
{
    for (int i = 0; i < 8; ++i) out[i] = 0.0;
    /* sums in the x87 extended format (64-bit significand): the definition is the exact sum, and a sequential
     * binary64 sum of 10^7 terms already carries a rounding error of 1e-11 relative */
    long double sum = 0.0L;
    double cnt = 0.0, amax = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        if (isnan(x[i])) { out[6] += 1.0; continue; }
        cnt += 1.0;
        sum += (long double)x[i];
        if (fabs((double)x[i]) > amax) amax = fabs((double)x[i]);
    }
    out[0] = cnt; out[5] = amax;
    if (cnt == 0.0) return;
    const long double mean = sum / (long double)cnt;
    long double s2 = 0.0L, s3 = 0.0L, s4 = 0.0L;
    for (int64_t i = 0; i < n; ++i) {
        if (isnan(x[i])) continue;
        const long double d = (long double)x[i] - mean;
        s2 += d * d;
        s3 += d * d * d;
        s4 += d * d * d * d;
    }
    out[1] = (double)mean; out[2] = (double)(s2 / cnt); out[3] = (double)(s3 / cnt); out[4] = (double)(s4 / cnt);
}

/* ---- The reduced-precision value of a quantized element (the v-tilde of Eq. 2): the value of its code times the
 * step size of its scale group, one binary32 multiply (the code's value is exact in binary32).  Layout of codes
 * and indexing of delta as written by orc_quantize: codes [batch][nc][kc] with the contracting axis last,
 * delta[(b % groups) * C + (per_channel ? row : 0)].  An FP8 NaN code gives NaN; the INT8 code 0x80, which the
 * encoder never produces, gives -128 delta. */
void orc_dequantize_codes(const uint8_t* codes, int64_t batch, int64_t nc, int64_t kc, int fmt,
                          int per_channel, int64_t groups, int64_t inner, const float* delta, float* out)
{
    const int64_t C = per_channel ? nc : 1;
    for (int64_t b = 0; b < batch; ++b)
        for (int64_t r = 0; r < nc; ++r) {
            const float d = delta[group_of(b, groups, inner) * C + (per_channel ? r : 0)];
            for (int64_t k = 0; k < kc; ++k) {
                const int64_t i = (b * nc + r) * kc + k;
                out[i] = (float)orc_code_value(fmt, codes[i]) * d;
            }
        }
}
