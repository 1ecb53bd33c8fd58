// Device-side helpers shared by the HIP kernels of libqmm: number formats of the
// paper (INT8, E4M3, E5M2; Methodology, Eq. 1 and the implementation bullets),
// their round-to-nearest-even and stochastic encoders, the Philox4x32-10 counter
// generator, and wavefront (64-lane) reductions.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qmm.h"

namespace qmm {

#define QMM_DEV __device__ __forceinline__

constexpr int kWave = 64;

QMM_DEV float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// ---------------------------------------------------------------------------
// Format constants.  E4M3: 1-4-3, bias 7, max 448 (0x7E), min normal 2^-6,
// min subnormal 2^-9, one NaN pattern, no inf.  E5M2: 1-5-2, bias 15, max
// 57344 (0x7B), min normal 2^-14, min subnormal 2^-16.
// ---------------------------------------------------------------------------
template <int FMT> struct Fp8;
template <> struct Fp8<QMM_FMT_E4M3> {
    static constexpr int M = 3, BIAS = 7;
    static constexpr uint32_t MAX_BITS = 0x43E00000u;      // 448.0f
    static constexpr uint32_t MINNORM_BITS = 0x3C800000u;  // 2^-6
    static constexpr uint32_t MAGIC_BITS = 0x46800000u;    // 2^14: ulp = 2^-9 = min subnormal
    static constexpr float TO_SUBNORMAL_UNITS = 512.0f;    // 1 / min subnormal
    static constexpr uint32_t MAX_CODE = 0x7Eu;
};
template <> struct Fp8<QMM_FMT_E5M2> {
    static constexpr int M = 2, BIAS = 15;
    static constexpr uint32_t MAX_BITS = 0x47600000u;      // 57344.0f
    static constexpr uint32_t MINNORM_BITS = 0x38800000u;  // 2^-14
    static constexpr uint32_t MAGIC_BITS = 0x43000000u;    // 2^7: ulp = 2^-16 = min subnormal
    static constexpr float TO_SUBNORMAL_UNITS = 65536.0f;
    static constexpr uint32_t MAX_CODE = 0x7Bu;
};

QMM_DEV float format_qmax(int fmt)
{
    return fmt == QMM_FMT_INT8 ? 127.0f : (fmt == QMM_FMT_E4M3 ? 448.0f : 57344.0f);
}

// Nearest finite FP8 value, ties to the even mantissa, saturating, sign kept,
// NaN -> 0x7F.  Integer arithmetic on the binary32 pattern: in the normal range
// of the target the mantissa is rounded from 23 to M bits by adding half an ulp
// (minus one when the kept LSB is even) and the exponent is rebiased; below the
// smallest normal the magnitude is added to 2^(23 + log2(min subnormal)), whose
// ulp is one subnormal step, so the adder's own RNE does the rounding.
template <int FMT> QMM_DEV uint32_t encode_fp8_rtne(float t)
{
    using F = Fp8<FMT>;
    const uint32_t u = __float_as_uint(t);
    const uint32_t sign = (u >> 24) & 0x80u;
    uint32_t a = u & 0x7FFFFFFFu;
    const bool is_nan = a > 0x7F800000u;
    a = min(a, F::MAX_BITS);
    const uint32_t r = a + ((1u << (22 - F::M)) - 1u) + ((a >> (23 - F::M)) & 1u);
    const uint32_t code_normal = (r >> (23 - F::M)) - ((127u - F::BIAS) << F::M);
    const float f = __uint_as_float(a) + __uint_as_float(F::MAGIC_BITS);
    const uint32_t code_sub = __float_as_uint(f) - F::MAGIC_BITS;
    const uint32_t code = a >= F::MINNORM_BITS ? code_normal : code_sub;
    return is_nan ? 0x7Fu : (sign | code);
}

// The same result for two values at once through the hardware converter.  v_cvt_pk_fp8_f32 / v_cvt_pk_bf8_f32
// round to nearest even onto the OCP grids including subnormals and keep the sign of zero; clamping to +-max first
// gives the saturation rule.  Compared against encode_fp8_rtne over all 2^32 binary32 patterns on gfx950: equal
// for every non-NaN input; NaN is handled here.  Returns code(t0) | code(t1) << 8.
template <int FMT> QMM_DEV uint32_t encode_fp8_rtne_pair(float t0, float t1)
{
    const float mx = FMT == QMM_FMT_E4M3 ? 448.0f : 57344.0f;
    const float c0 = __builtin_amdgcn_fmed3f(t0, -mx, mx), c1 = __builtin_amdgcn_fmed3f(t1, -mx, mx);
    uint32_t r;
    if constexpr (FMT == QMM_FMT_E4M3) r = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(c0, c1, 0, false);
    else r = (uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(c0, c1, 0, false);
    r &= 0xFFFFu;
    if (t0 != t0) r = (r & 0xFF00u) | 0x7Fu;
    if (t1 != t1) r = (r & 0x00FFu) | 0x7F00u;
    return r;
}

// Eq. 1 for INT8: round half to even, keep the symmetric range [-127, 127].
QMM_DEV uint32_t encode_int8_rtne(float t)
{
    const float c = fminf(fmaxf(t, -127.0f), 127.0f);
    const int q = (int)__builtin_rintf(c);
    return (t != t) ? 0u : ((uint32_t)q & 0xFFu);
}

// 16 bfloat16 values (two 16-byte vectors) times rho -> 16 RTNE codes (one 16-byte vector).
typedef unsigned int qmm_u32x4 __attribute__((ext_vector_type(4)));
template <int FMT> QMM_DEV qmm_u32x4 encode16_bf16_rtne(qmm_u32x4 w0, qmm_u32x4 w1, float rho)
{
    qmm_u32x4 out;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t wa = q < 2 ? w0[2 * q] : w1[2 * q - 4], wb = q < 2 ? w0[2 * q + 1] : w1[2 * q - 3];
        const float t0 = __uint_as_float(wa << 16) * rho, t1 = __uint_as_float(wa & 0xFFFF0000u) * rho;
        const float t2 = __uint_as_float(wb << 16) * rho, t3 = __uint_as_float(wb & 0xFFFF0000u) * rho;
        if constexpr (FMT == QMM_FMT_INT8)
            out[q] = encode_int8_rtne(t0) | (encode_int8_rtne(t1) << 8) | (encode_int8_rtne(t2) << 16) | (encode_int8_rtne(t3) << 24);
        else
            out[q] = encode_fp8_rtne_pair<FMT>(t0, t1) | (encode_fp8_rtne_pair<FMT>(t2, t3) << 16);
    }
    return out;
}

// Stochastic rounding: up iff u24 / 2^24 < (|t| - lo) / (hi - lo).  All
// quantities in the comparison are exact.
template <int FMT> QMM_DEV uint32_t encode_fp8_sr(float t, uint32_t u24)
{
    using F = Fp8<FMT>;
    const uint32_t u = __float_as_uint(t);
    const uint32_t sign = (u >> 24) & 0x80u;
    const uint32_t a = u & 0x7FFFFFFFu;
    if (a > 0x7F800000u) return 0x7Fu;
    if (a >= F::MAX_BITS) return sign | F::MAX_CODE;
    uint32_t code;
    if (a >= F::MINNORM_BITS) {
        const uint32_t rem = a & ((1u << (23 - F::M)) - 1u);              // fraction of one ulp, 23-M bits
        const uint32_t lo = (a >> (23 - F::M)) - ((127u - F::BIAS) << F::M);
        code = lo + (u24 < (rem << (F::M + 1)) ? 1u : 0u);
    } else {
        const float s = __uint_as_float(a) * F::TO_SUBNORMAL_UNITS;       // in units of the min subnormal
        const float lo = floorf(s);
        const float frac = s - lo;
        code = (uint32_t)lo + ((float)u24 < frac * 16777216.0f ? 1u : 0u);
    }
    return sign | code;
}

QMM_DEV uint32_t encode_int8_sr(float t, uint32_t u24)
{
    if (t != t) return 0u;
    const float a = fabsf(t);
    float r;
    if (a >= 127.0f) r = 127.0f;
    else {
        const float lo = floorf(a);
        const float frac = a - lo;
        r = lo + ((float)u24 < frac * 16777216.0f ? 1.0f : 0.0f);
    }
    const int q = (int)(__float_as_uint(t) >> 31 ? -r : r);
    return (uint32_t)q & 0xFFu;
}

template <int FMT, int MODE> QMM_DEV uint32_t encode(float t, uint32_t u24)
{
    if constexpr (MODE == QMM_ROUND_RTNE) {
        if constexpr (FMT == QMM_FMT_INT8) return encode_int8_rtne(t);
        else return encode_fp8_rtne<FMT>(t);
    } else {
        if constexpr (FMT == QMM_FMT_INT8) return encode_int8_sr(t, u24);
        else return encode_fp8_sr<FMT>(t, u24);
    }
}

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies
// with the Weyl key schedule.
struct Philox4 { uint32_t v[4]; };
QMM_DEV Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
        // one 32 x 32 -> 64 multiply per product (v_mad_u64_u32) instead of separate high and low halves: integer
        // multiplies issue at a quarter of the plain rate and are what bounds stochastic rounding
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    }
    return Philox4{{c0, c1, c2, c3}};
}

// 24 random bits of output element number g under key `seed`.
struct SrStream {
    uint64_t seed;
    uint64_t cached_block;
    Philox4 cached;
    bool valid;
    QMM_DEV explicit SrStream(uint64_t s) : seed(s), cached_block(0), cached{}, valid(false) {}
    QMM_DEV uint32_t bits(uint64_t g)
    {
        const uint64_t blk = g >> 2;
        if (!valid || blk != cached_block) {
            cached = philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), 0u, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
            cached_block = blk;
            valid = true;
        }
        // selected by compares: indexing the four words with a run-time index would put them in scratch memory
        const uint32_t j = (uint32_t)g & 3u;
        const uint32_t w = j == 0 ? cached.v[0] : j == 1 ? cached.v[1] : j == 2 ? cached.v[2] : cached.v[3];
        return w >> 8;
    }
};

// Step size from the magnitude bits of a group's absmax (Eq. 1): one IEEE
// division; zero group -> 1; quotient below 2^-126 raised to 2^-126.
QMM_DEV float delta_from_absmax_bits(uint32_t bits, float qmax)
{
    const float a = __uint_as_float(bits);
    float d = a / qmax;
    if (d < 0x1p-126f) d = 0x1p-126f;
    return bits == 0u ? 1.0f : d;
}

// ---------------------------------------------------------------------------
// Wavefront reductions (64 lanes) by shuffles.
// ---------------------------------------------------------------------------
QMM_DEV uint32_t wave_max_u32(uint32_t v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, off, kWave));
    return v;
}
QMM_DEV double wave_sum_f64(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}
QMM_DEV double wave_max_f64(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmax(v, __shfl_xor(v, off, kWave));
    return v;
}

// ---------------------------------------------------------------------------
// "The workgroup that arrives last folds the partial results": one launch per reduction instead of two.
// A call takes one slot (per reduced tensor) of a ring of arrival counters that live in the library's device
// image and are zero between calls; every workgroup publishes its partial result, counts itself in, and the one
// that completes the count folds all partials in a fixed order (so results do not depend on which one it is),
// then puts the counters back to zero.  Counting is in two levels -- workgroups of one residue class of
// blockIdx mod 8 (the XCD a workgroup runs on under round-robin dispatch) share a counter, the last of each class
// counts into the slot's first word -- so that no counter takes more than an eighth of the grid's arrivals, each in
// a cache line of its own.  The ring has kArrivalSlots slots handed out round robin: two calls can only meet on
// one slot if that many calls are issued while the first is still running.
// ---------------------------------------------------------------------------
constexpr int kArrivalSlots = 8192;
constexpr int kArrivalStride = 32;                       // words between the counters of a slot: 128 bytes
constexpr int kArrivalWords = 9 * kArrivalStride;        // per slot: the slot's counter + eight class counters
qmm_status arrival_slots(int count, uint32_t** first);   // host: `count` consecutive slots (qmm_api.hip)

// Partial results cross from one workgroup to another through device-coherent accesses (they bypass the per-XCD
// caches), not through fences: a release fence writes back the whole L2 of the XCD, and a thousand workgroups doing
// that cost more than the reduction itself.  publish_* stores and waits until the store has left the CU; the
// arrival is counted afterwards in program order; the last workgroup reads with coherent_load.
QMM_DEV void publish_u32(uint32_t* p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}
QMM_DEV void publish_f64(double* p, double v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}
QMM_DEV uint32_t coherent_load(const uint32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
QMM_DEV double coherent_load(const double* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Called by all threads of a workgroup after its partial results have been published; true, for every thread, in
// the one workgroup of the `total` that arrives last.
QMM_DEV bool arrive_last(uint32_t* slot, unsigned id, unsigned total)
{
    __shared__ int s_last;
    __syncthreads();                 // every publishing thread of the workgroup has waited for its store
    if (threadIdx.x == 0) {
        int last = 0;
        const unsigned cls = id & 7u, in_cls = (total - cls + 7u) >> 3, classes = total < 8u ? total : 8u;
        uint32_t* c = slot + (1 + cls) * kArrivalStride;
        if (__hip_atomic_fetch_add(c, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == in_cls - 1u) {
            __hip_atomic_store(c, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (__hip_atomic_fetch_add(slot, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == classes - 1u) {
                __hip_atomic_store(slot, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                last = 1;
            }
        }
        s_last = last;
    }
    __syncthreads();
    return s_last != 0;
}

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline qmm_status launch_status() { return hipGetLastError() == hipSuccess ? QMM_OK : QMM_ERR_LAUNCH; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace qmm
