// qmm_dequantize: the reduced-precision value of every quantized element (the v-tilde of Eq. 2): value of the
// code times the step size of its scale group, one binary32 multiply.  HBM-bound: 1 B read, 2 or 4 B written per
// element.  Codes [batch][rows][K] as qmm_quantize writes them; delta indexed the same way.
#include "qmm_device.h"

namespace qmm {
namespace {

constexpr int kThreads = 256;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Value of an FP8 code, by fields: sign, exponent (bias from the format), mantissa; exponent 0 is subnormal.
template <int FMT> QMM_DEV float decode_fp8(uint32_t code)
{
    using F = Fp8<FMT>;
    constexpr int E = 7 - F::M;
    const uint32_t sign = (code & 0x80u) << 24;
    const uint32_t e = (code >> F::M) & ((1u << E) - 1u), m = code & ((1u << F::M) - 1u);
    if (FMT == QMM_FMT_E4M3 ? ((code & 0x7Fu) == 0x7Fu) : (e == 31u && m != 0u)) return __uint_as_float(0x7FC00000u);
    if (FMT == QMM_FMT_E5M2 && e == 31u) return __uint_as_float(sign | 0x7F800000u);
    if (e == 0u) {
        const float v = (float)m * __uint_as_float((uint32_t)(127 + 1 - F::BIAS - F::M) << 23);   // m * 2^(1-bias-M)
        return __uint_as_float(__float_as_uint(v) | sign);
    }
    return __uint_as_float(sign | ((e + 127u - F::BIAS) << 23) | (m << (23 - F::M)));
}

template <int FMT> QMM_DEV float decode(uint32_t code)
{
    if constexpr (FMT == QMM_FMT_INT8) return (float)(int8_t)(uint8_t)code;
    else return decode_fp8<FMT>(code);
}

struct DArgs {
    const uint8_t* codes; const float* delta; void* out;
    int64_t rows, K, total_rows;      // total_rows = batch * rows
    int64_t groups; int64_t inner; int per_channel; int out_bf16;
};

// One thread per 16 consecutive codes of a row (K % 16 == 0), grid-stride.
template <int FMT> __global__ void __launch_bounds__(kThreads)
dequantize_vec(DArgs a)
{
    const int64_t vec_per_row = a.K >> 4;
    const int64_t nvec = a.total_rows * vec_per_row;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x; v < nvec; v += stride) {
        const int64_t row = v / vec_per_row;                       // b * rows + r
        const int64_t b = row / a.rows, r = row - b * a.rows;
        const float d = a.delta[((b / a.inner) % a.groups) * (a.per_channel ? a.rows : 1) + (a.per_channel ? r : 0)];
        const u32x4 w = reinterpret_cast<const u32x4*>(a.codes)[v];
        float y[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) y[i] = decode<FMT>((w[i >> 2] >> (8 * (i & 3))) & 0xFFu) * d;
        if (a.out_bf16) {
            typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
            typedef float f2 __attribute__((ext_vector_type(2)));
            uint32_t pk[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) pk[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{y[2 * i], y[2 * i + 1]}, bf2));
            u32x4* o = reinterpret_cast<u32x4*>(static_cast<uint16_t*>(a.out) + v * 16);
            o[0] = u32x4{pk[0], pk[1], pk[2], pk[3]};
            o[1] = u32x4{pk[4], pk[5], pk[6], pk[7]};
        } else {
            f32x4* o = reinterpret_cast<f32x4*>(static_cast<float*>(a.out) + v * 16);
#pragma unroll
            for (int q = 0; q < 4; ++q) o[q] = f32x4{y[4 * q], y[4 * q + 1], y[4 * q + 2], y[4 * q + 3]};
        }
    }
}

// Any K: one thread per element.
template <int FMT> __global__ void __launch_bounds__(kThreads)
dequantize_generic(DArgs a)
{
    const int64_t n = a.total_rows * a.K;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        const int64_t row = i / a.K;
        const int64_t b = row / a.rows, r = row - b * a.rows;
        const float d = a.delta[((b / a.inner) % a.groups) * (a.per_channel ? a.rows : 1) + (a.per_channel ? r : 0)];
        const float y = decode<FMT>(a.codes[i]) * d;
        if (a.out_bf16) static_cast<__bf16*>(a.out)[i] = (__bf16)y;
        else static_cast<float*>(a.out)[i] = y;
    }
}

template <int FMT> qmm_status launch(const DArgs& a, hipStream_t s)
{
    const int64_t n = a.total_rows * a.K;
    const bool vec = (a.K % 16 == 0) && aligned16(a.codes) && aligned16(a.out);
    const int64_t work = vec ? n / 16 : n;
    int64_t nb = (work + kThreads - 1) / kThreads;
    if (nb > 8192) nb = 8192;
    if (vec) dequantize_vec<FMT><<<(unsigned)nb, kThreads, 0, s>>>(a);
    else dequantize_generic<FMT><<<(unsigned)nb, kThreads, 0, s>>>(a);
    return launch_status();
}

}  // namespace
}  // namespace qmm

using namespace qmm;

extern "C" qmm_status qmm_dequantize(const uint8_t* codes, int64_t batch, int64_t rows, int64_t K, qmm_format fmt,
                                     const qmm_granularity* g, const float* delta, void* out, qmm_dtype out_dtype,
                                     void* stream)
{
    if (!g) return QMM_ERR_NULL;
    if (fmt != QMM_FMT_INT8 && fmt != QMM_FMT_E4M3 && fmt != QMM_FMT_E5M2) return QMM_ERR_ENUM;
    if (out_dtype != QMM_DT_BF16 && out_dtype != QMM_DT_F32) return QMM_ERR_ENUM;
    if (g->batch_groups < 1 || g->batch_inner < 0 || (g->per_channel != 0 && g->per_channel != 1)) return QMM_ERR_ENUM;
    if (batch < 0 || rows < 0 || K < 0) return QMM_ERR_SHAPE;
    if (batch * rows * K == 0) return QMM_OK;
    if (!codes || !delta || !out) return QMM_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(out) & (out_dtype == QMM_DT_BF16 ? 1u : 3u)) return QMM_ERR_ALIGN;
    DArgs a{codes, delta, out, rows, K, batch * rows, g->batch_groups, g->batch_inner > 0 ? g->batch_inner : 1,
            g->per_channel, out_dtype == QMM_DT_BF16};
    hipStream_t s = as_stream(stream);
    if (fmt == QMM_FMT_INT8) return launch<QMM_FMT_INT8>(a, s);
    if (fmt == QMM_FMT_E4M3) return launch<QMM_FMT_E4M3>(a, s);
    return launch<QMM_FMT_E5M2>(a, s);
}
