// qmm_mfma_rate: a measurement aid, not a step of the method.  Every wavefront keeps ten operand fragments in
// registers and issues matrix instructions on them back to back, with no memory traffic in the loop: the rate at
// which this runs is what the matrix units sustain for THESE operand bytes.  It depends on the bytes: the chip's
// clock under matrix load is set by power, and operands with many toggling bits draw more of it than constant
// ones, so the sustained rate for quantized activations is well below the datasheet figure quoted at the top
// clock.  The quantized-GEMM kernel is judged against both.
#include "qmm_device.h"

namespace qmm {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// One workgroup of four wavefronts per CU (one per SIMD), accumulators in AGPRs, as in the GEMM kernel.
template <bool F8, int FA, int FB>
__global__ void __launch_bounds__(256, 1)
mfma_rate_kernel(const uint8_t* __restrict__ operand_bytes, int64_t nbytes, int64_t rounds, float* __restrict__ sink)
{
    using Frag = typename std::conditional<F8, v8i, v4i>::type;
    using AccT = typename std::conditional<F8, v4f, v16i>::type;
    constexpr int NA = 2, NB = F8 ? 8 : 4, NACC_A = F8 ? 8 : 4;       // 64 (FP8) or 16 (INT8) accumulator blocks
    constexpr int FRAG_BYTES = F8 ? 32 : 16;
    Frag fa[NA], fb[NB];
    // fragments: consecutive FRAG_BYTES pieces of the operand buffer, a different window per lane and workgroup
    const int64_t pieces = nbytes / FRAG_BYTES;
    const int64_t first = ((int64_t)blockIdx.x * 256 + threadIdx.x) * (NA + NB);
#pragma unroll
    for (int i = 0; i < NA; ++i) fa[i] = *reinterpret_cast<const Frag*>(operand_bytes + ((first + i) % pieces) * FRAG_BYTES);
#pragma unroll
    for (int j = 0; j < NB; ++j) fb[j] = *reinterpret_cast<const Frag*>(operand_bytes + ((first + NA + j) % pieces) * FRAG_BYTES);
    AccT acc[NACC_A][NB];
#pragma unroll
    for (int i = 0; i < NACC_A; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int e = 0; e < (F8 ? 4 : 16); ++e) acc[i][j][e] = 0;
    asm volatile("s_nop 7" ::: "memory");
    for (int64_t r = 0; r < rounds; ++r) {
#pragma unroll
        for (int i = 0; i < NACC_A; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j) {
#if defined(__HIP_DEVICE_COMPILE__)
                if constexpr (F8) {
                    if constexpr (FA == QMM_FMT_E5M2 && FB == QMM_FMT_E5M2)
                        asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:1 blgp:1" : "+a"(acc[i][j]) : "v"(fa[i & 1]), "v"(fb[j]));
                    else if constexpr (FA == QMM_FMT_E5M2)
                        asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:1" : "+a"(acc[i][j]) : "v"(fa[i & 1]), "v"(fb[j]));
                    else if constexpr (FB == QMM_FMT_E5M2)
                        asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 blgp:1" : "+a"(acc[i][j]) : "v"(fa[i & 1]), "v"(fb[j]));
                    else
                        asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fa[i & 1]), "v"(fb[j]));
                } else {
                    asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fa[i & 1]), "v"(fb[j]));
                }
#endif
            }
    }
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NACC_A; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) s += (float)acc[i][j][0];
    sink[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// qmm_hbm_rate: the other measurement aid -- what a plain streaming kernel reaches on this part, against which the
// scale / quantize / metric passes are read next to the datasheet's 8 TB/s.  Every thread keeps four 16-byte loads in
// flight per trip and the grid sweeps the buffer front to back (the access pattern of the absmax kernel); with a
// destination the vectors are stored as they arrive (a copy), without one they are folded into one word per thread.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256)
hbm_rate_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t nvec, uint32_t* __restrict__ sink)
{
    const int64_t stride = (int64_t)gridDim.x * 1024;
    u32x4 f = {0u, 0u, 0u, 0u};
    for (int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x; base < nvec; base += stride) {
        u32x4 v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t idx = base + i * 256;
            v[i] = idx < nvec ? __builtin_nontemporal_load(src + idx) : f;
        }
        if (dst) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t idx = base + i * 256;
                if (idx < nvec) __builtin_nontemporal_store(v[i], dst + idx);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) f |= v[i];
        }
    }
    if (!dst) sink[(int64_t)blockIdx.x * 256 + threadIdx.x] = f[0] | f[1] | f[2] | f[3];
}

}  // namespace
}  // namespace qmm

using namespace qmm;

extern "C" qmm_status qmm_hbm_rate(const void* src, void* dst, int64_t nbytes, int32_t workgroups, uint32_t* sink, void* stream)
{
    if (!src || (!dst && !sink)) return QMM_ERR_NULL;
    if (nbytes < 0 || workgroups < 1) return QMM_ERR_SHAPE;
    if (nbytes % 16 != 0 || !aligned16(src) || (dst && !aligned16(dst))) return QMM_ERR_ALIGN;
    if (nbytes == 0) return QMM_OK;
    hbm_rate_kernel<<<workgroups, 256, 0, as_stream(stream)>>>(static_cast<const u32x4*>(src), static_cast<u32x4*>(dst),
                                                              nbytes / 16, sink);
    return launch_status();
}

extern "C" qmm_status qmm_mfma_rate(qmm_format a_format, qmm_format b_format, const void* operand_bytes, int64_t nbytes,
                                    int64_t rounds, int32_t workgroups, float* sink, double* flops_out, void* stream)
{
    if (!operand_bytes || !sink || !flops_out) return QMM_ERR_NULL;
    const bool i8 = a_format == QMM_FMT_INT8;
    if (i8 != (b_format == QMM_FMT_INT8)) return QMM_ERR_UNSUPPORTED;
    if (!i8 && !((a_format == QMM_FMT_E4M3 || a_format == QMM_FMT_E5M2) && (b_format == QMM_FMT_E4M3 || b_format == QMM_FMT_E5M2)))
        return QMM_ERR_ENUM;
    if (nbytes < 32 || rounds < 0 || workgroups < 1) return QMM_ERR_SHAPE;
    if (!aligned16(operand_bytes) || (reinterpret_cast<uintptr_t>(operand_bytes) & 31u)) return QMM_ERR_ALIGN;
    hipStream_t s = as_stream(stream);
    const uint8_t* p = static_cast<const uint8_t*>(operand_bytes);
    // per matrix instruction: 2 * 16 * 16 * 128 (FP8) or 2 * 32 * 32 * 32 (INT8) operations, 64 or 16 per round
    const double per_wave_round = i8 ? 16.0 * 2 * 32 * 32 * 32 : 64.0 * 2 * 16 * 16 * 128;
    *flops_out = per_wave_round * (double)rounds * 4.0 * (double)workgroups;
    if (i8) mfma_rate_kernel<false, QMM_FMT_INT8, QMM_FMT_INT8><<<workgroups, 256, 0, s>>>(p, nbytes, rounds, sink);
    else if (a_format == QMM_FMT_E4M3 && b_format == QMM_FMT_E4M3) mfma_rate_kernel<true, QMM_FMT_E4M3, QMM_FMT_E4M3><<<workgroups, 256, 0, s>>>(p, nbytes, rounds, sink);
    else if (a_format == QMM_FMT_E4M3) mfma_rate_kernel<true, QMM_FMT_E4M3, QMM_FMT_E5M2><<<workgroups, 256, 0, s>>>(p, nbytes, rounds, sink);
    else if (b_format == QMM_FMT_E4M3) mfma_rate_kernel<true, QMM_FMT_E5M2, QMM_FMT_E4M3><<<workgroups, 256, 0, s>>>(p, nbytes, rounds, sink);
    else mfma_rate_kernel<true, QMM_FMT_E5M2, QMM_FMT_E5M2><<<workgroups, 256, 0, s>>>(p, nbytes, rounds, sink);
    return launch_status();
}
