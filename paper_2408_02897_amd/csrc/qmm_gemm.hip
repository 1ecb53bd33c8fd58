// qmm_gemm: 8-bit x 8-bit matrix multiply in a wide accumulator followed by the
// descale (third Methodology bullet: scaling before and after the multiply, the
// result before re-scaling held by the multiply-accumulate unit's accumulator),
// plus the bfloat16 pass-through product used as the high-precision reference.
//
// Design (gfx950, wave64, MFMA):
//  * Workgroup = 4 wavefronts in a 2 x 2 grid; one wavefront owns 16*TM rows (m)
//    by 64*TG columns (n) of the output in registers.
//  * Operands are [rows][K] with K contiguous.  A K-slab of 128 bytes per row is
//    staged in LDS in "fragment blocks": 16 rows x 64 bytes = 1 KiB, lane l of a
//    wavefront owning the 16 bytes (row l%16, byte group l/16).  One
//    global_load_lds_dwordx4 per wavefront fills one block straight from global
//    memory (no staging registers), and one ds_read_b128 per lane reads a block
//    back with every lane on consecutive addresses, so reads are free of bank
//    conflicts by construction.
//  * A block is exactly one operand of v_mfma_i32_16x16x64_i8 or
//    v_mfma_f32_16x16x32_bf16; two blocks (the two 64-byte halves of the slab)
//    make one operand of v_mfma_f32_16x16x128_f8f6f4.  Which K bytes a lane holds
//    is the same for both operands, which is all a contraction needs.
//  * The B matrix (n) feeds the MFMA's first operand and A (m) the second, so a
//    lane ends up with 4 consecutive n of one m per MFMA.  The 16 rows of a B
//    block are picked so that the four MFMAs of a 64-column group give a lane 16
//    consecutive columns: stores are 32 (bf16) or 64 (fp32) contiguous bytes per
//    lane and whole 128-byte lines per row and wavefront.
//  * Two LDS stages; the slab for step k+1 is in flight while step k multiplies.
//  * Workgroup ids are spread so that each XCD (own L2) walks a compact band of
//    tiles.
#include <type_traits>

#include "qmm_device.h"

namespace qmm {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

enum Kind { KIND_I8 = 0, KIND_F8 = 1, KIND_BF16 = 2 };

constexpr int kThreads = 256;
constexpr int kSlabBytes = 128;      // K bytes per row per pipeline step
constexpr int kBlockBytes = 1024;    // one fragment block: 16 rows x 64 bytes
constexpr int kNumXcd = 8;

__device__ __attribute__((aligned(16))) const uint32_t g_zero16[4] = {0u, 0u, 0u, 0u};

struct GemmArgs {
    const uint8_t* a;        // [batch][M][rowbytes]
    const uint8_t* b;        // [batch][N][rowbytes]
    int64_t M, N, rowbytes;  // rowbytes = K * bytes per element
    int64_t batch;
    const float* da; const float* db;
    int64_t da_groups, db_groups;     // batch groups
    int da_per_channel, db_per_channel;
    void* y; int y_bf16;              // may be null
    void* acc_out;                    // may be null
    int tiles_m, tiles_n;
};

// LDS copy of 16 bytes per lane: lane l lands at lds_block + 16*l.
QMM_DEV void load_block_to_lds(const uint8_t* gptr, uint8_t* lds_block)
{
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    __builtin_amdgcn_global_load_lds((gptr_t)gptr, (lptr_t)lds_block, 16, 0, 0);
}

template <int KIND, int FA, int FB, int TM, int TG>
__global__ void __launch_bounds__(kThreads, 1)
gemm_kernel(GemmArgs g)
{
    constexpr int TN = 4 * TG;                 // 16-column MFMA tiles per wavefront
    constexpr int BM = 2 * 16 * TM;            // workgroup tile rows
    constexpr int BN = 2 * 64 * TG;            // workgroup tile columns
    constexpr int A_BLOCKS = BM / 16, B_BLOCKS = BN / 16;
    constexpr int STAGE_BYTES = (A_BLOCKS + B_BLOCKS) * 2 * kBlockBytes;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 15, lgrp = lane >> 4;

    // ---- workgroup id -> (batch, tile_m, tile_n), XCD-aware and grouped along m
    const int64_t tiles_per_batch = (int64_t)g.tiles_m * g.tiles_n;
    const int64_t total = tiles_per_batch * g.batch;
    int64_t pid = blockIdx.x;
    {
        const int64_t per = (total + kNumXcd - 1) / kNumXcd, tall = total % kNumXcd;
        const int64_t xcd = pid % kNumXcd, loc = pid / kNumXcd;
        pid = (tall == 0 || xcd < tall) ? xcd * per + loc : tall * per + (xcd - tall) * (per - 1) + loc;
    }
    const int64_t bidx = pid / tiles_per_batch;
    int64_t t = pid - bidx * tiles_per_batch;
    constexpr int GROUP_M = 8;
    const int64_t in_group = (int64_t)GROUP_M * g.tiles_n;
    const int64_t grp = t / in_group;
    const int64_t first_m = grp * GROUP_M;
    const int64_t gsz = min((int64_t)GROUP_M, g.tiles_m - first_m);
    const int64_t tile_m = first_m + (t - grp * in_group) % gsz;
    const int64_t tile_n = (t - grp * in_group) / gsz;
    const int64_t m0 = tile_m * BM, n0 = tile_n * BN;

    const uint8_t* A = g.a + bidx * g.M * g.rowbytes;
    const uint8_t* B = g.b + bidx * g.N * g.rowbytes;

    // ---- global sources of the blocks this wavefront copies: A row blocks wave*A_BLOCKS/4 .., same for B
    constexpr int A_PER_WAVE = A_BLOCKS / 4, B_PER_WAVE = B_BLOCKS / 4;
    const uint8_t* a_src[A_PER_WAVE];
    const uint8_t* b_src[B_PER_WAVE];
#pragma unroll
    for (int i = 0; i < A_PER_WAVE; ++i) {
        const int rb = wave * A_PER_WAVE + i;
        int64_t row = m0 + rb * 16 + lrow;
        row = row < g.M ? row : g.M - 1;
        a_src[i] = A + row * g.rowbytes + lgrp * 16;
    }
#pragma unroll
    for (int i = 0; i < B_PER_WAVE; ++i) {
        const int nb = wave * B_PER_WAVE + i;          // n block: 64-column group nb/4, MFMA tile nb%4
        int64_t row = n0 + (nb >> 2) * 64 + (lrow >> 2) * 16 + (nb & 3) * 4 + (lrow & 3);
        row = row < g.N ? row : g.N - 1;
        b_src[i] = B + row * g.rowbytes + lgrp * 16;
    }

    auto issue_loads = [&](int64_t k0, int stage) {
        uint8_t* sa = lds + stage * STAGE_BYTES;
        uint8_t* sb = sa + A_BLOCKS * 2 * kBlockBytes;
        const bool tail = k0 + kSlabBytes > g.rowbytes;   // uniform
        const uint8_t* zero = reinterpret_cast<const uint8_t*>(g_zero16);
#pragma unroll
        for (int piece = 0; piece < 2; ++piece) {
            const int64_t off = k0 + piece * 64;
            const bool oob = tail && (off + lgrp * 16 >= g.rowbytes);
#pragma unroll
            for (int i = 0; i < A_PER_WAVE; ++i) {
                const int rb = wave * A_PER_WAVE + i;
                load_block_to_lds(oob ? zero : a_src[i] + off, sa + (rb * 2 + piece) * kBlockBytes);
            }
#pragma unroll
            for (int i = 0; i < B_PER_WAVE; ++i) {
                const int nb = wave * B_PER_WAVE + i;
                load_block_to_lds(oob ? zero : b_src[i] + off, sb + (nb * 2 + piece) * kBlockBytes);
            }
        }
    };

    using AccT = typename std::conditional<KIND == KIND_I8, v4i, v4f>::type;
    AccT acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = AccT{0, 0, 0, 0};

    const int64_t nk = (g.rowbytes + kSlabBytes - 1) / kSlabBytes;
    issue_loads(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int64_t kt = 0; kt < nk; ++kt) {
        const int stage = (int)(kt & 1);
        if (kt + 1 < nk) issue_loads((kt + 1) * kSlabBytes, stage ^ 1);

        const uint8_t* sa = lds + stage * STAGE_BYTES + (wm * (A_BLOCKS / 2)) * 2 * kBlockBytes + lane * 16;
        const uint8_t* sb = lds + stage * STAGE_BYTES + A_BLOCKS * 2 * kBlockBytes +
                            (wn * (B_BLOCKS / 2)) * 2 * kBlockBytes + lane * 16;
        if constexpr (KIND == KIND_F8) {
            v8i fb[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const v4i p0 = *reinterpret_cast<const v4i*>(sb + (j * 2 + 0) * kBlockBytes);
                const v4i p1 = *reinterpret_cast<const v4i*>(sb + (j * 2 + 1) * kBlockBytes);
                fb[j] = v8i{p0[0], p0[1], p0[2], p0[3], p1[0], p1[1], p1[2], p1[3]};
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const v4i p0 = *reinterpret_cast<const v4i*>(sa + (i * 2 + 0) * kBlockBytes);
                const v4i p1 = *reinterpret_cast<const v4i*>(sa + (i * 2 + 1) * kBlockBytes);
                const v8i fa = v8i{p0[0], p0[1], p0[2], p0[3], p1[0], p1[1], p1[2], p1[3]};
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                        fb[j], fa, acc[i][j], FB == QMM_FMT_E5M2 ? 1 : 0, FA == QMM_FMT_E5M2 ? 1 : 0, 0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int piece = 0; piece < 2; ++piece) {
                v4i fb[TN];
#pragma unroll
                for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const v4i*>(sb + (j * 2 + piece) * kBlockBytes);
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const v4i fa = *reinterpret_cast<const v4i*>(sa + (i * 2 + piece) * kBlockBytes);
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        if constexpr (KIND == KIND_I8)
                            acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fb[j], fa, acc[i][j], 0, 0, 0);
                        else
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(v8bf, fb[j]), __builtin_bit_cast(v8bf, fa), acc[i][j], 0, 0, 0);
                    }
                }
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }

    // ---- epilogue: lane (lgrp, lrow) holds, for row block i and column group gq, the 16 columns
    //      n = n_base + gq*64 + lgrp*16 + [0,16) of row m = m_base + i*16 + lrow.
    const int64_t m_base = m0 + wm * (BM / 2), n_base = n0 + wn * (BN / 2);
    const float* da = g.da ? g.da + (bidx % g.da_groups) * (g.da_per_channel ? g.M : 1) : nullptr;
    const float* db = g.db ? g.db + (bidx % g.db_groups) * (g.db_per_channel ? g.N : 1) : nullptr;
    const bool descale = (KIND != KIND_BF16);
    const bool vec_ok = (g.N % 16) == 0;
    float sa_scalar = 1.0f, sb_scalar = 1.0f;
    if (descale) {
        if (!g.da_per_channel) sa_scalar = da[0];
        if (!g.db_per_channel) sb_scalar = db[0];
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int64_t m = m_base + i * 16 + lrow;
        if (m >= g.M) continue;
        const float sl = (descale && g.da_per_channel) ? da[m] : sa_scalar;
#pragma unroll
        for (int gq = 0; gq < TG; ++gq) {
            const int64_t n = n_base + gq * 64 + lgrp * 16;
            if (n >= g.N) continue;
            const int64_t o = (bidx * g.M + m) * g.N + n;
            float v[16];
            uint32_t raw[16];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int c = j * 4 + r;
                    float a;
                    if constexpr (KIND == KIND_I8) {
                        raw[c] = (uint32_t)acc[i][gq * 4 + j][r];
                        a = (float)acc[i][gq * 4 + j][r];
                    } else {
                        a = acc[i][gq * 4 + j][r];
                        raw[c] = __float_as_uint(a);
                    }
                    if (descale) {
                        const float sr = g.db_per_channel ? db[(n + c) < g.N ? (n + c) : (g.N - 1)] : sb_scalar;
                        a = (a * sl) * sr;
                    }
                    v[c] = a;
                }
            if (vec_ok) {
                if (g.acc_out) {
                    u32x4* dst = reinterpret_cast<u32x4*>(static_cast<uint32_t*>(g.acc_out) + o);
#pragma unroll
                    for (int q = 0; q < 4; ++q) dst[q] = u32x4{raw[4 * q], raw[4 * q + 1], raw[4 * q + 2], raw[4 * q + 3]};
                }
                if (g.y) {
                    if (g.y_bf16) {
                        uint32_t pk[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
                            typedef float f2 __attribute__((ext_vector_type(2)));
                            const bf2 h = __builtin_convertvector(f2{v[2 * q], v[2 * q + 1]}, bf2);
                            pk[q] = __builtin_bit_cast(uint32_t, h);
                        }
                        u32x4* dst = reinterpret_cast<u32x4*>(static_cast<uint16_t*>(g.y) + o);
                        dst[0] = u32x4{pk[0], pk[1], pk[2], pk[3]};
                        dst[1] = u32x4{pk[4], pk[5], pk[6], pk[7]};
                    } else {
                        u32x4* dst = reinterpret_cast<u32x4*>(static_cast<float*>(g.y) + o);
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            dst[q] = u32x4{__float_as_uint(v[4 * q]), __float_as_uint(v[4 * q + 1]),
                                           __float_as_uint(v[4 * q + 2]), __float_as_uint(v[4 * q + 3])};
                    }
                }
            } else {
#pragma unroll
                for (int c = 0; c < 16; ++c) {
                    if (n + c >= g.N) break;
                    if (g.acc_out) static_cast<uint32_t*>(g.acc_out)[o + c] = raw[c];
                    if (g.y) {
                        if (g.y_bf16) static_cast<__bf16*>(g.y)[o + c] = (__bf16)v[c];
                        else static_cast<float*>(g.y)[o + c] = v[c];
                    }
                }
            }
        }
    }
}

template <int KIND, int FA, int FB, int TM, int TG>
qmm_status launch_tile(GemmArgs& g, hipStream_t s)
{
    constexpr int BM = 2 * 16 * TM, BN = 2 * 64 * TG;
    constexpr int STAGE_BYTES = (BM / 16 + BN / 16) * 2 * kBlockBytes;
    constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    g.tiles_m = (int)((g.M + BM - 1) / BM);
    g.tiles_n = (int)((g.N + BN - 1) / BN);
    const int64_t total = (int64_t)g.tiles_m * g.tiles_n * g.batch;
    if (total > 0x7FFFFFFF) return QMM_ERR_UNSUPPORTED;
    auto kern = gemm_kernel<KIND, FA, FB, TM, TG>;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess)
            return QMM_ERR_LAUNCH;
        attr_set = true;
    }
    kern<<<(unsigned)total, kThreads, LDS_BYTES, s>>>(g);
    return launch_status();
}

template <int KIND, int FA, int FB>
qmm_status launch_kind(GemmArgs& g, hipStream_t s)
{
    // 256 x 256 tiles when they still give every CU work, else 128 x 128.
    const int64_t big = ((g.M + 255) / 256) * ((g.N + 255) / 256) * g.batch;
    if (big >= 192) return launch_tile<KIND, FA, FB, 8, 2>(g, s);
    return launch_tile<KIND, FA, FB, 4, 1>(g, s);
}

bool is8(int f) { return f == QMM_FMT_INT8 || f == QMM_FMT_E4M3 || f == QMM_FMT_E5M2; }

qmm_status check_operand(const qmm_operand* o)
{
    if (!o) return QMM_ERR_NULL;
    if (!is8(o->format) && o->format != QMM_FMT_BF16) return QMM_ERR_ENUM;
    if (o->is_codes != 0 && o->is_codes != 1) return QMM_ERR_ENUM;
    if (o->format == QMM_FMT_BF16 && o->is_codes) return QMM_ERR_ENUM;
    if (o->gran.batch_groups < 1 || o->gran.reserved != 0 || (o->gran.per_channel != 0 && o->gran.per_channel != 1))
        return QMM_ERR_ENUM;
    return QMM_OK;
}

}  // namespace
}  // namespace qmm

using namespace qmm;

extern "C" size_t qmm_gemm_workspace_size(const qmm_operand*, const qmm_operand*, int64_t, int64_t, int64_t, int64_t)
{
    return 0;
}

extern "C" qmm_status qmm_gemm(const qmm_operand* a, const qmm_operand* b, int64_t batch, int64_t M, int64_t N, int64_t K,
                               void* y, qmm_dtype y_dtype, void* acc_out, void* workspace, size_t workspace_bytes,
                               void* stream)
{
    (void)workspace; (void)workspace_bytes;
    qmm_status st = check_operand(a);
    if (st != QMM_OK) return st;
    st = check_operand(b);
    if (st != QMM_OK) return st;
    if (y_dtype != QMM_DT_BF16 && y_dtype != QMM_DT_F32) return QMM_ERR_ENUM;
    if (batch < 0 || M < 0 || N < 0 || K < 0) return QMM_ERR_SHAPE;
    const bool bf = a->format == QMM_FMT_BF16;
    if (bf != (b->format == QMM_FMT_BF16)) return QMM_ERR_UNSUPPORTED;
    if (!bf && ((a->format == QMM_FMT_INT8) != (b->format == QMM_FMT_INT8))) return QMM_ERR_UNSUPPORTED;
    if (!bf && (!a->is_codes || !b->is_codes)) return QMM_ERR_UNSUPPORTED;   // quantize-on-load: not in this build yet
    if (!y && !acc_out) return QMM_ERR_NULL;
    if (batch * M * N == 0) return QMM_OK;
    if (!bf && (!a->delta || !b->delta)) return QMM_ERR_NULL;
    const int64_t esz = bf ? 2 : 1;
    if ((K * esz) % 16 != 0) return QMM_ERR_ALIGN;
    if (K > 0 && (!a->data || !b->data)) return QMM_ERR_NULL;
    if (!aligned16(a->data) || !aligned16(b->data) || (y && !aligned16(y)) || (acc_out && !aligned16(acc_out)))
        return QMM_ERR_ALIGN;

    GemmArgs g{};
    g.a = static_cast<const uint8_t*>(a->data); g.b = static_cast<const uint8_t*>(b->data);
    g.M = M; g.N = N; g.rowbytes = K * esz; g.batch = batch;
    g.da = bf ? nullptr : a->delta; g.db = bf ? nullptr : b->delta;
    g.da_groups = a->gran.batch_groups; g.db_groups = b->gran.batch_groups;
    g.da_per_channel = a->gran.per_channel; g.db_per_channel = b->gran.per_channel;
    g.y = y; g.y_bf16 = y_dtype == QMM_DT_BF16; g.acc_out = acc_out;
    hipStream_t s = as_stream(stream);

    if (bf) return launch_kind<KIND_BF16, QMM_FMT_BF16, QMM_FMT_BF16>(g, s);
    if (a->format == QMM_FMT_INT8) return launch_kind<KIND_I8, QMM_FMT_INT8, QMM_FMT_INT8>(g, s);
    if (a->format == QMM_FMT_E4M3 && b->format == QMM_FMT_E4M3) return launch_kind<KIND_F8, QMM_FMT_E4M3, QMM_FMT_E4M3>(g, s);
    if (a->format == QMM_FMT_E4M3) return launch_kind<KIND_F8, QMM_FMT_E4M3, QMM_FMT_E5M2>(g, s);
    if (b->format == QMM_FMT_E4M3) return launch_kind<KIND_F8, QMM_FMT_E5M2, QMM_FMT_E4M3>(g, s);
    return launch_kind<KIND_F8, QMM_FMT_E5M2, QMM_FMT_E5M2>(g, s);
}
