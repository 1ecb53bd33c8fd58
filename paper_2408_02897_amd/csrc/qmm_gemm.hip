// qmm_gemm: 8-bit x 8-bit matrix multiply in a wide accumulator followed by the
// descale (third Methodology bullet: scaling before and after the multiply, the
// result before re-scaling held by the multiply-accumulate unit's accumulator),
// plus the bfloat16 pass-through product used as the high-precision reference.
//
// Design (gfx950, wave64, MFMA):
//  * Workgroup = 2 x NWN wavefronts; one wavefront owns 32*TM rows (m) by 64*TG
//    columns (n) of the output in accumulator registers.  Large tile: 256 x 256,
//    eight wavefronts of 128 x 64 (128 AGPRs each), two per SIMD; small tile:
//    128 x 128, four wavefronts.
//  * Operands are [rows][K] with K contiguous.  A K-slab of 128 bytes per row is
//    staged in LDS as plain 128-byte rows; the 16-byte chunk c of LDS row p sits
//    at chunk position c ^ ((p >> 1) & 7).  global_load_lds_dwordx4 copies
//    straight from global memory into LDS (no staging registers): one
//    instruction moves 8 rows x 128 bytes, so every 8 lanes read one whole
//    128-byte line of a row (the pattern the texture path handles best) and the
//    XOR is applied to the global chunk a lane fetches.  With that swizzle the
//    16 or 32 lanes of an MFMA operand that read the same logical chunk of
//    consecutive rows hit distinct banks (measured: same rate as linear reads).
//  * FP8 uses v_mfma_f32_16x16x128_f8f6f4; INT8 uses v_mfma_i32_32x32x32_i8 and
//    bfloat16 v_mfma_f32_32x32x16_bf16 (measured on this part: the 16x16 forms of
//    those two issue at ~60 % of the 32x32 rate).  Which K bytes a lane holds is
//    the same for both operands, which is all a contraction needs.
//  * The A matrix (m) feeds the MFMA's first operand and B (n) the second, so a
//    lane ends up holding several n of one m.  The rows of a B block are picked
//    from global memory in a permuted order such that a lane's values are TILES_N
//    consecutive columns: stores are 8 or 16 contiguous bytes per lane and whole
//    128-byte lines per row across the lanes.
//  * LDS holds a ring of three A slabs and two B slabs; the B fragments of the
//    current slab sit in registers for the whole K step.  One barrier per step;
//    copies are requested one at a time between matrix instructions.
//  * Workgroup ids are spread so that each XCD (own L2) walks a compact band of
//    tiles.
//  * Long K with few tiles: split-K with a second, fixed-order reduction kernel.
//    Outputs at most 64 wide or high: gemm_direct_kernel (no LDS).
//    Contractions of one slab at most with many whole tiles: gemm_shortk_kernel;
//    several whole tiles per CU and one step size per operand: gemm_stream_kernel
//    (both: workgroups that stay on their CU and overlap a tile's stores with the
//    next tile's work).
#include <atomic>
#include <type_traits>

#include <cstdlib>
#include "qmm_device.h"

namespace qmm {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

enum Kind { KIND_I8 = 0, KIND_F8 = 1, KIND_BF16 = 2 };

constexpr int kWavesM = 2;                 // wavefronts along M in a workgroup (along N: template parameter)
constexpr int kASlots = 3, kBSlots = 2;   // LDS ring depths of the two operands
constexpr int kSlabBytes = 128;      // K bytes per row per pipeline step = one LDS row
constexpr int kNumXcd = 8;


struct GemmArgs {
    const uint8_t* a;        // [batch][M][rowbytes]
    const uint8_t* b;        // [batch][N][rowbytes]
    int64_t M, N, rowbytes;  // rowbytes = K * bytes per element
    int64_t batch;
    const float* da; const float* db;
    int64_t da_groups, db_groups;     // batch groups
    int64_t da_inner, db_inner;       // consecutive matrices sharing a group: group = (b / inner) % groups
    int da_per_channel, db_per_channel;
    void* y; int y_bf16;              // may be null
    void* acc_out;                    // may be null
    int tiles_m, tiles_n;
    int direct_along_n;               // gemm_direct_kernel: the workgroup's four wavefronts lie along n (else along m)
    int splits;                       // split-K: workgroups per output tile (1 = none); partial sums go to `partial`
    void* partial;                    // [splits][batch][M][N] raw accumulators (int32 / float)
    const float* nsr_ref;             // NSR variant: high-precision product [batch][M][N], else null
    double* nsr_partial;              // NSR variant: per wavefront {sum (y - ref)^2, sum ref^2}
    double* nsr_out;                  // NSR variant: the two folded sums
    int stagger;                      // gemm_stream_kernel: every other workgroup of an XCD starts this many sleeps late
};

// 16 bytes per lane from global memory into LDS: lane l lands at lds_unit + 16*l.
QMM_DEV void dma16(const uint8_t* gptr, uint8_t* lds_unit)
{
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    __builtin_amdgcn_global_load_lds((gptr_t)gptr, (lptr_t)lds_unit, 16, 0, 0);
}

// The same copy with the source given as a wavefront-uniform base plus a 32-bit byte offset per lane, and the LDS
// unit as a wavefront-uniform LDS address: one scalar move and the copy instruction, no vector address arithmetic.
// Issued this way a copy costs the wavefront about ten cycles; with a 64-bit vector address and the LDS address
// taken through a lane read it costs several times that, and sixteen of them in a row held up the matrix
// instructions for longer than a whole A block takes.
QMM_DEV void dma16_uniform(const uint8_t* base, uint32_t lane_offset, uint32_t lds_unit_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_unit_addr), "v"(lane_offset), "s"(base) : "memory", "m0");
}

// s_waitcnt with a compile-time count of vector-memory operations that may remain outstanding
template <int N> QMM_DEV void wait_vm()
{
    static_assert(N >= 0 && N <= 63, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
template <int N> QMM_DEV void wait_vm_lgkm()
{
    static_assert(N >= 0 && N <= 63, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"(N) : "memory");
}

// The matrix instructions below are inline assembly, so the compiler does not know that they read the accumulator
// registers as MFMA operands: left alone it sinks the zero initialisation (v_accvgpr_write) to just in front of
// the first such statement that uses a block, closer than the wait states an MFMA needs after such a write.  An
// empty volatile statement with every block as an in-out AGPR operand makes the initialisation happen here;
// volatile statements keep their order, so the s_nop that follows it really separates the two.
template <typename AccT, int NI, int NJ> QMM_DEV void pin_accumulators(AccT (&acc)[NI][NJ])
{
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) asm volatile("" : "+a"(acc[i][j]));
#endif
}

// FUSE: bit 0 / bit 1 = the A / B operand arrives as bfloat16 values and is quantized (RTNE, with its step sizes)
// while it is staged into LDS; otherwise it arrives as 8-bit codes and is copied by LDS-DMA.
// NWN: wavefronts along N (2 or 4): the workgroup has 2 x NWN wavefronts, NWN / 2 on every SIMD.
// NSR: the epilogue also reads the high-precision product and accumulates, per wavefront and in binary64, the two
// sums of the noise-to-signal ratio over the values it stores (y as rounded to the output type): sum (y - ref)^2
// and sum ref^2, elements whose error is NaN left out as in qmm_metric.  No second pass over Y.
template <int KIND, int FA, int FB, int TM, int TG, int NWN, int FUSE, int NSR = 0>
__global__ void __launch_bounds__(64 * kWavesM * NWN, 1)
gemm_kernel(GemmArgs g)
{
    constexpr bool F8 = (KIND == KIND_F8);
    constexpr bool FUSE_A = (FUSE & 1) != 0, FUSE_B = (FUSE & 2) != 0;
    static_assert(FUSE == 0 || KIND != KIND_BF16, "only 8-bit operands are quantized on load");
    constexpr int NWAVES = kWavesM * NWN;
    constexpr int BM = kWavesM * 32 * TM;      // workgroup tile rows
    constexpr int BN = NWN * 64 * TG;          // workgroup tile columns
    constexpr int WM = 32 * TM, WN = 64 * TG;  // wavefront tile
    constexpr int R = F8 ? 16 : 32;            // rows of one MFMA operand block
    constexpr int BLOCKS_M = WM / R;           // A blocks per wavefront
    constexpr int TILES_N = WN / R;            // B blocks per wavefront
    constexpr int KS = F8 ? 1 : 4;             // MFMA K slices per 128-byte slab
    constexpr int A_SLOT = BM * kSlabBytes, B_SLOT = BN * kSlabBytes;   // one K slab of A / of B in LDS
    constexpr int B_BASE = kASlots * A_SLOT;                            // LDS: kASlots A slabs, then kBSlots B slabs
    constexpr int A_UNITS = BM / 8, B_UNITS = BN / 8;          // DMA units of 8 LDS rows
    constexpr int A_PER_WAVE = A_UNITS / NWAVES, B_PER_WAVE = B_UNITS / NWAVES;
    static_assert(BLOCKS_M % 2 == 0, "A fragments ping-pong between two register sets");
    static_assert(A_PER_WAVE % 2 == 0 && B_PER_WAVE % 2 == 0, "a wavefront's units start on an even LDS row pair");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: kept in a scalar register
    const int wm = wave / NWN, wn = wave % NWN;

    // ---- workgroup id -> (batch, tile_m, tile_n), XCD-aware and grouped along m
    // (all in 32-bit unsigned arithmetic: the host rejects launches of 2^31 workgroups or more, and 64-bit
    // divisions cost a few hundred instructions each, which counts when a workgroup's own work is small)
    const uint32_t tiles_per_batch = (uint32_t)g.tiles_m * (uint32_t)g.tiles_n;
    const uint32_t total_tiles = tiles_per_batch * (uint32_t)g.batch;
    const uint32_t total = total_tiles * (uint32_t)g.splits;
    uint32_t pid = blockIdx.x;
    {
        const uint32_t per = (total + kNumXcd - 1) / kNumXcd, tall = total % kNumXcd;
        const uint32_t xcd = pid % kNumXcd, loc = pid / kNumXcd;
        pid = (tall == 0 || xcd < tall) ? xcd * per + loc : tall * per + (xcd - tall) * (per - 1) + loc;
    }
    // the divisions run on the vector unit; their results are the same in every lane and are moved to scalar
    // registers, so that everything derived from them (tile base addresses above all) is scalar as well
    // split-K: consecutive workgroups (same XCD) work on neighbouring tiles of the same K range
    const int split = __builtin_amdgcn_readfirstlane((int)(pid / total_tiles));
    pid -= (uint32_t)split * total_tiles;
    const int64_t bidx = __builtin_amdgcn_readfirstlane((int)(pid / tiles_per_batch));
    const uint32_t t = pid - (uint32_t)bidx * tiles_per_batch;
    constexpr uint32_t GROUP_M = 8;
    const uint32_t in_group = GROUP_M * (uint32_t)g.tiles_n;
    const uint32_t grp = t / in_group;
    const uint32_t first_m = grp * GROUP_M;
    const uint32_t gsz = min(GROUP_M, (uint32_t)g.tiles_m - first_m);
    const int64_t tile_m = __builtin_amdgcn_readfirstlane((int)(first_m + (t - grp * in_group) % gsz));
    const int64_t tile_n = __builtin_amdgcn_readfirstlane((int)((t - grp * in_group) / gsz));
    const int64_t m0 = tile_m * BM, n0 = tile_n * BN;

    constexpr int A_ES = FUSE_A ? 2 : 1, B_ES = FUSE_B ? 2 : 1;   // source bytes per K byte of codes
    const uint8_t* A = g.a + bidx * g.M * g.rowbytes * A_ES;
    const uint8_t* B = g.b + bidx * g.N * g.rowbytes * B_ES;

    // ---- DMA sources.  Unit u = LDS rows 8u..8u+7; lane l fills row 8u + l/8, chunk position l%8, i.e. fetches
    //      logical chunk (l%8) ^ ((row>>1)&7) of the global row parked there.  LDS row p of the B region holds
    //      output column  WN*(p/WN) + TILES_N*(p%R) + (p/R)%TILES_N : MFMA block t, lane j  <->  column TILES_N*j + t,
    //      so that in the accumulators a lane owns TILES_N consecutive columns of a row.
    //      Sources are kept as 32-bit byte offsets from the tile's first A / B row.
    // K range of this workgroup in bytes of codes: whole slabs, the last split takes the ragged end
    int k_begin = 0, k_end = (int)g.rowbytes;
    if (g.splits > 1) {
        const int nslabs = ((int)g.rowbytes + kSlabBytes - 1) / kSlabBytes;
        const int base = nslabs / g.splits, rem = nslabs % g.splits;
        const int first = split * base + min(split, rem);
        k_begin = first * kSlabBytes;
        k_end = min((int)g.rowbytes, (first + base + (split < rem ? 1 : 0)) * kSlabBytes);
    }
    const uint8_t* a_tile = A + (m0 * g.rowbytes + k_begin) * A_ES;
    const uint8_t* b_tile = B + (n0 * g.rowbytes + k_begin) * B_ES;
    uint32_t a_src[A_PER_WAVE], b_src[B_PER_WAVE];
    const int lane_chunk_base = lane & 7;
#pragma unroll
    for (int i = 0; i < A_PER_WAVE; ++i) {
        const int p = (wave * A_PER_WAVE + i) * 8 + (lane >> 3);
        const int c = lane_chunk_base ^ ((p >> 1) & 7);
        int64_t row = p;
        row = m0 + row < g.M ? row : g.M - 1 - m0;
        a_src[i] = (uint32_t)((row * g.rowbytes + c * 16) * A_ES);
    }
#pragma unroll
    for (int i = 0; i < B_PER_WAVE; ++i) {
        const int p = (wave * B_PER_WAVE + i) * 8 + (lane >> 3);
        const int c = lane_chunk_base ^ ((p >> 1) & 7);
        int64_t row = WN * (p / WN) + TILES_N * (p % R) + (p / R) % TILES_N;
        row = n0 + row < g.N ? row : g.N - 1 - n0;
        b_src[i] = (uint32_t)((row * g.rowbytes + c * 16) * B_ES);
    }

    // Copy number i of this wavefront for the A (B) slab at byte k0 into ring slot `slot`.
    typedef __attribute__((address_space(3))) uint8_t* lds_ptr_t;
    const uint32_t lds_a_units = (uint32_t)(uintptr_t)(lds_ptr_t)(lds + wave * A_PER_WAVE * 1024);
    const uint32_t lds_b_units = (uint32_t)(uintptr_t)(lds_ptr_t)(lds + B_BASE + wave * B_PER_WAVE * 1024);
    // A partial last slab (K not a multiple of the slab width): lanes whose 16-byte chunk lies past the end of the
    // row write zeros to their place in LDS, the others copy as usual with those lanes masked off.
    const int rowbytes = k_end - k_begin;       // bytes of K this workgroup contracts over (g.rowbytes <= 2^22: host check)
    auto copy_unit = [&](const uint8_t* base, uint32_t lane_offset, uint32_t lds_unit_addr, uint8_t* lds_unit, int chunk,
                         int k0) {
        if (k0 + kSlabBytes <= rowbytes) {
            dma16_uniform(base + k0, lane_offset, lds_unit_addr);
        } else if (k0 + chunk * 16 < rowbytes) {
            dma16_uniform(base + k0, lane_offset, lds_unit_addr);
        } else {
            *reinterpret_cast<u32x4*>(lds_unit + lane * 16) = u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto copy_a = [&](int i, int k0, int slot) {
        const int chunk = lane_chunk_base ^ ((i * 4 + (lane >> 4)) & 7);
        copy_unit(a_tile, a_src[i], lds_a_units + slot * A_SLOT + i * 1024,
                  lds + slot * A_SLOT + (wave * A_PER_WAVE + i) * 1024, chunk, k0);
    };
    auto copy_b = [&](int i, int k0, int slot) {
        const int chunk = lane_chunk_base ^ ((i * 4 + (lane >> 4)) & 7);
        copy_unit(b_tile, b_src[i], lds_b_units + slot * B_SLOT + i * 1024,
                  lds + B_BASE + slot * B_SLOT + (wave * B_PER_WAVE + i) * 1024, chunk, k0);
    };

    // ---- quantize-on-load.  The fused units of this wavefront (first A's, then B's) are filled through registers:
    // 32 bytes of bfloat16 per lane and unit are loaded, multiplied by 1/delta of the lane's row, encoded (RTNE; the
    // same arithmetic as qmm_quantize, so the codes are identical) and written to the place in LDS where the DMA
    // would have put the codes.  Units are handled in batches, one batch per MFMA block: the loads of a batch are
    // issued one block before its codes are needed, so their latency sits behind matrix work.
    constexpr int UNITS_F = (FUSE_A ? A_PER_WAVE : 0) + (FUSE_B ? B_PER_WAVE : 0);
    constexpr int BATCH = UNITS_F == 0 ? 1 : (UNITS_F + BLOCKS_M - 1) / BLOCKS_M;     // units per batch
    constexpr int NBATCH = UNITS_F == 0 ? 0 : (UNITS_F + BATCH - 1) / BATCH;          // <= BLOCKS_M
    float f_rho[UNITS_F > 0 ? UNITS_F : 1];
    u32x4 f_raw[BATCH][2];
    if constexpr (UNITS_F > 0) {
#pragma unroll
        for (int f = 0; f < UNITS_F; ++f) {
            const bool is_a = FUSE_A && f < A_PER_WAVE;
            const int i = is_a ? f : f - (FUSE_A ? A_PER_WAVE : 0);
            const int p = (wave * (is_a ? A_PER_WAVE : B_PER_WAVE) + i) * 8 + (lane >> 3);
            float d;
            if (is_a) {
                int64_t row = m0 + p; row = row < g.M ? row : g.M - 1;
                d = g.da[((bidx / g.da_inner) % g.da_groups) * (g.da_per_channel ? g.M : 1) + (g.da_per_channel ? row : 0)];
            } else {
                int64_t row = n0 + WN * (p / WN) + TILES_N * (p % R) + (p / R) % TILES_N; row = row < g.N ? row : g.N - 1;
                d = g.db[((bidx / g.db_inner) % g.db_groups) * (g.db_per_channel ? g.N : 1) + (g.db_per_channel ? row : 0)];
            }
            f_rho[f] = 1.0f / d;
        }
    }
    auto fused_load = [&](int batch, int64_t k0) {
        if constexpr (UNITS_F > 0) {
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int f = batch * BATCH + u;
                if (f < UNITS_F) {
                    const bool is_a = FUSE_A && f < A_PER_WAVE;
                    const int i = is_a ? f : f - (FUSE_A ? A_PER_WAVE : 0);
                    const int p = (wave * (is_a ? A_PER_WAVE : B_PER_WAVE) + i) * 8 + (lane >> 3);
                    const int c = lane_chunk_base ^ ((p >> 1) & 7);
                    const uint8_t* src = (is_a ? a_tile + a_src[i] : b_tile + b_src[i]) + k0 * 2;
                    if (k0 + c * 16 < rowbytes) {
                        f_raw[u][0] = reinterpret_cast<const u32x4*>(src)[0];
                        f_raw[u][1] = reinterpret_cast<const u32x4*>(src)[1];
                    } else {
                        f_raw[u][0] = u32x4{0u, 0u, 0u, 0u};
                        f_raw[u][1] = u32x4{0u, 0u, 0u, 0u};
                    }
                }
            }
        }
    };
    auto fused_store = [&](int batch, int a_slot_w, int b_slot_w) {
        if constexpr (UNITS_F > 0) {
            uint8_t* sa = lds + a_slot_w * A_SLOT;
            uint8_t* sb = lds + B_BASE + b_slot_w * B_SLOT;
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int f = batch * BATCH + u;
                if (f < UNITS_F) {
                    const bool is_a = FUSE_A && f < A_PER_WAVE;
                    const int i = is_a ? f : f - (FUSE_A ? A_PER_WAVE : 0);
                    uint8_t* dst = (is_a ? sa + (wave * A_PER_WAVE + i) * 1024 : sb + (wave * B_PER_WAVE + i) * 1024) + lane * 16;
                    u32x4 codes;
                    if (is_a) codes = encode16_bf16_rtne<FA>(f_raw[u][0], f_raw[u][1], f_rho[f]);
                    else codes = encode16_bf16_rtne<FB>(f_raw[u][0], f_raw[u][1], f_rho[f]);
                    *reinterpret_cast<u32x4*>(dst) = codes;
                }
            }
        }
    };

    // ---- accumulators: acc[A block][B block]
    using AccT = typename std::conditional<F8, v4f, typename std::conditional<KIND == KIND_I8, v16i, v16f>::type>::type;
    using Frag = typename std::conditional<F8, v8i, v4i>::type;
    AccT acc[BLOCKS_M][TILES_N];
#pragma unroll
    for (int i = 0; i < BLOCKS_M; ++i)
#pragma unroll
        for (int j = 0; j < TILES_N; ++j)
#pragma unroll
            for (int e = 0; e < (F8 ? 4 : 16); ++e) acc[i][j][e] = 0;
    pin_accumulators(acc);

    // FP8: lane (r = l%16, g = l/16) reads chunks g and g+4 of row r of a 16-row block.
    // INT8/BF16: lane (r = l%32, h = l/32) reads chunk 2s+h of row r of a 32-row block for K slice s = 0..3.
    const int frow = lane & (R - 1);
    const int fkey = (frow >> 1) & 7;
    const int fsel = F8 ? (lane >> 4) : (lane >> 5);
    const int a_off = (wm * WM + frow) * kSlabBytes;
    const int b_off = B_BASE + (wn * WN + frow) * kSlabBytes;
    int coff[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) coff[s] = ((F8 ? fsel : 2 * s + fsel) ^ fkey) * 16;

    auto read_frag = [&](const uint8_t* row_ptr, int s) -> Frag {
        if constexpr (F8) {
            const v4i p0 = *reinterpret_cast<const v4i*>(row_ptr + coff[0]);
            const v4i p1 = *reinterpret_cast<const v4i*>(row_ptr + (coff[0] ^ 64));
            return v8i{p0[0], p0[1], p0[2], p0[3], p1[0], p1[1], p1[2], p1[3]};
        } else {
            return *reinterpret_cast<const v4i*>(row_ptr + coff[s]);
        }
    };
    // The matrix instructions are written out with the accumulator tied ("+a": same AGPRs in and out).  Left to the
    // compiler, some instantiations of this loop got the three-address form, which copies every accumulator
    // block through a temporary in front of its MFMA (four moves and a pipeline wait per instruction).
    // What the compiler no longer sees and this kernel guarantees itself: an accumulator block is next touched a
    // whole K step later (no back-to-back dependent MFMAs), and accumulators are first read (epilogue) behind the
    // wait states placed after the loop.
    auto mma = [&](const Frag& fa, const Frag& fb, AccT& c) {
        // first operand: A rows -> the 4-row groups held in a lane's registers; second: B rows -> lane%R
        // (device pass only: the host pass would check these register constraints against the host's)
#if defined(__HIP_DEVICE_COMPILE__)
        if constexpr (F8) {
            if constexpr (FA == QMM_FMT_E5M2 && FB == QMM_FMT_E5M2)
                asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:1 blgp:1" : "+a"(c) : "v"(fa), "v"(fb));
            else if constexpr (FA == QMM_FMT_E5M2)
                asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:1" : "+a"(c) : "v"(fa), "v"(fb));
            else if constexpr (FB == QMM_FMT_E5M2)
                asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 blgp:1" : "+a"(c) : "v"(fa), "v"(fb));
            else
                asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(c) : "v"(fa), "v"(fb));
        } else if constexpr (KIND == KIND_I8) {
            asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+a"(c) : "v"(fa), "v"(fb));
        } else {
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(fa), "v"(fb));
        }
#endif
    };

    Frag fb[KS][TILES_N];      // B fragments of the current slab
    Frag fa[2][KS];            // A fragments of one block, ping-pong between blocks

    auto read_a = [&](int slot, int i, int buf) {
        const uint8_t* sa = lds + slot * A_SLOT + a_off + i * R * kSlabBytes;
#pragma unroll
        for (int s = 0; s < KS; ++s) fa[buf][s] = read_frag(sa, s);
    };

    // ---- pipeline.  K slab s of A lives in A slot s % 3, of B in B slot s % 2; the B fragments of the current slab
    // live in registers for the whole step, which serves as a third B stage.  Once per K step, before the last A
    // block, the wavefronts meet (E_s): every LDS read of slab s has completed, and slabs s+1 have landed.  After
    // E_s, A slot s%3 and B slot s%2 are free.  Copies are requested one or two at a time between matrix
    // instructions (a burst of sixteen parks the wavefront at the memory pipeline for about 1000 cycles, with no
    // matrix work issued meanwhile), in this order:
    //     last block of step s   : the first half of B slab s+2
    //     blocks 0.. of step s+1 : the second half of B slab s+2, then A slab s+3
    // B slab s+2 has until E_(s+1) to arrive, A slab s+3 until E_(s+2).  Loads complete in order, so at E_s "at
    // most the A copies of this step outstanding" (vmcnt) means slabs s+1 are in LDS.
    // With quantize-on-load, a fused operand's slab s+1 is encoded into its slot during step s instead.
    constexpr int NA = FUSE_A ? 0 : A_PER_WAVE, NB = FUSE_B ? 0 : B_PER_WAVE;
    constexpr int NB_TAIL = NB / 2;                                 // B copies requested in a step's last block
    constexpr int MMAS_PER_BLOCK = KS * TILES_N;
    constexpr int N1 = (BLOCKS_M - 1) * MMAS_PER_BLOCK;             // MFMAs before E
    constexpr int NC = (NB - NB_TAIL) + NA;                         // copies requested among them
    static_assert(NC <= N1 && NB_TAIL <= MMAS_PER_BLOCK, "one copy per MFMA at most");

    const int nk = (rowbytes + kSlabBytes - 1) / kSlabBytes;
    // prologue: slab 0 of both operands, A slab 1, the first half of B slab 1 (what the steps before would have
    // requested); A slab 2 and the rest of B slab 1 follow inside step 0
    if constexpr (!FUSE_A) {
#pragma unroll
        for (int i = 0; i < A_PER_WAVE; ++i) copy_a(i, 0, 0);
    }
    if constexpr (!FUSE_B) {
#pragma unroll
        for (int i = 0; i < B_PER_WAVE; ++i) copy_b(i, 0, 0);
    }
    if constexpr (UNITS_F > 0) {
#pragma unroll
        for (int bt = 0; bt < NBATCH; ++bt) { fused_load(bt, 0); fused_store(bt, 0, 0); }
    }
    if (nk > 1) {
        if constexpr (!FUSE_A) {
#pragma unroll
            for (int i = 0; i < A_PER_WAVE; ++i) copy_a(i, kSlabBytes, 1);
        }
#pragma unroll
        for (int i = 0; i < NB_TAIL; ++i) copy_b(i, kSlabBytes, 1);
        wait_vm<NA + NB_TAIL>();
    } else {
        wait_vm<0>();
    }
    __syncthreads();
    if (nk > 1) fused_load(0, kSlabBytes);
    {
        const uint8_t* sb = lds + b_off;
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int j = 0; j < TILES_N; ++j) fb[s][j] = read_frag(sb + j * R * kSlabBytes, s);
    }
    read_a(0, 0, 0);

    asm volatile("s_nop 7" ::: "memory");     // accumulator initialisation -> first matrix instruction
    __builtin_amdgcn_sched_barrier(0);
    int a_slot = 0;                            // kt % 3
    // One K step.  STEADY: slabs kt+1 and kt+2 exist and are whole, so every copy is issued without a test; the
    // code between the matrix instructions is then free of branches (a taken branch stalls the wavefront's issue
    // for longer than a copy does).
    auto step = [&](int kt, auto steady_tag) {
        constexpr bool STEADY = decltype(steady_tag)::value;
        const int b_slot = kt & 1;
        const int a_next = a_slot == 2 ? 0 : a_slot + 1;          // slot of A slab kt+1
        const int a_free = a_slot == 0 ? 2 : a_slot - 1;          // slot of A slab kt+2 (slab kt-1 left it at E_(kt-1))
        const bool more = STEADY || kt + 1 < nk, more2 = STEADY || kt + 2 < nk;
        const int k1 = (kt + 1) * kSlabBytes, k2 = (kt + 2) * kSlabBytes;
        // copy number c of the blocks before E: the rest of B slab kt+1, then A slab kt+2
        auto copy_before_e = [&](int c) {
            if (c < NB - NB_TAIL) {
                if constexpr (STEADY) dma16_uniform(b_tile + k1, b_src[NB_TAIL + c], lds_b_units + (b_slot ^ 1) * B_SLOT + (NB_TAIL + c) * 1024);
                else if (more) copy_b(NB_TAIL + c, k1, b_slot ^ 1);
            } else {
                const int i = c - (NB - NB_TAIL);
                if constexpr (STEADY) dma16_uniform(a_tile + k2, a_src[i], lds_a_units + a_free * A_SLOT + i * 1024);
                else if (more2) copy_a(i, k2, a_free);
            }
        };
#pragma unroll
        for (int i = 0; i < BLOCKS_M - 1; ++i) {
            if constexpr (UNITS_F > 0) {
                // quantize-on-load: codes of batch i of the next slab go to LDS, batch i+1 is requested
                if (more) {
                    if (i < NBATCH) fused_store(i, a_next, b_slot ^ 1);
                    if (i + 1 < NBATCH) fused_load(i + 1, k1);
                }
            }
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int j = 0; j < TILES_N; ++j) {
                    const int q = s * TILES_N + j;                 // MFMA number within the block
                    const int m = i * MMAS_PER_BLOCK + q;          // MFMA number within the step
                    mma(fa[i & 1][s], fb[s][j], acc[i][j]);
                    if (q == 0) {
                        // the request for the next block's fragments follows the block's first MFMA, so that the
                        // wait in front of that MFMA never covers the newest request
                        __builtin_amdgcn_sched_barrier(0);
                        read_a(a_slot, i + 1, (i + 1) & 1);
                        __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                    for (int c = 0; c < NC; ++c)
                        if ((c * N1) / (NC > 0 ? NC : 1) == m) {
                            __builtin_amdgcn_sched_barrier(0);
                            copy_before_e(c);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (more) {
            if constexpr (UNITS_F > 0) { if (NBATCH == BLOCKS_M) fused_store(BLOCKS_M - 1, a_next, b_slot ^ 1); }
            // E_kt
            if (more2) wait_vm_lgkm<NA>(); else wait_vm_lgkm<0>();
            __syncthreads();
            if (more2) fused_load(0, k2);
            read_a(a_next, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        const uint8_t* sb_next = lds + (b_slot ^ 1) * B_SLOT + b_off;
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int j = 0; j < TILES_N; ++j) {
                const int q = s * TILES_N + j;
                mma(fa[(BLOCKS_M - 1) & 1][s], fb[s][j], acc[BLOCKS_M - 1][j]);
                if (more) fb[s][j] = read_frag(sb_next + j * R * kSlabBytes, s);
#pragma unroll
                for (int c = 0; c < NB_TAIL; ++c)
                    if ((c * MMAS_PER_BLOCK) / (NB_TAIL > 0 ? NB_TAIL : 1) == q) {
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (STEADY) dma16_uniform(b_tile + k2, b_src[c], lds_b_units + b_slot * B_SLOT + c * 1024);
                        else if (more2) copy_b(c, k2, b_slot);
                        __builtin_amdgcn_sched_barrier(0);
                    }
            }
        __builtin_amdgcn_sched_barrier(0);
        a_slot = a_next;
    };
    const int nk_steady = rowbytes / kSlabBytes - 2;    // steps whose two following slabs are whole
    int kt = 0;
    for (; kt < nk_steady; ++kt) step(kt, std::true_type{});
    for (; kt < nk; ++kt) step(kt, std::false_type{});

    // wait states between the last matrix instruction and the first read of an accumulator (the longest MFMA
    // here takes 16 passes; 32 states cover every case)
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);

    // ---- epilogue.  MFMA result D[i][j]: i = A row within the block, j = lane % R = B row within the block.
    //  16x16: a lane's register r of acc[ia][t] is row 16*ia + 4*(l/16) + r, column TILES_N*(l%16) + t
    //  32x32: a lane's register v of acc[ia][t] is row 32*ia + 8*(v/4) + 4*(l/32) + v%4, column TILES_N*(l%32) + t
    //  so for a fixed register the TILES_N accumulators of a lane are consecutive columns, and the lanes of a
    //  store instruction cover whole rows of the wavefront tile.
    const int64_t m_base = m0 + wm * WM, n_base = n0 + wn * WN;
    const float* da = g.da ? g.da + ((bidx / g.da_inner) % g.da_groups) * (g.da_per_channel ? g.M : 1) : nullptr;
    const float* db = g.db ? g.db + ((bidx / g.db_inner) % g.db_groups) * (g.db_per_channel ? g.N : 1) : nullptr;
    constexpr bool descale = (KIND != KIND_BF16);
    constexpr int REGS = F8 ? 4 : 16;
    const int64_t n = n_base + TILES_N * (lane & (R - 1));     // first of this lane's TILES_N columns
    const int lane_row = F8 ? 4 * (lane >> 4) : 4 * (lane >> 5);
    float sr[TILES_N];
#pragma unroll
    for (int tt = 0; tt < TILES_N; ++tt) {
        sr[tt] = 1.0f;
        if constexpr (descale) sr[tt] = g.db_per_channel ? db[(n + tt) < g.N ? (n + tt) : (g.N - 1)] : db[0];
    }
    float sa_scalar = 1.0f;
    if constexpr (descale) { if (!g.da_per_channel) sa_scalar = da[0]; }

    // value tt of register r of A block ia, descaled: (acc * deltaA[row]) * deltaB[column], in that order
    auto value = [&](int ia, int r, int tt, float sl, uint32_t& raw) -> float {
        float a;
        // accumulators live in AGPRs: each one is copied out where it is used (the register allocator must not
        // try to hold all of them in VGPRs at once)
        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(raw) : "a"(acc[ia][tt][r]));
        if constexpr (KIND == KIND_I8) a = (float)(int32_t)raw;
        else a = __uint_as_float(raw);
        if constexpr (descale) a = (a * sl) * sr[tt];
        return a;
    };
    auto row_in_block = [&](int r) -> int { return F8 ? lane_row + r : 8 * (r >> 2) + lane_row + (r & 3); };

    double nsr_ee = 0.0, nsr_rr = 0.0;
    auto nsr_add = [&](float stored, float ref) {
        const double e = (double)stored - (double)ref;
        if (e == e) { nsr_ee = fma(e, e, nsr_ee); nsr_rr = fma((double)ref, (double)ref, nsr_rr); }
    };
    // TILES_N consecutive reference values of output row (matrix bidx, row m), from column n on (whole tiles only)
    auto nsr_row = [&](int64_t m, float (&rv)[TILES_N]) {
        const float* p = g.nsr_ref + (bidx * g.M + m) * g.N + n;
        if constexpr (TILES_N == 4) { const v4f q = *reinterpret_cast<const v4f*>(p); rv[0] = q[0]; rv[1] = q[1]; rv[2] = q[2]; rv[3] = q[3]; }
        else if constexpr (TILES_N == 2) { typedef float f2v __attribute__((ext_vector_type(2))); const f2v q = *reinterpret_cast<const f2v*>(p); rv[0] = q[0]; rv[1] = q[1]; }
        else {
#pragma unroll
            for (int tt = 0; tt < TILES_N; ++tt) rv[tt] = p[tt];
        }
    };
    const bool interior = (m0 + BM <= g.M) && (n0 + BN <= g.N) && (g.N % TILES_N == 0);
    if (g.splits > 1) {
        // split-K: the raw accumulators of this K range go to the partial-sum buffer; a second kernel adds the
        // ranges in ascending order, descales and writes the outputs
        uint32_t* pbase = static_cast<uint32_t*>(g.partial) + ((int64_t)split * g.batch + bidx) * g.M * g.N;
#pragma unroll
        for (int ia = 0; ia < BLOCKS_M; ++ia) {
#pragma unroll
            for (int r = 0; r < REGS; ++r) {
                const int64_t m = m_base + ia * R + row_in_block(r);
                uint32_t raw[TILES_N];
#pragma unroll
                for (int tt = 0; tt < TILES_N; ++tt) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(raw[tt]) : "a"(acc[ia][tt][r]));
                uint32_t* dst = pbase + m * g.N + n;
                if (interior) {
                    if constexpr (TILES_N == 4) *reinterpret_cast<u32x4*>(dst) = u32x4{raw[0], raw[1], raw[2], raw[3]};
                    else if constexpr (TILES_N == 2) *reinterpret_cast<u32x2*>(dst) = u32x2{raw[0], raw[1]};
                    else {
#pragma unroll
                        for (int tt = 0; tt < TILES_N; ++tt) dst[tt] = raw[tt];
                    }
                } else if (m < g.M) {
#pragma unroll
                    for (int tt = 0; tt < TILES_N; ++tt)
                        if (n + tt < g.N) dst[tt] = raw[tt];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    } else if (interior && g.y && g.y_bf16 && !g.acc_out) {
        // fast path: whole tile inside the matrix, bfloat16 output only; 2*TILES_N bytes per lane and store
        uint8_t* ybase = static_cast<uint8_t*>(g.y) + ((bidx * g.M + m_base) * g.N + n) * 2;
        const int64_t row_bytes = g.N * 2;
        // Row step sizes are all fetched before the first store: loads and stores share one in-order counter, so
        // a load issued between the stores could only be waited for together with every store before it.
        float sl_rows[BLOCKS_M][REGS];
#pragma unroll
        for (int ia = 0; ia < BLOCKS_M; ++ia)
#pragma unroll
            for (int r = 0; r < REGS; ++r) sl_rows[ia][r] = sa_scalar;
        if constexpr (descale) {
            if (g.da_per_channel) {
#pragma unroll
                for (int ia = 0; ia < BLOCKS_M; ++ia)
#pragma unroll
                    for (int r = 0; r < REGS; ++r) sl_rows[ia][r] = da[m_base + ia * R + row_in_block(r)];
            }
        }
        typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
        typedef float f2 __attribute__((ext_vector_type(2)));
        auto packed_row = [&](int ia, int r, uint32_t (&pk)[TILES_N / 2]) {
#pragma unroll
            for (int q = 0; q < TILES_N / 2; ++q) {
                uint32_t raw0, raw1;
                const float v0 = value(ia, r, 2 * q, sl_rows[ia][r], raw0), v1 = value(ia, r, 2 * q + 1, sl_rows[ia][r], raw1);
                pk[q] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{v0, v1}, bf2));
            }
        };
#pragma unroll
        for (int ia = 0; ia < BLOCKS_M; ++ia) {
#pragma unroll
            for (int r = 0; r < REGS; ++r) {
                const int ml = ia * R + row_in_block(r);
                uint32_t pk[TILES_N / 2];
                float rv[TILES_N];
                if constexpr (NSR != 0) nsr_row(m_base + ml, rv);
                packed_row(ia, r, pk);
                if constexpr (NSR != 0) {
#pragma unroll
                    for (int q = 0; q < TILES_N / 2; ++q) {
                        nsr_add(__uint_as_float(pk[q] << 16), rv[2 * q]);
                        nsr_add(__uint_as_float(pk[q] & 0xFFFF0000u), rv[2 * q + 1]);
                    }
                }
                uint8_t* dst = ybase + ml * row_bytes;
                if constexpr (TILES_N == 8) *reinterpret_cast<u32x4*>(dst) = u32x4{pk[0], pk[1], pk[2], pk[3]};
                else if constexpr (TILES_N == 4) __builtin_nontemporal_store(u32x2{pk[0], pk[1]}, reinterpret_cast<u32x2*>(dst));
                else *reinterpret_cast<uint32_t*>(dst) = pk[0];
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    } else if (interior && g.y && !g.y_bf16 && !g.acc_out && TILES_N % 4 == 0) {
        // whole tile inside the matrix, binary32 output only: 16 bytes per store
        float* ybase = static_cast<float*>(g.y) + (bidx * g.M + m_base) * g.N + n;
        float sl_rows[BLOCKS_M][REGS];
#pragma unroll
        for (int ia = 0; ia < BLOCKS_M; ++ia)
#pragma unroll
            for (int r = 0; r < REGS; ++r) sl_rows[ia][r] = sa_scalar;
        if constexpr (descale) {
            if (g.da_per_channel) {
#pragma unroll
                for (int ia = 0; ia < BLOCKS_M; ++ia)
#pragma unroll
                    for (int r = 0; r < REGS; ++r) sl_rows[ia][r] = da[m_base + ia * R + row_in_block(r)];
            }
        }
#pragma unroll
        for (int ia = 0; ia < BLOCKS_M; ++ia) {
#pragma unroll
            for (int r = 0; r < REGS; ++r) {
                const int ml = ia * R + row_in_block(r);
                float* dst = ybase + (int64_t)ml * g.N;
                float rv[TILES_N];
                if constexpr (NSR != 0) nsr_row(m_base + ml, rv);
#pragma unroll
                for (int q = 0; q < TILES_N / 4; ++q) {
                    uint32_t raw;
                    v4f v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = value(ia, r, 4 * q + e, sl_rows[ia][r], raw);
                    if constexpr (NSR != 0) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) nsr_add(v[e], rv[4 * q + e]);
                    }
                    *reinterpret_cast<v4f*>(dst + 4 * q) = v;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    } else if (n < g.N) {
        // general path: edge tiles, raw accumulators, narrow lanes; element-wise with bounds checks
#pragma unroll
        for (int ia = 0; ia < BLOCKS_M; ++ia) {
#pragma unroll
            for (int r = 0; r < REGS; ++r) {
                const int64_t m = m_base + ia * R + row_in_block(r);
                if (m < g.M) {
                    float sl = sa_scalar;
                    if constexpr (descale) { if (g.da_per_channel) sl = da[m]; }
                    const int64_t o = (bidx * g.M + m) * g.N + n;
#pragma unroll
                    for (int tt = 0; tt < TILES_N; ++tt) {
                        uint32_t raw;
                        const float v = value(ia, r, tt, sl, raw);
                        if (n + tt < g.N) {
                            if (g.acc_out) static_cast<uint32_t*>(g.acc_out)[o + tt] = raw;
                            if (g.y) {
                                if (g.y_bf16) static_cast<__bf16*>(g.y)[o + tt] = (__bf16)v;
                                else static_cast<float*>(g.y)[o + tt] = v;
                            }
                            if constexpr (NSR != 0) nsr_add(g.y_bf16 ? (float)(__bf16)v : v, g.nsr_ref[o + tt]);
                        }
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if constexpr (NSR != 0) {
        // one pair of sums per wavefront; a second kernel folds them in a fixed order
        const double see = wave_sum_f64(nsr_ee), srr = wave_sum_f64(nsr_rr);
        if (lane == 0) {
            double* o = g.nsr_partial + ((int64_t)blockIdx.x * NWAVES + wave) * 2;
            o[0] = see; o[1] = srr;
        }
    }
}

// Fold of the NSR variant's per-wavefront sums: thread t takes pairs t, t + 256, ... in ascending order, then the
// fixed shuffle tree and the four wavefronts in order: the order of additions depends on the count only.
__global__ void __launch_bounds__(256)
nsr_finalize(const double* __restrict__ partial, int64_t count, double* __restrict__ out2)
{
    __shared__ double s[4][2];
    double ee = 0.0, rr = 0.0;
    for (int64_t i = threadIdx.x; i < count; i += 256) { ee += partial[2 * i]; rr += partial[2 * i + 1]; }
    ee = wave_sum_f64(ee); rr = wave_sum_f64(rr);
    if ((threadIdx.x & 63) == 0) { s[threadIdx.x >> 6][0] = ee; s[threadIdx.x >> 6][1] = rr; }
    __syncthreads();
    if (threadIdx.x == 0) {
        out2[0] = ((s[0][0] + s[1][0]) + s[2][0]) + s[3][0];
        out2[1] = ((s[0][1] + s[1][1]) + s[2][1]) + s[3][1];
    }
}

// Contraction of one slab at most (attention scores: K = head dimension) with a large output.  A tile of
// gemm_kernel would be: copies, wait a memory latency, 32 matrix instructions per wavefront, 128 KB of stores -- and
// with one workgroup per CU nothing overlaps, so the latency and the stores are paid in full for every tile.  Here
// the workgroup stays on its CU and walks tiles; LDS holds two slabs of each operand, and the copies of the next
// tile are requested right after the barrier that starts the current one, so they land behind its matrix
// instructions and stores.  Same tile (256 x 256, eight wavefronts), LDS layout, fragment reads and accumulator
// layout as gemm_kernel; whole tiles only (the host sends ragged shapes to gemm_kernel).
// Order of a wavefront's vector-memory operations: copies(t+1), stores(t), copies(t+2), ...; they complete in order,
// so "at most the stores of tile t outstanding" at the top of tile t+1 means its copies have landed.
template <int KIND, int FA, int FB>
__global__ void __launch_bounds__(512, 1)
gemm_shortk_kernel(GemmArgs g)
{
    constexpr bool F8 = (KIND == KIND_F8);
    constexpr int NWN = 4, NWAVES = 8;
    constexpr int BM = 256, BN = 256, WM = 128, WN = 64;
    constexpr int R = F8 ? 16 : 32;
    constexpr int BLOCKS_M = WM / R, TILES_N = WN / R;
    constexpr int KS = F8 ? 1 : 4;
    constexpr int REGS = F8 ? 4 : 16;
    constexpr int A_SLOT = BM * kSlabBytes, B_SLOT = BN * kSlabBytes;
    constexpr int B_BASE = 2 * A_SLOT;
    constexpr int A_PER_WAVE = BM / 8 / NWAVES, B_PER_WAVE = BN / 8 / NWAVES;
    constexpr int STORES = BLOCKS_M * REGS;          // store instructions of one tile's epilogue, one per row and lane
    using AccT = typename std::conditional<F8, v4f, typename std::conditional<KIND == KIND_I8, v16i, v16f>::type>::type;
    using Frag = typename std::conditional<F8, v8i, v4i>::type;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / NWN, wn = wave % NWN;
    const int rowbytes = (int)g.rowbytes;                       // <= kSlabBytes
    const uint32_t tiles_per_batch = (uint32_t)g.tiles_m * (uint32_t)g.tiles_n;
    const uint32_t total = tiles_per_batch * (uint32_t)g.batch;

    // ---- copy sources (32-bit byte offsets from a tile's first A / B row) and LDS targets, as in gemm_kernel
    uint32_t a_src[A_PER_WAVE], b_src[B_PER_WAVE];
    bool a_live[A_PER_WAVE], b_live[B_PER_WAVE];                // false: this lane's chunk lies past the end of the row
#pragma unroll
    for (int i = 0; i < A_PER_WAVE; ++i) {
        const int p = (wave * A_PER_WAVE + i) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((p >> 1) & 7);
        a_src[i] = (uint32_t)(p * rowbytes + c * 16);
        a_live[i] = c * 16 < rowbytes;
    }
#pragma unroll
    for (int i = 0; i < B_PER_WAVE; ++i) {
        const int p = (wave * B_PER_WAVE + i) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((p >> 1) & 7);
        const int row = WN * (p / WN) + TILES_N * (p % R) + (p / R) % TILES_N;
        b_src[i] = (uint32_t)(row * rowbytes + c * 16);
        b_live[i] = c * 16 < rowbytes;
    }
    typedef __attribute__((address_space(3))) uint8_t* lds_ptr_t;
    const uint32_t lds_a_units = (uint32_t)(uintptr_t)(lds_ptr_t)(lds + wave * A_PER_WAVE * 1024);
    const uint32_t lds_b_units = (uint32_t)(uintptr_t)(lds_ptr_t)(lds + B_BASE + wave * B_PER_WAVE * 1024);
    // Places in LDS whose chunk lies past the end of the rows never receive a copy: zeroed once, in both slots.
#pragma unroll
    for (int slot = 0; slot < 2; ++slot) {
#pragma unroll
        for (int i = 0; i < A_PER_WAVE; ++i)
            if (!a_live[i]) *reinterpret_cast<u32x4*>(lds + slot * A_SLOT + (wave * A_PER_WAVE + i) * 1024 + lane * 16) = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < B_PER_WAVE; ++i)
            if (!b_live[i]) *reinterpret_cast<u32x4*>(lds + B_BASE + slot * B_SLOT + (wave * B_PER_WAVE + i) * 1024 + lane * 16) = u32x4{0u, 0u, 0u, 0u};
    }

    // tile number -> first A row, first B row (scalar), output coordinates
    struct Tile { const uint8_t* a; const uint8_t* b; int64_t bidx, m0, n0; };
    auto tile_of = [&](uint32_t t) -> Tile {
        const int64_t bidx = __builtin_amdgcn_readfirstlane((int)(t / tiles_per_batch));
        const uint32_t r = t - (uint32_t)bidx * tiles_per_batch;
        const int64_t tm = __builtin_amdgcn_readfirstlane((int)(r / (uint32_t)g.tiles_n));
        const int64_t tn = __builtin_amdgcn_readfirstlane((int)(r % (uint32_t)g.tiles_n));
        Tile o;
        o.bidx = bidx; o.m0 = tm * BM; o.n0 = tn * BN;
        o.a = g.a + (bidx * g.M + o.m0) * g.rowbytes;
        o.b = g.b + (bidx * g.N + o.n0) * g.rowbytes;
        return o;
    };
    auto issue_copies = [&](const Tile& t, int slot) {
#pragma unroll
        for (int i = 0; i < A_PER_WAVE; ++i)
            if (a_live[i]) dma16_uniform(t.a, a_src[i], lds_a_units + slot * A_SLOT + i * 1024);
#pragma unroll
        for (int i = 0; i < B_PER_WAVE; ++i)
            if (b_live[i]) dma16_uniform(t.b, b_src[i], lds_b_units + slot * B_SLOT + i * 1024);
    };

    // ---- fragments (as in gemm_kernel)
    const int frow = lane & (R - 1);
    const int fkey = (frow >> 1) & 7;
    const int fsel = F8 ? (lane >> 4) : (lane >> 5);
    const int a_off = (wm * WM + frow) * kSlabBytes;
    const int b_off = B_BASE + (wn * WN + frow) * kSlabBytes;
    int coff[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) coff[s] = ((F8 ? fsel : 2 * s + fsel) ^ fkey) * 16;
    auto read_frag = [&](const uint8_t* row_ptr, int s) -> Frag {
        if constexpr (F8) {
            const v4i p0 = *reinterpret_cast<const v4i*>(row_ptr + coff[0]);
            const v4i p1 = *reinterpret_cast<const v4i*>(row_ptr + (coff[0] ^ 64));
            return v8i{p0[0], p0[1], p0[2], p0[3], p1[0], p1[1], p1[2], p1[3]};
        } else {
            return *reinterpret_cast<const v4i*>(row_ptr + coff[s]);
        }
    };
    auto mma = [&](const Frag& fa, const Frag& fb, AccT& c) {
#if defined(__HIP_DEVICE_COMPILE__)
        if constexpr (F8) {
            if constexpr (FA == QMM_FMT_E5M2 && FB == QMM_FMT_E5M2)
                asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:1 blgp:1" : "+a"(c) : "v"(fa), "v"(fb));
            else if constexpr (FA == QMM_FMT_E5M2)
                asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:1" : "+a"(c) : "v"(fa), "v"(fb));
            else if constexpr (FB == QMM_FMT_E5M2)
                asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 blgp:1" : "+a"(c) : "v"(fa), "v"(fb));
            else
                asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(c) : "v"(fa), "v"(fb));
        } else if constexpr (KIND == KIND_I8) {
            asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+a"(c) : "v"(fa), "v"(fb));
        } else {
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(fa), "v"(fb));
        }
#endif
    };

    AccT acc[BLOCKS_M][TILES_N];
    constexpr bool descale = (KIND != KIND_BF16);

    const uint32_t stride = gridDim.x;
    uint32_t t_cur = blockIdx.x;
    if (t_cur >= total) return;
    Tile cur = tile_of(t_cur);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");           // the zeroing above
    issue_copies(cur, 0);
    for (int it = 0;; ++it) {
        const int slot = it & 1;
#pragma unroll
        for (int i = 0; i < BLOCKS_M; ++i)
#pragma unroll
            for (int j = 0; j < TILES_N; ++j)
#pragma unroll
                for (int e = 0; e < REGS; ++e) acc[i][j][e] = 0;
        pin_accumulators(acc);
        // this tile's copies have landed (the stores of the tile before, issued after them, may still be under way)
        // (the count must not exceed the number of operations issued after those copies -- "at most n outstanding"
        // says nothing about the n newest -- so it is the exact number of stores of the path taken, or less)
        if (it == 0) wait_vm_lgkm<0>(); else wait_vm_lgkm<(STORES > 63 ? 63 : STORES)>();
        __syncthreads();
        // every wavefront has left the tile before: its slot is free for the tile after this one
        const uint32_t t_next = t_cur + stride;
        const bool has_next = t_next < total;
        Tile nxt = cur;
        if (has_next) {
            nxt = tile_of(t_next);
            issue_copies(nxt, slot ^ 1);
        }
        Frag fb[KS][TILES_N], fa[2][KS];
        {
            const uint8_t* sb = lds + slot * B_SLOT + b_off;
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int j = 0; j < TILES_N; ++j) fb[s][j] = read_frag(sb + j * R * kSlabBytes, s);
        }
        const uint8_t* sa = lds + slot * A_SLOT + a_off;
#pragma unroll
        for (int s = 0; s < KS; ++s) fa[0][s] = read_frag(sa, s);
        asm volatile("s_nop 7" ::: "memory");     // accumulator initialisation -> first matrix instruction
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < BLOCKS_M; ++i) {
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int j = 0; j < TILES_N; ++j) {
                    mma(fa[i & 1][s], fb[s][j], acc[i][j]);
                    if (s == 0 && j == 0 && i + 1 < BLOCKS_M) {
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int s2 = 0; s2 < KS; ++s2) fa[(i + 1) & 1][s2] = read_frag(sa + (i + 1) * R * kSlabBytes, s2);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            __builtin_amdgcn_sched_barrier(0);
        }
        // wait states between the last matrix instruction and the first read of an accumulator
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);

        // ---- epilogue of a whole tile: (acc * deltaA[row]) * deltaB[column], in that order
        {
            const int64_t bidx = cur.bidx;
            const int64_t m_base = cur.m0 + wm * WM, n_base = cur.n0 + wn * WN;
            const float* da = g.da ? g.da + ((bidx / g.da_inner) % g.da_groups) * (g.da_per_channel ? g.M : 1) : nullptr;
            const float* db = g.db ? g.db + ((bidx / g.db_inner) % g.db_groups) * (g.db_per_channel ? g.N : 1) : nullptr;
            int lane_e = lane;                    // kept out of the loop-invariant code the compiler would hoist
            asm volatile("" : "+v"(lane_e));
            const int64_t n = n_base + TILES_N * (lane_e & (R - 1));
            const int lane_row = F8 ? 4 * (lane_e >> 4) : 4 * (lane_e >> 5);
            auto row_in_block = [&](int r) -> int { return F8 ? lane_row + r : 8 * (r >> 2) + lane_row + (r & 3); };
            float sr[TILES_N];
#pragma unroll
            for (int tt = 0; tt < TILES_N; ++tt) {
                sr[tt] = 1.0f;
                if constexpr (descale) sr[tt] = g.db_per_channel ? db[n + tt] : db[0];
            }
            float sa_scalar = 1.0f;
            if constexpr (descale) { if (!g.da_per_channel) sa_scalar = da[0]; }
            float sl_rows[BLOCKS_M][REGS];
#pragma unroll
            for (int ia = 0; ia < BLOCKS_M; ++ia)
#pragma unroll
                for (int r = 0; r < REGS; ++r) {
                    sl_rows[ia][r] = sa_scalar;
                    if constexpr (descale) { if (g.da_per_channel) sl_rows[ia][r] = da[m_base + ia * R + row_in_block(r)]; }
                }
            auto value = [&](int ia, int r, int tt) -> float {
                uint32_t raw;
                asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(raw) : "a"(acc[ia][tt][r]));
                float a;
                if constexpr (KIND == KIND_I8) a = (float)(int32_t)raw;
                else a = __uint_as_float(raw);
                if constexpr (descale) a = (a * sl_rows[ia][r]) * sr[tt];
                return a;
            };
            if (g.y_bf16) {
                uint8_t* ybase = static_cast<uint8_t*>(g.y) + ((bidx * g.M + m_base) * g.N + n) * 2;
                const int64_t row_bytes = g.N * 2;
                typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
                typedef float f2 __attribute__((ext_vector_type(2)));
                auto packed_row = [&](int ia, int r, uint32_t (&pk)[TILES_N / 2]) {
#pragma unroll
                    for (int q = 0; q < TILES_N / 2; ++q) {
                        const float v0 = value(ia, r, 2 * q), v1 = value(ia, r, 2 * q + 1);
                        pk[q] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{v0, v1}, bf2));
                    }
                };
#pragma unroll
                for (int ia = 0; ia < BLOCKS_M; ++ia) {
#pragma unroll
                    for (int r = 0; r < REGS; ++r) {
                        uint32_t pk[TILES_N / 2];
                        packed_row(ia, r, pk);
                        uint8_t* dst = ybase + (ia * R + row_in_block(r)) * row_bytes;
                        if constexpr (TILES_N == 4) __builtin_nontemporal_store(u32x2{pk[0], pk[1]}, reinterpret_cast<u32x2*>(dst));
                        else __builtin_nontemporal_store(pk[0], reinterpret_cast<uint32_t*>(dst));
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else if constexpr (TILES_N == 4) {
                float* ybase = static_cast<float*>(g.y) + (bidx * g.M + m_base) * g.N + n;
#pragma unroll
                for (int ia = 0; ia < BLOCKS_M; ++ia) {
#pragma unroll
                    for (int r = 0; r < REGS; ++r) {
                        v4f v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = value(ia, r, e);
                        __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(ybase + (int64_t)(ia * R + row_in_block(r)) * g.N));
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        if (!has_next) break;
        cur = nxt; t_cur = t_next;
    }
}

// Several 256 x 256 tiles per CU and a contraction of three slabs or more (the linear layers of a transformer).
// With gemm_kernel every tile pays a fixed price that no matrix instruction covers: the first copies' latency, and
// above all its 128 KB of stores, which all CUs issue at the same moment (8-9 us per tile at K = 1024, where the
// matrix work itself takes 11 us).  Here the workgroup stays on its CU and the slabs of all its tiles form ONE
// stream through the same LDS ring (three slots of A, two of B) with the same step schedule as gemm_kernel: at a
// tile's last steps the slabs requested are simply the first ones of the next tile, so the next tile's first step
// starts right behind the epilogue, and the stores drain while it runs.
// Vector-memory operations complete in order, loads and stores alike, so "slab q+1 has landed" is "at most n newer
// operations outstanding".  At a tile boundary the copies that the next tile's first step would request before its
// barrier are requested in front of the stores instead; that step then requests none and waits with the exact number
// of stores allowed outstanding, and the stores are only waited for one step later (they have had 2-3 us by then).
// Codes in, whole tiles, whole slabs, no split, output in y alone; same fragment, accumulator and store layout as
// gemm_kernel.
template <int KIND, int FA, int FB>
__global__ void __launch_bounds__(512, 1)
gemm_stream_kernel(GemmArgs g)
{
    constexpr bool F8 = (KIND == KIND_F8);
    constexpr int NWN = 4, NWAVES = 8;
    constexpr int BM = 256, BN = 256, WM = 128, WN = 64;
    constexpr int R = F8 ? 16 : 32;
    constexpr int BLOCKS_M = WM / R, TILES_N = WN / R;
    constexpr int KS = F8 ? 1 : 4;
    constexpr int REGS = F8 ? 4 : 16;
    constexpr int A_SLOT = BM * kSlabBytes, B_SLOT = BN * kSlabBytes;
    constexpr int B_BASE = kASlots * A_SLOT;
    constexpr int NA = BM / 8 / NWAVES, NB = BN / 8 / NWAVES;      // copies per wavefront and slab
    constexpr int NB_TAIL = NB / 2;
    constexpr int MMAS_PER_BLOCK = KS * TILES_N;
    constexpr int N1 = (BLOCKS_M - 1) * MMAS_PER_BLOCK;
    constexpr int NC = (NB - NB_TAIL) + NA;
    constexpr int STORES = BLOCKS_M * REGS;                        // of one tile's epilogue: one per row and lane
    constexpr int STORES_W = STORES > 63 ? 63 : STORES;            // (the counter has six bits: waiting for more is safe)
    static_assert(kASlots == 3 && kBSlots == 2, "slot arithmetic below");
    static_assert(NC <= N1 && NB_TAIL <= MMAS_PER_BLOCK, "one copy per MFMA at most");
    using AccT = typename std::conditional<F8, v4f, v16i>::type;
    using Frag = typename std::conditional<F8, v8i, v4i>::type;
    static_assert(KIND == KIND_F8 || KIND == KIND_I8, "8-bit codes only");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / NWN, wn = wave % NWN;
    const int rowbytes = (int)g.rowbytes;
    const int nk = rowbytes / kSlabBytes;                          // >= 3, exact (host)
    const uint32_t tiles_per_batch = (uint32_t)g.tiles_m * (uint32_t)g.tiles_n;
    const uint32_t total = tiles_per_batch * (uint32_t)g.batch;

    // ---- copy sources (32-bit byte offsets from a tile's first A / B row) and LDS targets, as in gemm_kernel
    uint32_t a_src[NA], b_src[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int p = (wave * NA + i) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((p >> 1) & 7);
        a_src[i] = (uint32_t)(p * rowbytes + c * 16);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int p = (wave * NB + i) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((p >> 1) & 7);
        const int row = WN * (p / WN) + TILES_N * (p % R) + (p / R) % TILES_N;
        b_src[i] = (uint32_t)(row * rowbytes + c * 16);
    }
    typedef __attribute__((address_space(3))) uint8_t* lds_ptr_t;
    const uint32_t lds_a_units = (uint32_t)(uintptr_t)(lds_ptr_t)(lds + wave * NA * 1024);
    const uint32_t lds_b_units = (uint32_t)(uintptr_t)(lds_ptr_t)(lds + B_BASE + wave * NB * 1024);
    auto copy_a = [&](const uint8_t* slab, int i, int slot) { dma16_uniform(slab, a_src[i], lds_a_units + slot * A_SLOT + i * 1024); };
    auto copy_b = [&](const uint8_t* slab, int i, int slot) { dma16_uniform(slab, b_src[i], lds_b_units + slot * B_SLOT + i * 1024); };

    // workgroup-wide tile number -> tile, with gemm_kernel's mapping (XCD-aware, grouped along m); the tiles of one
    // workgroup (numbers blockIdx.x + i * gridDim.x, the grid a multiple of the XCD count) stay within its XCD's range
    struct Tile { const uint8_t* a; const uint8_t* b; int64_t bidx, m0, n0; };
    auto tile_of = [&](uint32_t pid) -> Tile {
        const uint32_t per = (total + kNumXcd - 1) / kNumXcd, tall = total % kNumXcd;
        const uint32_t xcd = pid % kNumXcd, loc = pid / kNumXcd;
        pid = (tall == 0 || xcd < tall) ? xcd * per + loc : tall * per + (xcd - tall) * (per - 1) + loc;
        const int64_t bidx = __builtin_amdgcn_readfirstlane((int)(pid / tiles_per_batch));
        const uint32_t t = pid - (uint32_t)bidx * tiles_per_batch;
        constexpr uint32_t GROUP_M = 8;
        const uint32_t in_group = GROUP_M * (uint32_t)g.tiles_n;
        const uint32_t grp = t / in_group;
        const uint32_t first_m = grp * GROUP_M;
        const uint32_t gsz = min(GROUP_M, (uint32_t)g.tiles_m - first_m);
        const int64_t tile_m = __builtin_amdgcn_readfirstlane((int)(first_m + (t - grp * in_group) % gsz));
        const int64_t tile_n = __builtin_amdgcn_readfirstlane((int)((t - grp * in_group) / gsz));
        Tile o;
        o.bidx = bidx; o.m0 = tile_m * BM; o.n0 = tile_n * BN;
        o.a = g.a + (bidx * g.M + o.m0) * g.rowbytes;
        o.b = g.b + (bidx * g.N + o.n0) * g.rowbytes;
        return o;
    };

    // ---- fragments and matrix instructions (as in gemm_kernel)
    const int frow = lane & (R - 1);
    const int fkey = (frow >> 1) & 7;
    const int fsel = F8 ? (lane >> 4) : (lane >> 5);
    const int a_off = (wm * WM + frow) * kSlabBytes;
    const int b_off = B_BASE + (wn * WN + frow) * kSlabBytes;
    int coff[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) coff[s] = ((F8 ? fsel : 2 * s + fsel) ^ fkey) * 16;
    auto read_frag = [&](const uint8_t* row_ptr, int s) -> Frag {
        if constexpr (F8) {
            const v4i p0 = *reinterpret_cast<const v4i*>(row_ptr + coff[0]);
            const v4i p1 = *reinterpret_cast<const v4i*>(row_ptr + (coff[0] ^ 64));
            return v8i{p0[0], p0[1], p0[2], p0[3], p1[0], p1[1], p1[2], p1[3]};
        } else {
            return *reinterpret_cast<const v4i*>(row_ptr + coff[s]);
        }
    };
    // FIRST (a tile's first slab): the product alone, with the constant 0 as the addend, written to the accumulator
    // block as a fresh value.  So the accumulators are never initialised by separate instructions (whose 128 zeros
    // passed through vector registers next to the live fragments) and no value of theirs is carried around the loop.
    auto mma = [&](const Frag& fa, const Frag& fb, AccT& c, auto first_tag) {
        constexpr bool FIRST = decltype(first_tag)::value;
#if defined(__HIP_DEVICE_COMPILE__)
        if constexpr (FIRST) {
            if constexpr (F8) {
                if constexpr (FA == QMM_FMT_E5M2 && FB == QMM_FMT_E5M2)
                    asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, 0 cbsz:1 blgp:1" : "=a"(c) : "v"(fa), "v"(fb));
                else if constexpr (FA == QMM_FMT_E5M2)
                    asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, 0 cbsz:1" : "=a"(c) : "v"(fa), "v"(fb));
                else if constexpr (FB == QMM_FMT_E5M2)
                    asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, 0 blgp:1" : "=a"(c) : "v"(fa), "v"(fb));
                else
                    asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, 0" : "=a"(c) : "v"(fa), "v"(fb));
            } else {
                asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, 0" : "=a"(c) : "v"(fa), "v"(fb));
            }
        } else {
            if constexpr (F8) {
                if constexpr (FA == QMM_FMT_E5M2 && FB == QMM_FMT_E5M2)
                    asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:1 blgp:1" : "+a"(c) : "v"(fa), "v"(fb));
                else if constexpr (FA == QMM_FMT_E5M2)
                    asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:1" : "+a"(c) : "v"(fa), "v"(fb));
                else if constexpr (FB == QMM_FMT_E5M2)
                    asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 blgp:1" : "+a"(c) : "v"(fa), "v"(fb));
                else
                    asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(c) : "v"(fa), "v"(fb));
            } else {
                asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+a"(c) : "v"(fa), "v"(fb));
            }
        }
#endif
    };
    AccT acc[BLOCKS_M][TILES_N];
    Frag fb[KS][TILES_N];      // B fragments of the current slab
    Frag fa[2][KS];            // A fragments of one block, ping-pong between blocks
    auto read_a = [&](int slot, int i, int buf) {
        const uint8_t* sa = lds + slot * A_SLOT + a_off + i * R * kSlabBytes;
#pragma unroll
        for (int s = 0; s < KS; ++s) fa[buf][s] = read_frag(sa, s);
    };

    const uint32_t stride = gridDim.x;
    uint32_t t_cur = blockIdx.x;
    if (t_cur >= total) return;
    // Two phases.  Every workgroup has the same work, so left alone all 256 reach their tile boundaries together and
    // 33 MB of output leave at once: a wavefront's copies behind its stores are only known to have landed when those
    // stores have drained (one in-order counter), so the matrix units idle while memory takes the burst.  With every
    // other workgroup of an XCD some 4 us behind, half of the chip stores while the other half multiplies.  Worth its
    // idle start from four tiles per workgroup on (host); measured on 16384 x 4096 x 1024, launches back to back:
    // 69 -> 62 us (more phases or other offsets: the same within noise).
    if (g.stagger > 0 && ((blockIdx.x / kNumXcd) & 1u))
        for (int i = 0; i < g.stagger; ++i) __builtin_amdgcn_s_sleep(8);       // 512 cycles each
    Tile cur = tile_of(t_cur);

    // ---- prologue of the stream: slab 0 of both operands, then what the steps before a tile's first step request
    // for it (A slab 1, B slab 1) and what is requested in front of the stores at a tile boundary (A slab 2)
#pragma unroll
    for (int i = 0; i < NA; ++i) copy_a(cur.a, i, 0);
#pragma unroll
    for (int i = 0; i < NB; ++i) copy_b(cur.b, i, 0);
#pragma unroll
    for (int i = 0; i < NA; ++i) copy_a(cur.a + kSlabBytes, i, 1);
#pragma unroll
    for (int i = 0; i < NB; ++i) copy_b(cur.b + kSlabBytes, i, 1);
#pragma unroll
    for (int i = 0; i < NA; ++i) copy_a(cur.a + 2 * kSlabBytes, i, 2);
    wait_vm<NA + NB + NA>();
    __syncthreads();
    // The two step sizes of the plain case (one per operand), fetched here and moved
    // to scalar registers at once: inside the loop there is then no load the compiler knows of, only stores -- with
    // both kinds outstanding it places full waits (vmcnt(0)) in front of the first use of a loaded register, and on
    // the way round the loop such a wait landed in the first step of every tile, behind all of the stores.
    const float delta_a = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, g.da[0])));
    const float delta_b = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, g.db[0])));
    // any other granularity: the step sizes are fetched per tile, in the epilogue
    const bool scales_in_loop = g.da_per_channel || g.db_per_channel || g.da_groups != 1 || g.db_groups != 1;

    // step sizes of the current tile when they are not one per operand: rows lane and 64 + lane, the lane's columns
    float sc_a0 = 0.0f, sc_a1 = 0.0f, sc_b0 = 0.0f, sc_b1 = 0.0f, sc_b2 = 0.0f, sc_b3 = 0.0f;
    int a_slot = 0, b_slot = 0;                // ring slots of the stream's current slab
    for (;;) {
        const uint32_t t_next = t_cur + stride;
        const bool has_next = t_next < total;
        Tile nxt = cur;        // set behind the tile's first step (first wanted two steps before the tile's end)
        // The fragments of the tile's first slab are read here, not at the end of the tile before (its last step's
        // barrier made them available): across the epilogue they would hold 48 registers that it needs.
        {
            const uint8_t* sb = lds + b_slot * B_SLOT + b_off;
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int j = 0; j < TILES_N; ++j) fb[s][j] = read_frag(sb + j * R * kSlabBytes, s);
        }
        read_a(a_slot, 0, 0);
        __builtin_amdgcn_sched_barrier(0);

        // One step of the stream (slab kt of the current tile).  The slabs after it are the current tile's, or the
        // first ones of the next tile.  STEADY: slabs +1 and +2 exist, every copy is requested without a test.
        // START: a tile's first step: its copies were requested in front of the stores of the tile before (in the
        // prologue for the first tile), and its matrix instructions start the accumulators.
        // (One chain of steps per tile, without alternatives: where the flow of control split over whole steps, the
        // accumulator blocks that met again behind them were moved through vector registers and memory.)
        auto step = [&](int kt, auto steady_tag, auto start_tag, auto last_tag) {
            constexpr bool STEADY = decltype(steady_tag)::value, START = decltype(start_tag)::value;
            constexpr bool LAST = decltype(last_tag)::value;      // a tile's last step: the next slab's fragments are not read
            constexpr bool START_OR_FIRST = START;
            const bool in1 = kt + 1 < nk, in2 = kt + 2 < nk;
            const bool more = STEADY || has_next || in1, more2 = STEADY || has_next || in2;
            const uint8_t* pb1 = in1 ? cur.b + (kt + 1) * kSlabBytes : nxt.b + (kt + 1 - nk) * kSlabBytes;
            const uint8_t* pa2 = in2 ? cur.a + (kt + 2) * kSlabBytes : nxt.a + (kt + 2 - nk) * kSlabBytes;
            const uint8_t* pb2 = in2 ? cur.b + (kt + 2) * kSlabBytes : nxt.b + (kt + 2 - nk) * kSlabBytes;
            const int a_next = a_slot == 2 ? 0 : a_slot + 1;
            const int a_free = a_slot == 0 ? 2 : a_slot - 1;
            auto copy_before_e = [&](int c) {
                if (c < NB - NB_TAIL) { if (more) copy_b(pb1, NB_TAIL + c, b_slot ^ 1); }
                else { if (more2) copy_a(pa2, c - (NB - NB_TAIL), a_free); }
            };
#pragma unroll
            for (int i = 0; i < BLOCKS_M - 1; ++i) {
#pragma unroll
                for (int s = 0; s < KS; ++s)
#pragma unroll
                    for (int j = 0; j < TILES_N; ++j) {
                        const int q = s * TILES_N + j;
                        const int m = i * MMAS_PER_BLOCK + q;
                        if (START_OR_FIRST && s == 0) mma(fa[i & 1][s], fb[s][j], acc[i][j], std::true_type{});
                        else mma(fa[i & 1][s], fb[s][j], acc[i][j], std::false_type{});
                        if (q == 0) {
                            __builtin_amdgcn_sched_barrier(0);
                            read_a(a_slot, i + 1, (i + 1) & 1);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        if constexpr (!START) {
#pragma unroll
                            for (int c = 0; c < NC; ++c)
                                if ((c * N1) / NC == m) {
                                    __builtin_amdgcn_sched_barrier(0);
                                    copy_before_e(c);
                                    __builtin_amdgcn_sched_barrier(0);
                                }
                        }
                    }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (more) {
                // E: every LDS read of this slab has completed and the next slab has landed
                if constexpr (START) {
                    // the newest operations are the stores of the tile before; for the first tile, the copies of A slab 2
                    if (t_cur == blockIdx.x) wait_vm_lgkm<NA>(); else wait_vm_lgkm<STORES_W>();
                } else {
                    if (more2) wait_vm_lgkm<NA>(); else wait_vm_lgkm<0>();
                }
                __syncthreads();
                if constexpr (!LAST) read_a(a_next, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            const uint8_t* sb_next = lds + (b_slot ^ 1) * B_SLOT + b_off;
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int j = 0; j < TILES_N; ++j) {
                    const int q = s * TILES_N + j;
                    if (START_OR_FIRST && s == 0) mma(fa[(BLOCKS_M - 1) & 1][s], fb[s][j], acc[BLOCKS_M - 1][j], std::true_type{});
                    else mma(fa[(BLOCKS_M - 1) & 1][s], fb[s][j], acc[BLOCKS_M - 1][j], std::false_type{});
                    if constexpr (!LAST) { if (more) fb[s][j] = read_frag(sb_next + j * R * kSlabBytes, s); }
#pragma unroll
                    for (int c = 0; c < NB_TAIL; ++c)
                        if ((c * MMAS_PER_BLOCK) / NB_TAIL == q) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (more2) copy_b(pb2, c, b_slot);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                }
            __builtin_amdgcn_sched_barrier(0);
            a_slot = a_next;
            b_slot ^= 1;
        };
        using T = std::true_type; using F = std::false_type;
        step(0, T{}, T{}, F{});
        // Step sizes per channel or batch group of this tile: requested here, behind the first step's wait (whose count
        // is exact) and in front of the second step's copies, by loads the compiler does not see and nobody waits for:
        // the second step's wait allows only its newest copies outstanding, so these have landed from then on, and
        // they are first used in the epilogue.  Six registers across the tile (four with INT8).
        if (scales_in_loop) {
            const uint32_t ga = ((uint32_t)cur.bidx / (uint32_t)g.da_inner) % (uint32_t)g.da_groups;
            const uint32_t gb = ((uint32_t)cur.bidx / (uint32_t)g.db_inner) % (uint32_t)g.db_groups;
            int lane_s = lane;
            asm volatile("" : "+v"(lane_s));
            const float* pa = g.da + (g.da_per_channel ? (int64_t)ga * g.M + cur.m0 + wm * WM + lane_s : (int64_t)ga);
            const float* pa1 = g.da_per_channel ? pa + 64 : pa;
            const float* pb = g.db + (g.db_per_channel ? (int64_t)gb * g.N + cur.n0 + wn * WN + TILES_N * (lane_s & (R - 1)) : (int64_t)gb);
#if defined(__HIP_DEVICE_COMPILE__)
            // (in-out operands: the loads write the very registers that are carried round the tile loop, so that no copy of
            // a register that has not landed yet is made behind them; build --check-asm looks for such reads)
            asm volatile("global_load_dword %0, %2, off\n\tglobal_load_dword %1, %3, off"
                         : "+v"(sc_a0), "+v"(sc_a1) : "v"(pa), "v"(pa1));
            // (one register per load -- a vector's registers were copied behind the load -- and one statement whatever the
            // granularity -- registers that met behind a branch were copied there: with one step size per group the
            // lane's four loads read the same word)
            const float* pb1 = g.db_per_channel ? pb + 1 : pb;
            if constexpr (F8) {
                const float* pb2 = g.db_per_channel ? pb + 2 : pb;
                const float* pb3 = g.db_per_channel ? pb + 3 : pb;
                asm volatile("global_load_dword %0, %4, off\n\tglobal_load_dword %1, %5, off\n\t"
                             "global_load_dword %2, %6, off\n\tglobal_load_dword %3, %7, off"
                             : "+v"(sc_b0), "+v"(sc_b1), "+v"(sc_b2), "+v"(sc_b3) : "v"(pb), "v"(pb1), "v"(pb2), "v"(pb3));
            } else {
                asm volatile("global_load_dword %0, %2, off\n\tglobal_load_dword %1, %3, off"
                             : "+v"(sc_b0), "+v"(sc_b1) : "v"(pb), "v"(pb1));
            }
#endif
        }
        // the next tile's coordinates: a few hundred scalar and vector instructions (divisions), here behind matrix
        // instructions already issued rather than between the epilogue and the first of them
        if (has_next) nxt = tile_of(t_next);
        for (int kt = 1; kt < nk - 2; ++kt) step(kt, T{}, F{}, F{});
        step(nk - 2, F{}, F{}, F{});
        step(nk - 1, F{}, F{}, T{});

        // what the next tile's first step would request before its barrier: the second half of its B slab 1 and its
        // A slab 2 (a_slot, b_slot now belong to its slab 0); then the wait states between the last matrix
        // instruction and the first read of an accumulator
        auto before_stores = [&]() {
            if (has_next) {
                const int a_free = a_slot == 0 ? 2 : a_slot - 1;
#pragma unroll
                for (int c = 0; c < NB - NB_TAIL; ++c) copy_b(nxt.b + kSlabBytes, NB_TAIL + c, b_slot ^ 1);
#pragma unroll
                for (int i = 0; i < NA; ++i) copy_a(nxt.a + 2 * kSlabBytes, i, a_free);
            }
            asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
        };
        const int64_t m_base = cur.m0 + wm * WM, n_base = cur.n0 + wn * WN;
        int lane_e = lane;                    // kept out of the loop-invariant code the compiler would hoist
        asm volatile("" : "+v"(lane_e));
        const int64_t n = n_base + TILES_N * (lane_e & (R - 1));
        const int lane_row = F8 ? 4 * (lane_e >> 4) : 4 * (lane_e >> 5);
        auto row_in_block = [&](int r) -> int { return F8 ? lane_row + r : 8 * (r >> 2) + lane_row + (r & 3); };
        auto accumulator = [&](int ia, int r, int tt) -> float {
            uint32_t raw;
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(raw) : "a"(acc[ia][tt][r]));
            if constexpr (KIND == KIND_I8) return (float)(int32_t)raw;
            else return __uint_as_float(raw);
        };
        // the stores of a whole tile; value(ia, r, tt) = the descaled element of A block ia, register r, column tt.
        // Streaming (nontemporal) stores: the 100-270 MB outputs of these shapes then leave for memory while this
        // kernel, which leaves most of the HBM bandwidth unused, is still running.  With ordinary stores much of an
        // output stays behind as dirty cache lines whose write-back competes with the reads of whatever pass comes
        // next: measured on the benchmark's step, this kernel takes 2 (QKV) and 7 us (FFN1) longer and the metric
        // pass over the four outputs 20 us less.
        auto store_tile = [&](auto&& value) {
            if (g.y_bf16) {
                uint8_t* ybase = static_cast<uint8_t*>(g.y) + ((cur.bidx * g.M + m_base) * g.N + n) * 2;
                const int64_t row_bytes = g.N * 2;
                typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
                typedef float f2 __attribute__((ext_vector_type(2)));
#pragma unroll
                for (int ia = 0; ia < BLOCKS_M; ++ia) {
#pragma unroll
                    for (int r = 0; r < REGS; ++r) {
                        uint32_t pk[TILES_N / 2];
#pragma unroll
                        for (int q = 0; q < TILES_N / 2; ++q) {
                            const float v0 = value(ia, r, 2 * q), v1 = value(ia, r, 2 * q + 1);
                            pk[q] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{v0, v1}, bf2));
                        }
                        uint8_t* dst = ybase + (ia * R + row_in_block(r)) * row_bytes;
                        if constexpr (TILES_N == 4) __builtin_nontemporal_store(u32x2{pk[0], pk[1]}, reinterpret_cast<u32x2*>(dst));
                        else __builtin_nontemporal_store(pk[0], reinterpret_cast<uint32_t*>(dst));
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                float* ybase = static_cast<float*>(g.y) + (cur.bidx * g.M + m_base) * g.N + n;
#pragma unroll
                for (int ia = 0; ia < BLOCKS_M; ++ia) {
#pragma unroll
                    for (int r = 0; r < REGS; ++r) {
                        float* dst = ybase + (int64_t)(ia * R + row_in_block(r)) * g.N;
                        if constexpr (TILES_N == 4) {
                            v4f v;
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] = value(ia, r, e);
                            __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(dst));
                        } else {
                            typedef float f2 __attribute__((ext_vector_type(2)));
                            __builtin_nontemporal_store(f2{value(ia, r, 0), value(ia, r, 1)}, reinterpret_cast<f2*>(dst));
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        // ---- epilogue of a whole tile: (acc * deltaA[row]) * deltaB[column], in that order
        if (!scales_in_loop) {
            before_stores();
            store_tile([&](int ia, int r, int tt) -> float { return (accumulator(ia, r, tt) * delta_a) * delta_b; });
        } else {
            // Step sizes per channel or per batch group were requested behind the tile's first step (above) and have
            // landed long since: every later step's wait left only operations newer than them outstanding.  A lane
            // holds the step sizes of rows lane and 64 + lane of the wavefront's 128; the one for an accumulator's row
            // comes across the lanes (ds_bpermute: no LDS memory, no vector-memory operation between the stores).
            auto finish = [&](auto a_tag, auto b_tag) {
                constexpr bool A_PC = decltype(a_tag)::value, B_PC = decltype(b_tag)::value;
                before_stores();
                store_tile([&](int ia, int r, int tt) -> float {
                    float sl, sr;
                    if constexpr (A_PC) {
                        const int row = ia * R + row_in_block(r);                  // 0 .. 127, rows < 64 for the first half of the blocks
                        const int got = __builtin_amdgcn_ds_bpermute((row & 63) * 4, __builtin_bit_cast(int, ia * R < 64 ? sc_a0 : sc_a1));
                        sl = __builtin_bit_cast(float, got);
                    } else sl = sc_a0;
                    if constexpr (B_PC) sr = tt == 0 ? sc_b0 : tt == 1 ? sc_b1 : tt == 2 ? sc_b2 : sc_b3; else sr = sc_b0;
                    return (accumulator(ia, r, tt) * sl) * sr;
                });
            };
            using T2 = std::true_type; using F2 = std::false_type;
            if (g.da_per_channel) { if (g.db_per_channel) finish(T2{}, T2{}); else finish(T2{}, F2{}); }
            else { if (g.db_per_channel) finish(F2{}, T2{}); else finish(F2{}, F2{}); }
        }
        if (!has_next) break;
        cur = nxt; t_cur = t_next;
    }
}

// An output at most 64 wide or high (attention: probabilities x values, N = head dimension) makes the product
// HBM-bound: the long operand is read exactly once and nothing of it is reused, so staging it in LDS buys nothing,
// while a 128 x 128 tile wastes half its columns and its ring admits two workgroups per CU at most.  Here a
// wavefront loads the fragments of its 64 x 64 block straight from global memory into registers (a lane fetches two
// 16-byte pieces (FP8) or 64 contiguous bytes (INT8) of a row per slab: whole 128-byte lines per row across the
// lanes; which K bytes a lane holds has to agree between the two operands, and for FP8 it is the LDS kernels'
// assignment so that the accumulators come out the same), with no barrier and no LDS, so a dozen wavefronts per
// CU overlap each other's loads and stores.  The four wavefronts of a workgroup lie along the long side of the
// output (blocks of 32 rows, i.e. twice the wavefronts, were slower: every wavefront re-reads the short operand).
// Accumulator and store layout are those of gemm_kernel (a lane owns TILES_N consecutive columns of a row).
// (Not for short contractions with a large output, e.g. attention scores: there every operand row is wanted by many
// blocks, and fetching fragments per block through the vector memory path -- sixteen row segments per instruction
// -- is slower than one LDS copy per workgroup; measured 95 us against 78 us for Q K^T of BERT-large.)
template <int KIND, int FA, int FB>
__global__ void __launch_bounds__(256)
gemm_direct_kernel(GemmArgs g)
{
    constexpr bool F8 = (KIND == KIND_F8);
    constexpr int R = F8 ? 16 : 32;
    constexpr int WM = 64, WN = 64;
    constexpr int BLOCKS_M = WM / R, TILES_N = WN / R;
    constexpr int KS = F8 ? 1 : 4;
    constexpr int REGS = F8 ? 4 : 16;
    using AccT = typename std::conditional<F8, v4f, typename std::conditional<KIND == KIND_I8, v16i, v16f>::type>::type;
    using Frag = typename std::conditional<F8, v8i, v4i>::type;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // the workgroup's wavefronts: 4 x 1 (along m) or 1 x 4 (along n)
    const int wm = g.direct_along_n ? 0 : wave, wn = g.direct_along_n ? wave : 0;
    const int BM = g.direct_along_n ? WM : 4 * WM, BN = g.direct_along_n ? 4 * WN : WN;

    const uint32_t tiles_per_batch = (uint32_t)g.tiles_m * (uint32_t)g.tiles_n;
    const uint32_t total = tiles_per_batch * (uint32_t)g.batch;
    uint32_t pid = blockIdx.x;
    {   // each XCD (own L2) takes one contiguous range of the tile sequence
        const uint32_t per = (total + kNumXcd - 1) / kNumXcd, tall = total % kNumXcd;
        const uint32_t xcd = pid % kNumXcd, loc = pid / kNumXcd;
        pid = (tall == 0 || xcd < tall) ? xcd * per + loc : tall * per + (xcd - tall) * (per - 1) + loc;
    }
    const int64_t bidx = __builtin_amdgcn_readfirstlane((int)(pid / tiles_per_batch));
    const uint32_t t = pid - (uint32_t)bidx * tiles_per_batch;
    const int64_t tile_m = __builtin_amdgcn_readfirstlane((int)(t / (uint32_t)g.tiles_n));
    const int64_t tile_n = __builtin_amdgcn_readfirstlane((int)(t % (uint32_t)g.tiles_n));
    const int64_t m_base = tile_m * BM + wm * WM, n_base = tile_n * BN + wn * WN;
    if (m_base >= g.M || n_base >= g.N) return;          // nothing of this wavefront's block lies inside the output

    // lane (r, h): row r of an operand block.  FP8 (h = 0..3): K bytes [16 h, 16 h + 16) and [64 + 16 h, 64 + 16 h + 16)
    // of a slab, the assignment of the LDS kernels' fragments -- the matrix instruction adds its operand registers up in
    // a fixed order, so with the same assignment every kernel returns the same accumulators for the same codes (and a
    // load instruction covers 64 contiguous bytes of each row).  INT8 (h = 0, 1): K bytes [64 h, 64 h + 64).
    const int frow = lane & (R - 1);
    const int fsel = F8 ? (lane >> 4) : (lane >> 5);
    const int kofs = fsel * (F8 ? 16 : 64);
    const int rowbytes = (int)g.rowbytes;
    const uint8_t* a_rows[BLOCKS_M];
    const uint8_t* b_rows[TILES_N];
#pragma unroll
    for (int i = 0; i < BLOCKS_M; ++i) {
        int64_t row = m_base + i * R + frow;
        row = row < g.M ? row : g.M - 1;
        a_rows[i] = g.a + (bidx * g.M + row) * g.rowbytes + kofs;
    }
#pragma unroll
    for (int j = 0; j < TILES_N; ++j) {
        int64_t row = n_base + TILES_N * frow + j;      // block j, lane row r  <->  output column TILES_N * r + j
        row = row < g.N ? row : g.N - 1;
        b_rows[j] = g.b + (bidx * g.N + row) * g.rowbytes + kofs;
    }

    AccT acc[BLOCKS_M][TILES_N];
#pragma unroll
    for (int i = 0; i < BLOCKS_M; ++i)
#pragma unroll
        for (int j = 0; j < TILES_N; ++j)
#pragma unroll
            for (int e = 0; e < REGS; ++e) acc[i][j][e] = 0;

    // 16 bytes at byte k of a row, zeros past the end of the row (K is a multiple of 16 bytes: host check)
    auto load16 = [&](const uint8_t* row_ptr, int k) -> v4i {
        if (k + kofs < rowbytes) return *reinterpret_cast<const v4i*>(row_ptr + k);
        return v4i{0, 0, 0, 0};
    };
    auto load_frags = [&](const uint8_t* row_ptr, int k0, Frag (&f)[KS]) {
        if constexpr (F8) {
            const v4i p0 = load16(row_ptr, k0), p1 = load16(row_ptr, k0 + 64);
            f[0] = v8i{p0[0], p0[1], p0[2], p0[3], p1[0], p1[1], p1[2], p1[3]};
        } else {
#pragma unroll
            for (int s = 0; s < KS; ++s) f[s] = load16(row_ptr, k0 + 16 * s);
        }
    };
    auto mma = [&](const Frag& fa, const Frag& fb, AccT& c) {
        if constexpr (F8) {
            c = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fa, fb, c, FA == QMM_FMT_E5M2 ? 1 : 0,
                                                                 FB == QMM_FMT_E5M2 ? 1 : 0, 0, 0, 0, 0);
        } else if constexpr (KIND == KIND_I8) {
            c = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb, c, 0, 0, 0);
        } else {
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, fa), __builtin_bit_cast(v8bf, fb), c, 0, 0, 0);
        }
    };

    for (int k0 = 0; k0 < rowbytes; k0 += kSlabBytes) {
        Frag fa[BLOCKS_M][KS], fb[TILES_N][KS];
#pragma unroll
        for (int j = 0; j < TILES_N; ++j) load_frags(b_rows[j], k0, fb[j]);
#pragma unroll
        for (int i = 0; i < BLOCKS_M; ++i) load_frags(a_rows[i], k0, fa[i]);
#pragma unroll
        for (int i = 0; i < BLOCKS_M; ++i)
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int j = 0; j < TILES_N; ++j) mma(fa[i][s], fb[j][s], acc[i][j]);
    }

    // ---- epilogue: (acc * deltaA[row]) * deltaB[column], in that order
    const float* da = g.da ? g.da + ((bidx / g.da_inner) % g.da_groups) * (g.da_per_channel ? g.M : 1) : nullptr;
    const float* db = g.db ? g.db + ((bidx / g.db_inner) % g.db_groups) * (g.db_per_channel ? g.N : 1) : nullptr;
    constexpr bool descale = (KIND != KIND_BF16);
    const int64_t n = n_base + TILES_N * (lane & (R - 1));
    const int lane_row = F8 ? 4 * (lane >> 4) : 4 * (lane >> 5);
    float sr[TILES_N];
#pragma unroll
    for (int tt = 0; tt < TILES_N; ++tt) {
        sr[tt] = 1.0f;
        if constexpr (descale) sr[tt] = g.db_per_channel ? db[(n + tt) < g.N ? (n + tt) : (g.N - 1)] : db[0];
    }
    float sa_scalar = 1.0f;
    if constexpr (descale) { if (!g.da_per_channel) sa_scalar = da[0]; }
    auto row_in_block = [&](int r) -> int { return F8 ? lane_row + r : 8 * (r >> 2) + lane_row + (r & 3); };
    auto raw_of = [&](int ia, int r, int tt) -> uint32_t {
        if constexpr (KIND == KIND_I8) return (uint32_t)acc[ia][tt][r];
        else return __float_as_uint(acc[ia][tt][r]);
    };
    auto value = [&](int ia, int r, int tt, float sl) -> float {
        float a;
        if constexpr (KIND == KIND_I8) a = (float)acc[ia][tt][r];
        else a = acc[ia][tt][r];
        if constexpr (descale) a = (a * sl) * sr[tt];
        return a;
    };
    const bool interior = (m_base + WM <= g.M) && (n_base + WN <= g.N) && (g.N % TILES_N == 0);
    const bool fast = interior && g.y && !g.acc_out;
    // row step sizes are fetched before the first store (loads and stores share one in-order counter)
    float sl_rows[BLOCKS_M][REGS];
#pragma unroll
    for (int ia = 0; ia < BLOCKS_M; ++ia)
#pragma unroll
        for (int r = 0; r < REGS; ++r) {
            sl_rows[ia][r] = sa_scalar;
            if constexpr (descale) {
                if (g.da_per_channel) {
                    const int64_t m = m_base + ia * R + row_in_block(r);
                    sl_rows[ia][r] = da[m < g.M ? m : g.M - 1];
                }
            }
        }
    if (fast && g.y_bf16) {
        uint8_t* ybase = static_cast<uint8_t*>(g.y) + ((bidx * g.M + m_base) * g.N + n) * 2;
#pragma unroll
        for (int ia = 0; ia < BLOCKS_M; ++ia)
#pragma unroll
            for (int r = 0; r < REGS; ++r) {
                typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
                typedef float f2 __attribute__((ext_vector_type(2)));
                uint32_t pk[TILES_N / 2];
#pragma unroll
                for (int q = 0; q < TILES_N / 2; ++q)
                    pk[q] = __builtin_bit_cast(uint32_t, __builtin_convertvector(
                        f2{value(ia, r, 2 * q, sl_rows[ia][r]), value(ia, r, 2 * q + 1, sl_rows[ia][r])}, bf2));
                uint8_t* dst = ybase + (int64_t)(ia * R + row_in_block(r)) * g.N * 2;
                if constexpr (TILES_N == 4) *reinterpret_cast<u32x2*>(dst) = u32x2{pk[0], pk[1]};
                else *reinterpret_cast<uint32_t*>(dst) = pk[0];
            }
    } else if (fast && TILES_N == 4) {
        float* ybase = static_cast<float*>(g.y) + (bidx * g.M + m_base) * g.N + n;
#pragma unroll
        for (int ia = 0; ia < BLOCKS_M; ++ia)
#pragma unroll
            for (int r = 0; r < REGS; ++r) {
                v4f v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = value(ia, r, e < TILES_N ? e : 0, sl_rows[ia][r]);
                *reinterpret_cast<v4f*>(ybase + (int64_t)(ia * R + row_in_block(r)) * g.N) = v;
            }
    } else if (n < g.N) {
#pragma unroll
        for (int ia = 0; ia < BLOCKS_M; ++ia)
#pragma unroll
            for (int r = 0; r < REGS; ++r) {
                const int64_t m = m_base + ia * R + row_in_block(r);
                if (m < g.M) {
                    const int64_t o = (bidx * g.M + m) * g.N + n;
#pragma unroll
                    for (int tt = 0; tt < TILES_N; ++tt) {
                        if (n + tt < g.N) {
                            const float v = value(ia, r, tt, sl_rows[ia][r]);
                            if (g.acc_out) static_cast<uint32_t*>(g.acc_out)[o + tt] = raw_of(ia, r, tt);
                            if (g.y) {
                                if (g.y_bf16) static_cast<__bf16*>(g.y)[o + tt] = (__bf16)v;
                                else static_cast<float*>(g.y)[o + tt] = v;
                            }
                        }
                    }
                }
            }
    }
}

// Second kernel of split-K: out = descale(sum over the K ranges, in ascending order, of the partial accumulators).
// INT8 partials are integers (the sum is exact); FP8 / bfloat16 partials are binary32 and added in binary32.
// One thread per four consecutive columns.
template <int KIND>
__global__ void __launch_bounds__(256)
splitk_reduce(GemmArgs g)
{
    const int64_t quads_per_row = (g.N + 3) / 4;
    const int64_t total = g.batch * g.M * quads_per_row;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= total) return;
    const int64_t row = id / quads_per_row, n = (id - row * quads_per_row) * 4;     // row = b * M + m
    const int64_t bidx = row / g.M, m = row - bidx * g.M;
    const int64_t plane = g.batch * g.M * g.N;
    const bool full = (n + 4 <= g.N) && (g.N % 4 == 0);
    int32_t si[4] = {0, 0, 0, 0};
    float sf[4] = {0.f, 0.f, 0.f, 0.f};
    for (int sp = 0; sp < g.splits; ++sp) {
        const uint32_t* p = static_cast<const uint32_t*>(g.partial) + sp * plane + row * g.N + n;
        uint32_t v[4] = {0u, 0u, 0u, 0u};
        if (full) {
            const u32x4 q = *reinterpret_cast<const u32x4*>(p);
            v[0] = q[0]; v[1] = q[1]; v[2] = q[2]; v[3] = q[3];
        } else {
            for (int e = 0; e < 4; ++e)
                if (n + e < g.N) v[e] = p[e];
        }
        for (int e = 0; e < 4; ++e) {
            if constexpr (KIND == KIND_I8) si[e] += (int32_t)v[e];
            else sf[e] = sp == 0 ? __uint_as_float(v[e]) : sf[e] + __uint_as_float(v[e]);
        }
    }
    float sl = 1.0f;
    if constexpr (KIND != KIND_BF16) sl = g.da[((bidx / g.da_inner) % g.da_groups) * (g.da_per_channel ? g.M : 1) + (g.da_per_channel ? m : 0)];
    for (int e = 0; e < 4; ++e) {
        if (n + e >= g.N) break;
        float a;
        uint32_t raw;
        if constexpr (KIND == KIND_I8) { raw = (uint32_t)si[e]; a = (float)si[e]; }
        else { raw = __float_as_uint(sf[e]); a = sf[e]; }
        if constexpr (KIND != KIND_BF16) {
            const float sr = g.db[((bidx / g.db_inner) % g.db_groups) * (g.db_per_channel ? g.N : 1) + (g.db_per_channel ? n + e : 0)];
            a = (a * sl) * sr;
        }
        const int64_t o = row * g.N + n + e;
        if (g.acc_out) static_cast<uint32_t*>(g.acc_out)[o] = raw;
        if (g.y) {
            if (g.y_bf16) static_cast<__bf16*>(g.y)[o] = (__bf16)a;
            else static_cast<float*>(g.y)[o] = a;
        }
    }
}

// Split-K plan: used when 128 x 128 tiles would not give every CU its two workgroups and K is long (weight-gradient
// shapes: small output, contraction over all tokens).  Returns the number of K ranges (1 = no split).  The ranges run
// as workgroups of the 128 x 128 kernel, about 512 of them (two per CU): measured on 1024 x 1024 x 16384 that takes
// 29 us where sixteen ranges of 256 x 256 tiles took 37 (half as many partial sums for the second pass to add), and on
// 3072 x 1024 x 16384 two ranges take 60 us where the unsplit product took 65; from 256 small tiles on (4096 x 1024)
// the second pass costs more than the idle halves of the CUs.
int plan_splits(int64_t M, int64_t N, int64_t rowbytes, int64_t batch, int fuse)
{
    if (fuse != 0) return 1;
    const int64_t small = ((M + 127) / 128) * ((N + 127) / 128) * batch;
    const int64_t nslabs = (rowbytes + kSlabBytes - 1) / kSlabBytes;
    if (small >= 256 || nslabs < 16) return 1;
    int64_t splits = 512 / small;
    if (splits > nslabs / 8) splits = nslabs / 8;      // at least eight slabs per range
    return splits >= 2 ? (int)splits : 1;
}

// The dynamic-LDS limit of a kernel is a property of the function on one device: it is applied once per
// (instantiation, device), the devices already served kept as a bit mask (devices past 63 are served on every call).
// Two host threads that meet here both apply it, which is harmless; nothing else is remembered between calls.
static inline bool ensure_lds_attr(std::atomic<uint64_t>& done, const void* kern, int bytes)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    const uint64_t bit = dev < 64 ? (1ull << dev) : 0;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return true;
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return false;
    if (bit) done.fetch_or(bit, std::memory_order_release);
    return true;
}

template <int KIND, int FA, int FB, int TM, int TG, int NWN, int FUSE, int NSR = 0>
qmm_status launch_tile(GemmArgs& g, hipStream_t s)
{
    constexpr int BM = kWavesM * 32 * TM, BN = NWN * 64 * TG;
    constexpr int LDS_BYTES = (kASlots * BM + kBSlots * BN) * kSlabBytes;
    g.tiles_m = (int)((g.M + BM - 1) / BM);
    g.tiles_n = (int)((g.N + BN - 1) / BN);
    const int64_t total = (int64_t)g.tiles_m * g.tiles_n * g.batch * g.splits;
    if (total > 0x7FFFFFFF) return QMM_ERR_UNSUPPORTED;
    auto kern = gemm_kernel<KIND, FA, FB, TM, TG, NWN, FUSE, NSR>;
    static std::atomic<uint64_t> lds_attr_done{0};
    if (!ensure_lds_attr(lds_attr_done, reinterpret_cast<const void*>(kern), LDS_BYTES)) return QMM_ERR_LAUNCH;
    kern<<<(unsigned)total, 64 * kWavesM * NWN, LDS_BYTES, s>>>(g);
    if constexpr (NSR != 0) {
        if (hipGetLastError() != hipSuccess) return QMM_ERR_LAUNCH;
        nsr_finalize<<<1, 256, 0, s>>>(g.nsr_partial, total * kWavesM * NWN, g.nsr_out);
    }
    if (g.splits > 1) {
        if (hipGetLastError() != hipSuccess) return QMM_ERR_LAUNCH;
        const int64_t threads = g.batch * g.M * ((g.N + 3) / 4);
        splitk_reduce<KIND><<<(unsigned)((threads + 255) / 256), 256, 0, s>>>(g);
    }
    return launch_status();
}

template <int KIND, int FA, int FB>
qmm_status launch_direct(GemmArgs& g, hipStream_t s)
{
    g.direct_along_n = (g.M <= 64 && g.N > 64) ? 1 : 0;
    const int bm = g.direct_along_n ? 64 : 256, bn = g.direct_along_n ? 256 : 64;
    g.tiles_m = (int)((g.M + bm - 1) / bm);
    g.tiles_n = (int)((g.N + bn - 1) / bn);
    const int64_t total = (int64_t)g.tiles_m * g.tiles_n * g.batch;
    if (total > 0x7FFFFFFF) return QMM_ERR_UNSUPPORTED;
    gemm_direct_kernel<KIND, FA, FB><<<(unsigned)total, 256, 0, s>>>(g);
    return launch_status();
}

// True for the shapes gemm_direct_kernel is for: codes in, no split, an output at most 64 wide or high, and enough
// 64 x 64 blocks to give every CU a couple of wavefronts.
bool use_direct(const GemmArgs& g, int fuse)
{
    if (fuse != 0 || g.splits > 1) return false;
    const int64_t blocks = ((g.M + 63) / 64) * ((g.N + 63) / 64) * g.batch;
    return blocks >= 512 && (g.M <= 64 || g.N <= 64);
}

// gemm_shortk_kernel: codes in, no split, one slab of K at most, whole 256 x 256 tiles only, output in y alone
// (binary32 only where a lane owns four columns), and at least two tiles for every workgroup of the grid.
constexpr int kShortKGrid = 256;
template <int KIND>
bool use_shortk(const GemmArgs& g, int fuse)
{
    if (fuse != 0 || g.splits > 1 || g.rowbytes > kSlabBytes) return false;
    if (g.M % 256 != 0 || g.N % 256 != 0 || !g.y || g.acc_out) return false;
    if (!g.y_bf16 && KIND != KIND_F8) return false;
    return (g.M / 256) * (g.N / 256) * g.batch >= 2 * kShortKGrid;
}

template <int KIND, int FA, int FB>
qmm_status launch_shortk(GemmArgs& g, hipStream_t s)
{
    constexpr int LDS_BYTES = 4 * 256 * kSlabBytes;
    g.tiles_m = (int)(g.M / 256);
    g.tiles_n = (int)(g.N / 256);
    if ((int64_t)g.tiles_m * g.tiles_n * g.batch > 0x7FFFFFFF) return QMM_ERR_UNSUPPORTED;
    auto kern = gemm_shortk_kernel<KIND, FA, FB>;
    static std::atomic<uint64_t> lds_attr_done{0};
    if (!ensure_lds_attr(lds_attr_done, reinterpret_cast<const void*>(kern), LDS_BYTES)) return QMM_ERR_LAUNCH;
    kern<<<kShortKGrid, 512, LDS_BYTES, s>>>(g);
    return launch_status();
}

// gemm_stream_kernel: codes in, no split, whole 256 x 256 tiles, whole slabs and at
// least three of them, output in y alone, and more tiles than workgroups in the grid (with one tile each there is nothing to overlap).
constexpr int kStreamGrid = 256;
bool use_stream(const GemmArgs& g, int fuse)
{
    if (fuse != 0 || g.splits > 1 || g.rowbytes % kSlabBytes != 0 || g.rowbytes < 3 * kSlabBytes) return false;
    if (g.M % 256 != 0 || g.N % 256 != 0 || !g.y || g.acc_out) return false;
    // (step sizes per channel are fetched four rows / columns at a time)
    if (!aligned16(g.da) || !aligned16(g.db) || g.da_groups > 0x7FFFFFFF || g.db_groups > 0x7FFFFFFF ||
        g.da_inner > 0x7FFFFFFF || g.db_inner > 0x7FFFFFFF) return false;
    return (g.M / 256) * (g.N / 256) * g.batch > kStreamGrid;
}

template <int KIND, int FA, int FB>
qmm_status launch_stream(GemmArgs& g, hipStream_t s)
{
    constexpr int LDS_BYTES = (kASlots + kBSlots) * 256 * kSlabBytes;
    g.tiles_m = (int)(g.M / 256);
    g.tiles_n = (int)(g.N / 256);
    if ((int64_t)g.tiles_m * g.tiles_n * g.batch > 0x7FFFFFFF) return QMM_ERR_UNSUPPORTED;
    g.stagger = ((int64_t)g.tiles_m * g.tiles_n * g.batch >= 4 * kStreamGrid) ? 16 : 0;
    auto kern = gemm_stream_kernel<KIND, FA, FB>;
    static std::atomic<uint64_t> lds_attr_done{0};
    if (!ensure_lds_attr(lds_attr_done, reinterpret_cast<const void*>(kern), LDS_BYTES)) return QMM_ERR_LAUNCH;
    kern<<<kStreamGrid, 512, LDS_BYTES, s>>>(g);
    return launch_status();
}

template <int KIND, int FA, int FB, int FUSE>
qmm_status launch_fuse(GemmArgs& g, hipStream_t s)
{
    if constexpr (FUSE == 0 && KIND != KIND_BF16) {
        if (g.nsr_ref) {      // the variant that also accumulates the noise-to-signal sums: gemm_kernel only, no split
            const int64_t big_tiles = ((g.M + 255) / 256) * ((g.N + 255) / 256) * g.batch;
            if (big_tiles >= 192 && g.M > 128 && g.N > 128) return launch_tile<KIND, FA, FB, 4, 1, 4, 0, 1>(g, s);
            return launch_tile<KIND, FA, FB, 2, 1, 2, 0, 1>(g, s);
        }
    }
    if (g.nsr_ref) return QMM_ERR_UNSUPPORTED;
    if constexpr (FUSE == 0) {
        if (use_direct(g, 0)) return launch_direct<KIND, FA, FB>(g, s);
        if (use_shortk<KIND>(g, 0)) return launch_shortk<KIND, FA, FB>(g, s);
        if constexpr (KIND != KIND_BF16) { if (use_stream(g, 0)) return launch_stream<KIND, FA, FB>(g, s); }
    }
    // 256 x 256 tiles (eight wavefronts, two per SIMD: while one waits at a copy or a fragment read the other
    // issues matrix instructions) when they still give every CU work, else 128 x 128 tiles (four wavefronts, two
    // workgroups per CU).
    const int64_t big = ((g.M + 255) / 256) * ((g.N + 255) / 256) * g.batch;
    // an output narrower than half a big tile wastes less of a small one
    const bool narrow = g.M <= 128 || g.N <= 128;
    if (big >= 192 && !narrow && g.splits == 1) return launch_tile<KIND, FA, FB, 4, 1, 4, FUSE>(g, s);
    return launch_tile<KIND, FA, FB, 2, 1, 2, FUSE>(g, s);
}

// fuse: bit 0 = A is quantized on load, bit 1 = B is
template <int KIND, int FA, int FB>
qmm_status launch_kind(GemmArgs& g, hipStream_t s, int fuse)
{
    if constexpr (KIND == KIND_BF16) {
        return launch_fuse<KIND, FA, FB, 0>(g, s);
    } else {
        if (fuse == 0) return launch_fuse<KIND, FA, FB, 0>(g, s);
        if (fuse == 1) return launch_fuse<KIND, FA, FB, 1>(g, s);
        if (fuse == 2) return launch_fuse<KIND, FA, FB, 2>(g, s);
        return launch_fuse<KIND, FA, FB, 3>(g, s);
    }
}

bool is8(int f) { return f == QMM_FMT_INT8 || f == QMM_FMT_E4M3 || f == QMM_FMT_E5M2; }

qmm_status check_operand(const qmm_operand* o)
{
    if (!o) return QMM_ERR_NULL;
    if (!is8(o->format) && o->format != QMM_FMT_BF16) return QMM_ERR_ENUM;
    if (o->is_codes != 0 && o->is_codes != 1) return QMM_ERR_ENUM;
    if (o->format == QMM_FMT_BF16 && o->is_codes) return QMM_ERR_ENUM;
    if (o->gran.batch_groups < 1 || o->gran.batch_inner < 0 || (o->gran.per_channel != 0 && o->gran.per_channel != 1))
        return QMM_ERR_ENUM;
    return QMM_OK;
}

}  // namespace
}  // namespace qmm

using namespace qmm;

extern "C" size_t qmm_gemm_workspace_size(const qmm_operand* a, const qmm_operand* b, int64_t batch, int64_t M, int64_t N,
                                          int64_t K)
{
    if (!a || !b || batch <= 0 || M <= 0 || N <= 0 || K <= 0) return 0;
    const bool bf = a->format == QMM_FMT_BF16;
    const int fuse = bf ? 0 : ((a->is_codes ? 0 : 1) | (b->is_codes ? 0 : 2));
    const int splits = plan_splits(M, N, K * (bf ? 2 : 1), batch, fuse);
    return splits > 1 ? (size_t)splits * (size_t)batch * (size_t)M * (size_t)N * 4u : 0;
}

namespace {
size_t nsr_workspace_bytes(int64_t batch, int64_t M, int64_t N)
{
    // a pair of binary64 sums per wavefront; 128 x 128 tiles of four wavefronts are the finest partition used
    const int64_t tiles = ((M + 127) / 128) * ((N + 127) / 128) * batch;
    return (size_t)(tiles > 0 ? tiles : 1) * 4u * 2u * sizeof(double);
}

// qmm_gemm, and with y_ref != NULL the variant that also accumulates the noise-to-signal sums into nsr_out2.
qmm_status gemm_impl(const qmm_operand* a, const qmm_operand* b, int64_t batch, int64_t M, int64_t N, int64_t K,
                     void* y, qmm_dtype y_dtype, void* acc_out, const float* y_ref, double* nsr_out2,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    const bool nsr = y_ref != nullptr;
    qmm_status st = check_operand(a);
    if (st != QMM_OK) return st;
    st = check_operand(b);
    if (st != QMM_OK) return st;
    if (y_dtype != QMM_DT_BF16 && y_dtype != QMM_DT_F32) return QMM_ERR_ENUM;
    if (batch < 0 || M < 0 || N < 0 || K < 0) return QMM_ERR_SHAPE;
    const bool bf = a->format == QMM_FMT_BF16;
    if (bf != (b->format == QMM_FMT_BF16)) return QMM_ERR_UNSUPPORTED;
    if (!bf && ((a->format == QMM_FMT_INT8) != (b->format == QMM_FMT_INT8))) return QMM_ERR_UNSUPPORTED;
    const int fuse = bf ? 0 : ((a->is_codes ? 0 : 1) | (b->is_codes ? 0 : 2));
    if (!y && !acc_out) return QMM_ERR_NULL;
    if (nsr) {
        if (bf || fuse != 0) return QMM_ERR_UNSUPPORTED;
        if (!y || !nsr_out2) return QMM_ERR_NULL;
        if (acc_out) return QMM_ERR_UNSUPPORTED;
        if (!aligned16(y_ref) || (reinterpret_cast<uintptr_t>(nsr_out2) & 7u)) return QMM_ERR_ALIGN;
        if (!workspace || workspace_bytes < nsr_workspace_bytes(batch, M, N)) return QMM_ERR_WORKSPACE;
        if (!aligned16(workspace)) return QMM_ERR_ALIGN;
    }
    if (batch * M * N == 0) return QMM_OK;
    if (!bf && (!a->delta || !b->delta)) return QMM_ERR_NULL;
    const int64_t esz = bf ? 2 : 1;
    if ((K * esz) % 16 != 0) return QMM_ERR_ALIGN;
    if (K * esz > (int64_t(1) << 22)) return QMM_ERR_UNSUPPORTED;   // the kernels keep 32-bit byte offsets within a tile's rows
    if (K > 0 && (!a->data || !b->data)) return QMM_ERR_NULL;
    if (!aligned16(a->data) || !aligned16(b->data) || (y && !aligned16(y)) || (acc_out && !aligned16(acc_out)))
        return QMM_ERR_ALIGN;

    GemmArgs g{};
    g.a = static_cast<const uint8_t*>(a->data); g.b = static_cast<const uint8_t*>(b->data);
    g.M = M; g.N = N; g.rowbytes = K * esz; g.batch = batch;
    g.da = bf ? nullptr : a->delta; g.db = bf ? nullptr : b->delta;
    g.da_groups = a->gran.batch_groups; g.db_groups = b->gran.batch_groups;
    g.da_inner = a->gran.batch_inner > 0 ? a->gran.batch_inner : 1;
    g.db_inner = b->gran.batch_inner > 0 ? b->gran.batch_inner : 1;
    g.da_per_channel = a->gran.per_channel; g.db_per_channel = b->gran.per_channel;
    g.y = y; g.y_bf16 = y_dtype == QMM_DT_BF16; g.acc_out = acc_out;
    g.splits = nsr ? 1 : plan_splits(M, N, g.rowbytes, batch, fuse);
    if (nsr) { g.nsr_ref = y_ref; g.nsr_partial = static_cast<double*>(workspace); g.nsr_out = nsr_out2; }
    if (g.splits > 1) {
        const size_t need = (size_t)g.splits * (size_t)batch * (size_t)M * (size_t)N * 4u;
        if (!workspace || workspace_bytes < need) return QMM_ERR_WORKSPACE;
        if (!aligned16(workspace)) return QMM_ERR_ALIGN;
        g.partial = workspace;
    }
    hipStream_t s = as_stream(stream);

    if (bf) return launch_kind<KIND_BF16, QMM_FMT_BF16, QMM_FMT_BF16>(g, s, 0);
    if (a->format == QMM_FMT_INT8) return launch_kind<KIND_I8, QMM_FMT_INT8, QMM_FMT_INT8>(g, s, fuse);
    if (a->format == QMM_FMT_E4M3 && b->format == QMM_FMT_E4M3) return launch_kind<KIND_F8, QMM_FMT_E4M3, QMM_FMT_E4M3>(g, s, fuse);
    if (a->format == QMM_FMT_E4M3) return launch_kind<KIND_F8, QMM_FMT_E4M3, QMM_FMT_E5M2>(g, s, fuse);
    if (b->format == QMM_FMT_E4M3) return launch_kind<KIND_F8, QMM_FMT_E5M2, QMM_FMT_E4M3>(g, s, fuse);
    return launch_kind<KIND_F8, QMM_FMT_E5M2, QMM_FMT_E5M2>(g, s, fuse);
}
}  // namespace

extern "C" qmm_status qmm_gemm(const qmm_operand* a, const qmm_operand* b, int64_t batch, int64_t M, int64_t N, int64_t K,
                               void* y, qmm_dtype y_dtype, void* acc_out, void* workspace, size_t workspace_bytes,
                               void* stream)
{
    return gemm_impl(a, b, batch, M, N, K, y, y_dtype, acc_out, nullptr, nullptr, workspace, workspace_bytes, stream);
}

extern "C" size_t qmm_gemm_nsr_workspace_size(int64_t batch, int64_t M, int64_t N)
{
    if (batch < 0 || M < 0 || N < 0) return 0;
    return nsr_workspace_bytes(batch, M, N);
}

extern "C" qmm_status qmm_gemm_nsr(const qmm_operand* a, const qmm_operand* b, int64_t batch, int64_t M, int64_t N,
                                   int64_t K, void* y, qmm_dtype y_dtype, const float* y_ref, double* out2,
                                   void* workspace, size_t workspace_bytes, void* stream)
{
    if (batch >= 0 && M >= 0 && N >= 0 && K >= 0 && batch * M * N == 0) {
        // an empty output (its pointers may be NULL): both sums are zero
        qmm_status st = check_operand(a);
        if (st != QMM_OK) return st;
        st = check_operand(b);
        if (st != QMM_OK) return st;
        if (!out2) return QMM_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(out2) & 7u) return QMM_ERR_ALIGN;
        nsr_finalize<<<1, 256, 0, as_stream(stream)>>>(nullptr, 0, out2);
        return launch_status();
    }
    if (!y_ref) return QMM_ERR_NULL;
    return gemm_impl(a, b, batch, M, N, K, y, y_dtype, nullptr, y_ref, out2, workspace, workspace_bytes, stream);
}
