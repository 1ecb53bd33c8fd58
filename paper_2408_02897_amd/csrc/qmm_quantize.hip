// qmm_quantize: codes = round(X / delta) onto INT8 / E4M3 / E5M2 (Eq. 1, left
// half; Methodology bullets on saturation, underflow and the two rounding
// modes).  HBM-bound: 2 B read + 1 B written per bfloat16 element.  The quotient
// is x * (1/delta) with one IEEE reciprocal per thread-row and one product per
// element.  Codes are written with the contracting axis contiguous; when the
// input contracts over its rows the tile is transposed through LDS.
#include <algorithm>
#include "qmm_device.h"

namespace qmm {
namespace {

constexpr int kThreads = 256;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

struct QArgs {
    const void* x;
    const float* delta;
    uint8_t* codes;
    int64_t batch, rows, cols, batch_stride, row_stride;
    int64_t groups;        // batch groups
    int64_t inner;         // consecutive matrices sharing a group: group = (b / inner) % groups
    int64_t channels;      // step sizes per group (1 when not per-channel)
    uint64_t seed, offset;
};

template <typename T> QMM_DEV float load_f32(const T* p);
template <> QMM_DEV float load_f32<uint16_t>(const uint16_t* p) { return bf16_bits_to_f32(*p); }
template <> QMM_DEV float load_f32<float>(const float* p) { return *p; }

// Row-contracting fast path: bfloat16, cols % 16 == 0, 16-byte aligned rows.  One thread = 16 consecutive
// elements of a row: two 16-byte loads, one 16-byte store.  grid (ceil(rows*cols/16 / 256), batch).
template <int FMT, int MODE> __global__ void __launch_bounds__(kThreads)
quantize_rows_bf16x16(QArgs a)
{
    const int64_t vpr = a.cols >> 4;
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (v >= vpr * a.rows) return;
    const int64_t b = blockIdx.y;
    const int64_t r = v / vpr, cv = v - r * vpr;
    const float d = a.delta[((b / a.inner) % a.groups) * a.channels + (a.channels > 1 ? r : 0)];
    const float rho = 1.0f / d;
    const u32x4* src = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(a.x) + b * a.batch_stride +
                                                      r * a.row_stride + cv * 16);
    const u32x4 w0 = src[0], w1 = src[1];
    const int64_t p0 = (b * a.rows + r) * a.cols + cv * 16;
    u32x4 out;
    if constexpr (MODE == QMM_ROUND_RTNE) {
        out = encode16_bf16_rtne<FMT>(w0, w1, rho);
    } else {
        // element number g = p0 + e + offset draws word g % 4 of Philox block g / 4.  When the thread's first element
        // starts a block (always, unless the caller's offset is not a multiple of 4) its 16 elements are exactly the
        // four blocks g0/4 .. g0/4 + 3, one per output dword; otherwise the generic stream looks each element up.
        const uint64_t g0 = (uint64_t)p0 + a.offset;
        const bool aligned = (g0 & 3u) == 0;              // uniform over the grid
        SrStream sr(a.seed);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            Philox4 blk{};
            if (aligned) {
                const uint64_t c = (g0 >> 2) + q;
                blk = philox4x32_10((uint32_t)c, (uint32_t)(c >> 32), 0u, 0u, (uint32_t)a.seed, (uint32_t)(a.seed >> 32));
            }
            uint32_t packed = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int e = q * 4 + j;
                const uint32_t word = e < 8 ? w0[e >> 1] : w1[(e - 8) >> 1];
                const float xv = (e & 1) ? __uint_as_float(word & 0xFFFF0000u) : __uint_as_float(word << 16);
                const float t = xv * rho;
                const uint32_t u24 = aligned ? blk.v[j] >> 8 : sr.bits(g0 + e);
                packed |= encode<FMT, MODE>(t, u24) << (8 * j);
            }
            out[q] = packed;
        }
    }
    *reinterpret_cast<u32x4*>(a.codes + p0) = out;
}

// Several dense bfloat16 tensors with one step size each, RTNE, rows contracting, in one launch
// (qmm_quantize_multi): blockIdx.y picks the tensor; the arithmetic is quantize_rows_bf16x16's.
constexpr int kMaxMulti = 8;
struct MultiQ {
    const uint16_t* x[kMaxMulti];
    uint8_t* codes[kMaxMulti];
    const float* delta[kMaxMulti];
    int64_t nvec16[kMaxMulti];
};
template <int FMT> __global__ void __launch_bounds__(kThreads)
quantize_flat_multi(MultiQ a)
{
    const int t = blockIdx.y;
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (v >= a.nvec16[t]) return;
    const float rho = 1.0f / a.delta[t][0];
    const u32x4* src = reinterpret_cast<const u32x4*>(a.x[t]) + 2 * v;
    const u32x4 w0 = src[0], w1 = src[1];
    reinterpret_cast<u32x4*>(a.codes[t])[v] = encode16_bf16_rtne<FMT>(w0, w1, rho);
}

// Generic path: one thread per output code, any dtype / stride / contracting axis.
template <typename T, int FMT, int MODE> __global__ void __launch_bounds__(kThreads)
quantize_generic(QArgs a, int contract_axis)
{
    const int64_t NC = contract_axis == 1 ? a.rows : a.cols;
    const int64_t KC = contract_axis == 1 ? a.cols : a.rows;
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= NC * KC) return;
    const int64_t b = blockIdx.y;
    const int64_t n = i / KC, k = i - n * KC;
    const int64_t r = contract_axis == 1 ? n : k, c = contract_axis == 1 ? k : n;
    const float d = a.delta[((b / a.inner) % a.groups) * a.channels + (a.channels > 1 ? n : 0)];
    const float rho = 1.0f / d;
    const float t = load_f32<T>(static_cast<const T*>(a.x) + b * a.batch_stride + r * a.row_stride + c) * rho;
    const int64_t p = (b * NC + n) * KC + k;
    uint32_t u24 = 0;
    if constexpr (MODE == QMM_ROUND_STOCHASTIC) {
        SrStream sr(a.seed);
        u24 = sr.bits((uint64_t)p + a.offset);
    }
    a.codes[p] = (uint8_t)encode<FMT, MODE>(t, u24);
}

// Column-contracting fast path (the input is [K][N], codes are [N][K]): bfloat16, rows % 16 == 0 is NOT
// required; cols % 8 == 0 and 16-byte aligned rows are.  Workgroup tile = 128 k x 128 n.  Thread (tn, tk)
// loads 8 rows (k) x 8 columns (n) as eight 16-byte vectors, packs the 8 codes of each column into two
// dwords and parks them in an LDS tile [n][k]; then every thread writes 16-byte pieces of finished code
// rows, 128 contiguous bytes per n.  grid (ceil(cols/128), ceil(rows/128), batch).
constexpr int kTile = 128;
constexpr int kTileRowBytes = kTile + 16;   // padded row of the LDS code tile

template <int FMT, int MODE> __global__ void __launch_bounds__(kThreads)
quantize_cols_bf16(QArgs a)
{
    __shared__ __attribute__((aligned(16))) uint8_t tile[kTile * kTileRowBytes];
    const int tn = threadIdx.x & 15, tk = threadIdx.x >> 4;
    const int64_t b = blockIdx.z;
    const int64_t n0 = (int64_t)blockIdx.x * kTile, k0 = (int64_t)blockIdx.y * kTile;
    const int64_t K = a.rows, N = a.cols;
    const int64_t n = n0 + tn * 8;
    const uint16_t* base = static_cast<const uint16_t*>(a.x) + b * a.batch_stride;
    float rho[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int64_t nn = n + j < N ? n + j : N - 1;
        rho[j] = 1.0f / a.delta[((b / a.inner) % a.groups) * a.channels + (a.channels > 1 ? nn : 0)];
    }
    uint32_t lo[8] = {}, hi[8] = {};
    SrStream sr(a.seed);
    if constexpr (MODE == QMM_ROUND_STOCHASTIC) {
        // Column by column: the eight codes of a column are consecutive output elements, i.e. two whole Philox
        // blocks when the column's first element number is a multiple of 4 (K and the caller's offset both are);
        // going row by row instead would draw a fresh block for every single element.
        if (n < N) {
            u32x4 w[8];
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const int64_t k = k0 + tk * 8 + kk;
                w[kk] = u32x4{0u, 0u, 0u, 0u};
                if (k < K) w[kk] = *reinterpret_cast<const u32x4*>(base + k * a.row_stride + n);
            }
            const bool aligned = ((K & 3) == 0) && ((a.offset & 3u) == 0);           // uniform over the grid
            auto column = [&](int j, int kk, uint32_t u24) {
                const uint32_t word = w[kk][j >> 1];
                const float xv = (j & 1) ? __uint_as_float(word & 0xFFFF0000u) : __uint_as_float(word << 16);
                const uint32_t code = encode<FMT, MODE>(xv * rho[j], u24);
                if (kk < 4) lo[j] |= code << (8 * kk); else hi[j] |= code << (8 * (kk - 4));
            };
            const uint64_t g_first = (uint64_t)((b * N + n) * K + k0 + tk * 8) + a.offset;    // column j: + j * K
            if (aligned) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint64_t c = (g_first + (uint64_t)j * (uint64_t)K) >> 2;
                    const Philox4 ba = philox4x32_10((uint32_t)c, (uint32_t)(c >> 32), 0u, 0u, (uint32_t)a.seed,
                                                     (uint32_t)(a.seed >> 32));
                    const Philox4 bb = philox4x32_10((uint32_t)(c + 1), (uint32_t)((c + 1) >> 32), 0u, 0u, (uint32_t)a.seed,
                                                     (uint32_t)(a.seed >> 32));
#pragma unroll
                    for (int kk = 0; kk < 8; ++kk) column(j, kk, (kk < 4 ? ba.v[kk] : bb.v[kk - 4]) >> 8);
                    // one column at a time: interleaved, the sixteen generator blocks of a thread need 240 registers
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
#pragma unroll
                    for (int kk = 0; kk < 8; ++kk) column(j, kk, sr.bits(g_first + (uint64_t)j * (uint64_t)K + kk));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    } else if (n < N) {
        // rows in pairs: the FP8 formats go through the two-at-a-time hardware converter (encode_fp8_rtne_pair)
#pragma unroll
        for (int kk = 0; kk < 8; kk += 2) {
            const int64_t k = k0 + tk * 8 + kk;
            u32x4 wa = {0u, 0u, 0u, 0u}, wb = {0u, 0u, 0u, 0u};
            if (k < K) wa = *reinterpret_cast<const u32x4*>(base + k * a.row_stride + n);
            if (k + 1 < K) wb = *reinterpret_cast<const u32x4*>(base + (k + 1) * a.row_stride + n);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t worda = wa[j >> 1], wordb = wb[j >> 1];
                const float ta = ((j & 1) ? __uint_as_float(worda & 0xFFFF0000u) : __uint_as_float(worda << 16)) * rho[j];
                const float tb = ((j & 1) ? __uint_as_float(wordb & 0xFFFF0000u) : __uint_as_float(wordb << 16)) * rho[j];
                uint32_t pair;
                if constexpr (FMT == QMM_FMT_INT8) pair = encode_int8_rtne(ta) | (encode_int8_rtne(tb) << 8);
                else pair = encode_fp8_rtne_pair<FMT>(ta, tb);
                if (kk < 4) lo[j] |= pair << (8 * kk); else hi[j] |= pair << (8 * (kk - 4));
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        u32x2 v = {lo[j], hi[j]};
        *reinterpret_cast<u32x2*>(&tile[(tn * 8 + j) * kTileRowBytes + tk * 8]) = v;
    }
    __syncthreads();
    // 128 code rows x 8 pieces of 16 bytes = 1024 pieces, 4 per thread
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int piece = it * kThreads + threadIdx.x;
        const int row = piece >> 3, seg = piece & 7;
        const int64_t nn = n0 + row, kk = k0 + seg * 16;
        if (nn >= N || kk >= K) continue;
        uint8_t* dst = a.codes + (b * N + nn) * K + kk;
        const uint8_t* srcp = &tile[row * kTileRowBytes + seg * 16];
        if (kk + 16 <= K && (K & 15) == 0) {
            *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<const u32x4*>(srcp);
        } else {
            for (int e = 0; e < 16 && kk + e < K; ++e) dst[e] = srcp[e];
        }
    }
}

template <int FMT, int MODE> qmm_status launch(const qmm_tensor* x, const QArgs& a, hipStream_t s)
{
    const bool bf16 = x->dtype == QMM_DT_BF16;
    const bool aligned = aligned16(x->data) && (x->row_stride % 8 == 0) && (x->batch_stride % 8 == 0);
    if (bf16 && aligned && x->contract_axis == 1 && (x->cols % 16 == 0) && aligned16(a.codes)) {
        const int64_t nv = x->rows * (x->cols / 16);
        quantize_rows_bf16x16<FMT, MODE><<<dim3((unsigned)((nv + kThreads - 1) / kThreads), (unsigned)x->batch), kThreads, 0, s>>>(a);
    } else if (bf16 && aligned && x->contract_axis == 0 && (x->cols % 8 == 0) && aligned16(a.codes)) {
        quantize_cols_bf16<FMT, MODE><<<dim3((unsigned)((x->cols + kTile - 1) / kTile), (unsigned)((x->rows + kTile - 1) / kTile),
                                              (unsigned)x->batch), kThreads, 0, s>>>(a);
    } else {
        const int64_t n = x->rows * x->cols;
        const dim3 grid((unsigned)((n + kThreads - 1) / kThreads), (unsigned)x->batch);
        if (bf16) quantize_generic<uint16_t, FMT, MODE><<<grid, kThreads, 0, s>>>(a, x->contract_axis);
        else quantize_generic<float, FMT, MODE><<<grid, kThreads, 0, s>>>(a, x->contract_axis);
    }
    return launch_status();
}

template <int FMT> qmm_status launch_mode(const qmm_tensor* x, const QArgs& a, qmm_round mode, hipStream_t s)
{
    return mode == QMM_ROUND_RTNE ? launch<FMT, QMM_ROUND_RTNE>(x, a, s) : launch<FMT, QMM_ROUND_STOCHASTIC>(x, a, s);
}

}  // namespace
}  // namespace qmm

using namespace qmm;

namespace {
// Everything qmm_quantize can refuse, checked without launching: QMM_OK means the call will enqueue (or has nothing to do).
qmm_status quantize_check(const qmm_tensor* x, qmm_format fmt, const qmm_granularity* g, const float* delta,
                          qmm_round mode, const uint8_t* codes_out)
{
    if (!x || !g) return QMM_ERR_NULL;
    if (x->dtype != QMM_DT_BF16 && x->dtype != QMM_DT_F32) return QMM_ERR_ENUM;
    if (x->contract_axis != 0 && x->contract_axis != 1) return QMM_ERR_ENUM;
    if (fmt != QMM_FMT_INT8 && fmt != QMM_FMT_E4M3 && fmt != QMM_FMT_E5M2) return QMM_ERR_ENUM;
    if (mode != QMM_ROUND_RTNE && mode != QMM_ROUND_STOCHASTIC) return QMM_ERR_ENUM;
    if (g->batch_groups < 1 || g->batch_inner < 0 || (g->per_channel != 0 && g->per_channel != 1)) return QMM_ERR_ENUM;
    if (x->batch < 0 || x->rows < 0 || x->cols < 0 || x->row_stride < x->cols) return QMM_ERR_SHAPE;
    if (x->batch > 1 && x->rows > 0 && x->batch_stride < (x->rows - 1) * x->row_stride + x->cols) return QMM_ERR_SHAPE;
    if (x->batch > 65535) return QMM_ERR_UNSUPPORTED;
    if (x->batch * x->rows * x->cols == 0) return QMM_OK;
    if (!x->data || !delta || !codes_out) return QMM_ERR_NULL;
    return QMM_OK;
}
}  // namespace

extern "C" qmm_status qmm_quantize(const qmm_tensor* x, qmm_format fmt, const qmm_granularity* g, const float* delta,
                                   qmm_round mode, uint64_t seed, uint64_t offset, uint8_t* codes_out, void* stream)
{
    const qmm_status chk = quantize_check(x, fmt, g, delta, mode, codes_out);
    if (chk != QMM_OK) return chk;
    if (x->batch * x->rows * x->cols == 0) return QMM_OK;

    QArgs a;
    a.x = x->data; a.delta = delta; a.codes = codes_out;
    a.batch = x->batch; a.rows = x->rows; a.cols = x->cols;
    a.batch_stride = x->batch_stride; a.row_stride = x->row_stride;
    a.groups = g->batch_groups;
    a.inner = g->batch_inner > 0 ? g->batch_inner : 1;
    a.channels = g->per_channel ? (x->contract_axis == 1 ? x->rows : x->cols) : 1;
    a.seed = seed; a.offset = offset;
    hipStream_t s = as_stream(stream);
    switch (fmt) {
    case QMM_FMT_INT8: return launch_mode<QMM_FMT_INT8>(x, a, mode, s);
    case QMM_FMT_E4M3: return launch_mode<QMM_FMT_E4M3>(x, a, mode, s);
    default: return launch_mode<QMM_FMT_E5M2>(x, a, mode, s);
    }
}

extern "C" qmm_status qmm_quantize_multi(int32_t count, const qmm_tensor* x, qmm_format fmt, const qmm_granularity* g,
                                         const float* const* delta, qmm_round mode, uint64_t seed, const uint64_t* offsets,
                                         uint8_t* const* codes_out, void* stream)
{
    if (count < 0) return QMM_ERR_SHAPE;
    if (count == 0) return QMM_OK;
    if (!x || !g || !delta || !codes_out) return QMM_ERR_NULL;
    if (fmt != QMM_FMT_INT8 && fmt != QMM_FMT_E4M3 && fmt != QMM_FMT_E5M2) return QMM_ERR_ENUM;
    if (mode != QMM_ROUND_RTNE && mode != QMM_ROUND_STOCHASTIC) return QMM_ERR_ENUM;
    bool one_launch = count <= kMaxMulti && mode == QMM_ROUND_RTNE;
    for (int32_t t = 0; t < count && one_launch; ++t) {
        const qmm_tensor& q = x[t];
        one_launch = q.data && delta[t] && codes_out[t] && q.dtype == QMM_DT_BF16 && q.contract_axis == 1 && q.batch == 1 &&
                     !g[t].per_channel && g[t].batch_groups == 1 && g[t].batch_inner >= 0 && q.rows >= 1 && q.cols >= 16 &&
                     q.cols % 16 == 0 && q.row_stride == q.cols && aligned16(q.data) && aligned16(codes_out[t]);
    }
    if (!one_launch) {
        for (int32_t t = 0; t < count; ++t) {      // every tensor's arguments before the first launch
            const qmm_status st = quantize_check(x + t, fmt, g + t, delta[t], mode, codes_out[t]);
            if (st != QMM_OK) return st;
        }
        for (int32_t t = 0; t < count; ++t) {
            const qmm_status st = qmm_quantize(x + t, fmt, g + t, delta[t], mode, seed, offsets ? offsets[t] : 0, codes_out[t], stream);
            if (st != QMM_OK) return st;
        }
        return QMM_OK;
    }
    MultiQ a{};
    int64_t max_vec = 1;
    for (int32_t t = 0; t < count; ++t) {
        a.x[t] = static_cast<const uint16_t*>(x[t].data);
        a.codes[t] = codes_out[t];
        a.delta[t] = delta[t];
        a.nvec16[t] = x[t].rows * x[t].cols / 16;
        max_vec = std::max(max_vec, a.nvec16[t]);
    }
    const int64_t blocks = (max_vec + kThreads - 1) / kThreads;
    if (blocks > 0x7FFFFFFF) return QMM_ERR_UNSUPPORTED;
    hipStream_t s = as_stream(stream);
    const dim3 grid((unsigned)blocks, (unsigned)count);
    if (fmt == QMM_FMT_INT8) quantize_flat_multi<QMM_FMT_INT8><<<grid, kThreads, 0, s>>>(a);
    else if (fmt == QMM_FMT_E4M3) quantize_flat_multi<QMM_FMT_E4M3><<<grid, kThreads, 0, s>>>(a);
    else quantize_flat_multi<QMM_FMT_E5M2><<<grid, kThreads, 0, s>>>(a);
    return launch_status();
}
