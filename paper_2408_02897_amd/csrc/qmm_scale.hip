// qmm_scale: step size delta = max|X| / qmax per scale group (Eq. 1, right half;
// Methodology bullets on scale granularity and on aligning the absmax with the
// format maximum).  HBM-bound: every element is read once (2 B for bfloat16),
// the maximum is taken on magnitude bit patterns (exact, order-free), partial
// maxima go to the workspace and are folded per group, followed by the one
// division: by a second small kernel, or -- dense tensors with one step size,
// from 32 MB, and the several-tensors call -- by the workgroup that finishes
// last (one launch).  The maximum is order-free, so the result does not depend
// on launch geometry or on which workgroup folds.
#include <algorithm>
#include <atomic>
#include "qmm_device.h"

namespace qmm {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxFlatBlocks = 1024;   // 4 workgroups per CU on 256 CUs; 4 partials per thread in the fold
constexpr int kColSlabRows = 128;      // rows folded by one workgroup in the column-group kernel

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

QMM_DEV uint32_t block_max_u32(uint32_t v)
{
    __shared__ uint32_t s[kThreads / kWave];
    v = wave_max_u32(v);
    if ((threadIdx.x & (kWave - 1)) == 0) s[threadIdx.x / kWave] = v;
    __syncthreads();
    uint32_t r = s[0];
#pragma unroll
    for (int i = 1; i < kThreads / kWave; ++i) r = max(r, s[i]);
    return r;
}

// 8 bfloat16 magnitudes packed in a 16-byte vector -> running packed maxima.
QMM_DEV void fold_bf16x8(u32x4 w, u16x2 (&m)[4])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t a = w[i] & 0x7FFF7FFFu;
        m[i] = __builtin_elementwise_max(m[i], __builtin_bit_cast(u16x2, a));
    }
}
QMM_DEV uint32_t finish_bf16(const u16x2 (&m)[4])
{
    uint32_t r = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) r = max(r, max((uint32_t)m[i][0], (uint32_t)m[i][1]));
    return r << 16;   // bfloat16 magnitude -> binary32 magnitude bits
}

// The fold of a tensor's partial maxima by the workgroup that arrived last: all of them are one scale group.
QMM_DEV void fold_all_partials(const uint32_t* partial, int64_t count, float qmax, float* delta)
{
    uint32_t v[4] = {0u, 0u, 0u, 0u}, m = 0;
    int64_t i = threadIdx.x;
    for (; i + 3 * kThreads < count; i += 4 * kThreads) {         // four requests in flight
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = coherent_load(partial + i + k * kThreads);
        m = max(max(m, max(v[0], v[1])), max(v[2], v[3]));
    }
    for (; i < count; i += kThreads) m = max(m, coherent_load(partial + i));
    m = block_max_u32(m);
    if (threadIdx.x == 0) delta[0] = delta_from_absmax_bits(m, qmax);
}

// Dense matrix (row_stride == cols), bfloat16, 16-byte vectors: grid (nblk, batch).  With `slot` (one scale group
// for the whole batch) the workgroup that arrives last folds the partial maxima and writes the step size.
__global__ void __launch_bounds__(kThreads)
absmax_flat_bf16(const uint16_t* __restrict__ x, int64_t batch_stride, int64_t nvec, uint32_t* __restrict__ partial,
                 uint32_t* __restrict__ slot, float qmax, float* __restrict__ delta)
{
    const u32x4* p = reinterpret_cast<const u32x4*>(x + (int64_t)blockIdx.y * batch_stride);
    u16x2 m[4] = {};
    // A workgroup takes four consecutive 4 KB pieces per trip and the grid sweeps the tensor front to back: the
    // four loads a thread has in flight are then neighbours in memory.  (With the loads a whole grid stride apart
    // the same kernel reads a large tensor up to 25 % slower: four distant streams per thread.)  Ordinary loads on
    // purpose: streaming loads make this pass 7 % faster on a 134 MB tensor (23.0 against 24.6 us), but the quantize
    // pass that follows then finds less of the tensor in the memory-side cache and loses twice that.
    const int64_t stride = (int64_t)gridDim.x * kThreads * 4;
    int64_t i = (int64_t)blockIdx.x * kThreads * 4 + threadIdx.x;
    for (; i + 3 * kThreads < nvec; i += stride) {
        const u32x4 a = p[i], b = p[i + kThreads];
        const u32x4 c = p[i + 2 * kThreads], d = p[i + 3 * kThreads];
        fold_bf16x8(a, m); fold_bf16x8(b, m); fold_bf16x8(c, m); fold_bf16x8(d, m);
    }
    // the ragged end: at most three pieces of one workgroup
    if (i < nvec) {
        for (int u = 0; u < 4; ++u)
            if (i + u * kThreads < nvec) fold_bf16x8(p[i + u * kThreads], m);
    }
    const uint32_t r = block_max_u32(finish_bf16(m));
    const unsigned id = blockIdx.y * gridDim.x + blockIdx.x, total = gridDim.x * gridDim.y;
    if (threadIdx.x == 0) {
        if (slot) publish_u32(partial + id, r); else partial[id] = r;
    }
    if (slot && arrive_last(slot, id, total)) {
        __syncthreads();                         // block_max_u32's shared words are reused by the fold
        fold_all_partials(partial, total, qmax, delta);
    }
}

// Several dense bfloat16 tensors, one step size each, in one launch (qmm_scale_multi): blockIdx.y picks the tensor,
// workgroups past a tensor's own count leave at once.  The 2-8 MB weight matrices of a layer are latency-bound on
// their own; launched beside the activations they cost next to nothing.
constexpr int kMaxMulti = 8;
struct MultiFlat {
    const uint16_t* x[kMaxMulti];
    int64_t nvec[kMaxMulti];        // 16-byte vectors
    uint32_t* partial[kMaxMulti];
    float* delta[kMaxMulti];
    int nblk[kMaxMulti];
    uint32_t* slots;                // kMaxMulti consecutive slots of arrival counters, one per tensor
    float qmax;
};
__global__ void __launch_bounds__(kThreads)
absmax_flat_multi(MultiFlat a)
{
    const int t = blockIdx.y;
    const int nblk = a.nblk[t];
    if ((int)blockIdx.x >= nblk) return;
    const u32x4* p = reinterpret_cast<const u32x4*>(a.x[t]);
    const int64_t nvec = a.nvec[t];
    u16x2 m[4] = {};
    const int64_t stride = (int64_t)nblk * kThreads * 4;
    int64_t i = (int64_t)blockIdx.x * kThreads * 4 + threadIdx.x;
    for (; i + 3 * kThreads < nvec; i += stride) {
        const u32x4 v0 = p[i], v1 = p[i + kThreads];
        const u32x4 v2 = p[i + 2 * kThreads], v3 = p[i + 3 * kThreads];
        fold_bf16x8(v0, m); fold_bf16x8(v1, m); fold_bf16x8(v2, m); fold_bf16x8(v3, m);
    }
    if (i < nvec) {
        for (int u = 0; u < 4; ++u)
            if (i + u * kThreads < nvec) fold_bf16x8(p[i + u * kThreads], m);
    }
    const uint32_t r = block_max_u32(finish_bf16(m));
    if (threadIdx.x == 0) publish_u32(a.partial[t] + blockIdx.x, r);
    // the tensor's last workgroup folds its partial maxima (at most kMaxFlatBlocks) and writes its step size
    if (arrive_last(a.slots + (size_t)t * kArrivalWords, blockIdx.x, (unsigned)nblk)) {
        __syncthreads();
        fold_all_partials(a.partial[t], nblk, a.qmax, a.delta[t]);
    }
}

template <typename T> QMM_DEV uint32_t mag_bits(T v);
template <> QMM_DEV uint32_t mag_bits<uint16_t>(uint16_t v) { return ((uint32_t)v & 0x7FFFu) << 16; }
template <> QMM_DEV uint32_t mag_bits<float>(float v) { return __float_as_uint(v) & 0x7FFFFFFFu; }

// One wavefront per (matrix, row): partial[b*rows + r] = absmax of the row.  Any stride, any dtype.
template <typename T> __global__ void __launch_bounds__(kThreads)
absmax_rows(const T* __restrict__ x, int64_t batch_stride, int64_t row_stride, int64_t rows, int64_t cols,
            int64_t total_rows, uint32_t* __restrict__ partial, float qmax, float* __restrict__ delta)
{
    const int64_t wr = (int64_t)blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
    if (wr >= total_rows) return;
    const int64_t b = wr / rows, r = wr % rows;
    const T* p = x + b * batch_stride + r * row_stride;
    const int lane = threadIdx.x & (kWave - 1);
    uint32_t m = 0;
    if constexpr (sizeof(T) == 2) {
        if ((cols & 7) == 0 && (reinterpret_cast<uintptr_t>(p) & 15u) == 0) {
            const u32x4* pv = reinterpret_cast<const u32x4*>(p);
            u16x2 mm[4] = {};
            for (int64_t i = lane; i < cols / 8; i += kWave) fold_bf16x8(pv[i], mm);
            m = finish_bf16(mm);
        } else {
            for (int64_t i = lane; i < cols; i += kWave) m = max(m, mag_bits<T>(p[i]));
        }
    } else {
        for (int64_t i = lane; i < cols; i += kWave) m = max(m, mag_bits<T>(p[i]));
    }
    m = wave_max_u32(m);
    // delta != NULL: every row is a scale group of its own (one step size per row, one matrix per batch group), so
    // the row's maximum is final and the step size is written here, without the second kernel
    if (lane == 0) { if (delta) delta[wr] = delta_from_absmax_bits(m, qmax); else partial[wr] = m; }
}

// Short rows (at most 256 bfloat16 columns, 16-byte aligned rows): LPR lanes per row, one 16-byte vector each, so a
// wavefront takes 64 / LPR rows at once instead of one (with the rows dense in memory it reads 1 KB contiguous).
template <int LPR> __global__ void __launch_bounds__(kThreads)
absmax_rows_short(const uint16_t* __restrict__ x, int64_t batch_stride, int64_t row_stride, int64_t rows, int64_t cols,
                  int64_t total_rows, uint32_t* __restrict__ partial, float qmax, float* __restrict__ delta)
{
    constexpr int RPW = kWave / LPR;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t w = (int64_t)blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
    const int64_t row = w * RPW + lane / LPR;
    const int v = lane % LPR;
    uint32_t m = 0;
    if (row < total_rows && v < cols / 8) {
        const int64_t b = row / rows, r = row - b * rows;
        u16x2 mm[4] = {};
        fold_bf16x8(*reinterpret_cast<const u32x4*>(x + b * batch_stride + r * row_stride + v * 8), mm);
        m = finish_bf16(mm);
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off, kWave));
    if (v == 0 && row < total_rows) { if (delta) delta[row] = delta_from_absmax_bits(m, qmax); else partial[row] = m; }
}

// Column groups: workgroup = 32 column-vectors (256 columns) x 8 row lanes over a slab of rows.
// partial[(b*nslab + slab)*cols + c].  bfloat16, cols % 8 == 0, 16-byte aligned rows.
__global__ void __launch_bounds__(kThreads)
absmax_cols_bf16(const uint16_t* __restrict__ x, int64_t batch_stride, int64_t row_stride, int64_t rows, int64_t cols,
                 uint32_t* __restrict__ partial)
{
    __shared__ uint32_t s[8][32][4];
    const int cv = threadIdx.x & 31, rl = threadIdx.x >> 5;
    const int64_t vcol = (int64_t)blockIdx.x * 32 + cv;
    const int64_t r0 = (int64_t)blockIdx.y * kColSlabRows;
    const int64_t r1 = min(rows, r0 + (int64_t)kColSlabRows);
    u16x2 m[4] = {};
    if (vcol * 8 < cols) {
        const uint16_t* base = x + (int64_t)blockIdx.z * batch_stride + vcol * 8;
        int64_t r = r0 + rl;
        // four rows per trip: the loads are in flight together
        for (; r + 24 < r1; r += 32) {
            const u32x4 a = *reinterpret_cast<const u32x4*>(base + r * row_stride);
            const u32x4 b = *reinterpret_cast<const u32x4*>(base + (r + 8) * row_stride);
            const u32x4 c = *reinterpret_cast<const u32x4*>(base + (r + 16) * row_stride);
            const u32x4 d = *reinterpret_cast<const u32x4*>(base + (r + 24) * row_stride);
            fold_bf16x8(a, m); fold_bf16x8(b, m); fold_bf16x8(c, m); fold_bf16x8(d, m);
        }
        for (; r < r1; r += 8)
            fold_bf16x8(*reinterpret_cast<const u32x4*>(base + r * row_stride), m);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) s[rl][cv][i] = __builtin_bit_cast(uint32_t, m[i]);
    __syncthreads();
    if (rl == 0 && vcol * 8 < cols) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            u16x2 a = m[i];
            for (int k = 1; k < 8; ++k) a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, s[k][cv][i]));
            uint32_t* out = partial + ((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * cols + vcol * 8 + 2 * i;
            out[0] = (uint32_t)a[0] << 16;
            out[1] = (uint32_t)a[1] << 16;
        }
    }
}

// Generic column groups (any dtype / alignment): one thread per column over a slab of rows.
template <typename T> __global__ void __launch_bounds__(kThreads)
absmax_cols_generic(const T* __restrict__ x, int64_t batch_stride, int64_t row_stride, int64_t rows, int64_t cols,
                    uint32_t* __restrict__ partial)
{
    const int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (c >= cols) return;
    const int64_t r0 = (int64_t)blockIdx.y * kColSlabRows;
    const int64_t r1 = min(rows, r0 + (int64_t)kColSlabRows);
    const T* base = x + (int64_t)blockIdx.z * batch_stride + c;
    uint32_t m = 0;
    for (int64_t r = r0; r < r1; ++r) m = max(m, mag_bits<T>(base[r * row_stride]));
    partial[((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * cols + c] = m;
}

// Fold partial[b][P][C] over the matrices b of group g, (b / inner) % G == g, and over p; then delta = absmax / qmax.
// The matrices of a group: b = q * inner + i for q = g, g + G, ... and i = 0 .. inner - 1.
// C == 1: one workgroup per group.  C > 1: one thread per (g, c).
__global__ void __launch_bounds__(kThreads)
finalize_single(const uint32_t* __restrict__ partial, int64_t batch, int64_t P, int64_t G, int64_t inner, float qmax,
                float* __restrict__ delta)
{
    const int64_t g = blockIdx.x;
    uint32_t m = 0;
    if (inner == 1 && batch <= G && P <= 4 * kThreads) {
        // one matrix per group and few partials: request them all before folding
        uint32_t v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int64_t p = threadIdx.x + k * kThreads;
            v[k] = (g < batch && p < P) ? partial[g * P + p] : 0u;
        }
        m = max(max(v[0], v[1]), max(v[2], v[3]));
    } else {
        // the (matrix, partial) pairs of the group, spread over the threads: the k-th matrix of group g is
        // b = ((k / inner) * G + g) * inner + k % inner, increasing with k
        for (int64_t it = threadIdx.x;; it += kThreads) {
            const int64_t k = it / P, p = it - k * P;
            const int64_t b = ((k / inner) * G + g) * inner + k % inner;
            if (b >= batch) break;
            m = max(m, partial[b * P + p]);
        }
    }
    m = block_max_u32(m);
    if (threadIdx.x == 0) delta[g] = delta_from_absmax_bits(m, qmax);
}
// Workgroup = 32 channels x 8 lanes over the (matrix, partial) pairs of the group; max is order-free.
__global__ void __launch_bounds__(kThreads)
finalize_channels(const uint32_t* __restrict__ partial, int64_t batch, int64_t P, int64_t C, int64_t G, int64_t inner,
                  float qmax, float* __restrict__ delta)
{
    __shared__ uint32_t s[8][32];
    const int cl = threadIdx.x & 31, pl = threadIdx.x >> 5;
    const int64_t c = (int64_t)blockIdx.x * 32 + cl;
    const int64_t g = blockIdx.y;
    uint32_t m = 0;
    if (c < C) {
        // the (matrix, partial) pairs of the group over the eight lanes of a channel (k-th matrix of group g:
        // b = ((k / inner) * G + g) * inner + k % inner, increasing with k), four loads in flight
        auto item = [&](int64_t it) -> uint32_t {
            const int64_t k = it / P, p = it - k * P;
            const int64_t b = ((k / inner) * G + g) * inner + k % inner;
            return b < batch ? partial[(b * P + p) * C + c] : 0u;
        };
        const int64_t groups_of_inner = (batch + inner - 1) / inner;                     // q = 0 .. groups_of_inner - 1
        const int64_t nq = groups_of_inner > g ? (groups_of_inner - g + G - 1) / G : 0;  // those with q % G == g
        const int64_t nitems = nq * inner * P;                                           // (items past the batch read as 0)
        int64_t it = pl;
        for (; it + 24 < nitems; it += 32) {
            const uint32_t v0 = item(it), v1 = item(it + 8), v2 = item(it + 16), v3 = item(it + 24);
            m = max(m, max(max(v0, v1), max(v2, v3)));
        }
        for (; it < nitems; it += 8) m = max(m, item(it));
    }
    s[pl][cl] = m;
    __syncthreads();
    if (pl == 0 && c < C) {
#pragma unroll
        for (int k = 1; k < 8; ++k) m = max(m, s[k][cl]);
        delta[g * C + c] = delta_from_absmax_bits(m, qmax);
    }
}

struct Plan {
    enum Kind { FLAT, ROWS, COLS_VEC, COLS_GENERIC } kind;
    int64_t P;        // partials per matrix (per channel for the column kinds)
    int64_t C;        // channels
    int flat_blocks;
    bool vec;         // bfloat16 with 16-byte aligned rows of whole 8-element vectors
};

bool valid_tensor(const qmm_tensor* x, qmm_status* st)
{
    if (!x) { *st = QMM_ERR_NULL; return false; }
    if (x->dtype != QMM_DT_BF16 && x->dtype != QMM_DT_F32) { *st = QMM_ERR_ENUM; return false; }
    if (x->contract_axis != 0 && x->contract_axis != 1) { *st = QMM_ERR_ENUM; return false; }
    if (x->batch < 0 || x->rows < 0 || x->cols < 0) { *st = QMM_ERR_SHAPE; return false; }
    if (x->row_stride < x->cols) { *st = QMM_ERR_SHAPE; return false; }
    if (x->batch > 1 && x->rows > 0 && x->batch_stride < (x->rows - 1) * x->row_stride + x->cols) {
        *st = QMM_ERR_SHAPE; return false;
    }
    return true;
}

Plan make_plan(const qmm_tensor* x, const qmm_granularity* g)
{
    Plan p{};
    const bool bf16 = x->dtype == QMM_DT_BF16;
    const bool vec_ok = bf16 && aligned16(x->data) && (x->cols % 8 == 0) && (x->row_stride % 8 == 0) &&
                        (x->batch_stride % 8 == 0);
    p.vec = vec_ok;
    if (!g->per_channel) {
        p.C = 1;
        const int64_t n = x->rows * x->cols;
        if (vec_ok && x->row_stride == x->cols && n > 0) {
            p.kind = Plan::FLAT;
            const int64_t nvec = n / 8;
            int64_t nb = (nvec + (int64_t)kThreads * 4 - 1) / ((int64_t)kThreads * 4);
            const int64_t cap = x->batch > 1 ? (kMaxFlatBlocks + x->batch - 1) / x->batch : kMaxFlatBlocks;
            nb = nb < 1 ? 1 : (nb > cap ? cap : nb);
            p.flat_blocks = (int)nb;
            p.P = nb;
        } else {
            p.kind = Plan::ROWS;
            p.P = x->rows;
        }
    } else if (x->contract_axis == 1) {
        p.kind = Plan::ROWS;
        p.P = 1;
        p.C = x->rows;
    } else {
        p.kind = vec_ok ? Plan::COLS_VEC : Plan::COLS_GENERIC;
        p.P = (x->rows + kColSlabRows - 1) / kColSlabRows;
        p.C = x->cols;
    }
    return p;
}

}  // namespace
}  // namespace qmm

using namespace qmm;

extern "C" int64_t qmm_num_scales(const qmm_tensor* x, const qmm_granularity* g)
{
    if (!x || !g) return 0;
    const int64_t c = g->per_channel ? (x->contract_axis == 1 ? x->rows : x->cols) : 1;
    return g->batch_groups * c;
}

extern "C" size_t qmm_scale_workspace_size(const qmm_tensor* x, const qmm_granularity* g)
{
    qmm_status st;
    if (!g || !valid_tensor(x, &st)) return 0;
    const Plan p = make_plan(x, g);
    const int64_t words = x->batch * p.P * p.C;
    return (size_t)(words > 0 ? words : 1) * sizeof(uint32_t);
}

namespace {
// Everything qmm_scale can refuse, checked without launching.
qmm_status scale_check(const qmm_tensor* x, qmm_format fmt, const qmm_granularity* g, const float* delta_out,
                       const void* workspace, size_t workspace_bytes)
{
    qmm_status st;
    if (!g || !delta_out) return QMM_ERR_NULL;
    if (!valid_tensor(x, &st)) return st;
    if (fmt != QMM_FMT_INT8 && fmt != QMM_FMT_E4M3 && fmt != QMM_FMT_E5M2) return QMM_ERR_ENUM;
    if (g->batch_groups < 1 || g->batch_inner < 0 || (g->per_channel != 0 && g->per_channel != 1)) return QMM_ERR_ENUM;
    if (x->batch > 65535) return QMM_ERR_UNSUPPORTED;          // the batch index is a grid dimension in some plans
    if (qmm_num_scales(x, g) == 0) return QMM_OK;
    if (x->batch * x->rows * x->cols > 0 && !x->data) return QMM_ERR_NULL;
    if (!workspace || workspace_bytes < qmm_scale_workspace_size(x, g)) return QMM_ERR_WORKSPACE;
    if (!aligned16(workspace)) return QMM_ERR_ALIGN;
    return QMM_OK;
}
}  // namespace

extern "C" qmm_status qmm_scale(const qmm_tensor* x, qmm_format fmt, const qmm_granularity* g, float* delta_out,
                                void* workspace, size_t workspace_bytes, void* stream)
{
    const qmm_status chk = scale_check(x, fmt, g, delta_out, workspace, workspace_bytes);
    if (chk != QMM_OK) return chk;
    if (qmm_num_scales(x, g) == 0) return QMM_OK;

    hipStream_t s = as_stream(stream);
    uint32_t* partial = static_cast<uint32_t*>(workspace);
    const Plan p = make_plan(x, g);
    const float qmax = fmt == QMM_FMT_INT8 ? 127.0f : (fmt == QMM_FMT_E4M3 ? 448.0f : 57344.0f);
    const bool bf16 = x->dtype == QMM_DT_BF16;
    const int64_t nelem = x->batch * x->rows * x->cols;
    const int64_t C = p.C;
    int64_t P = p.P;

    // one step size per row with every matrix a batch group of its own: a row's maximum is its group's maximum
    const bool rows_are_groups = nelem > 0 && p.kind == Plan::ROWS && g->per_channel && x->contract_axis == 1 && p.P == 1 &&
                                 x->batch == g->batch_groups && g->batch_inner <= 1;
    if (nelem > 0) {
        switch (p.kind) {
        case Plan::FLAT: {
            // One scale group for the whole batch and a large tensor: one launch, the workgroup that arrives last folds.
            // (Publishing, counting and the coherent reads of the fold are a chain of device-wide round trips of
            // 2-3 us each: about 11 us for a tensor of any size up to 32 MB, against 9-10 us for two small launches;
            // from 32 MB on the single launch wins, 25 us against 27 us at 134 MB.)
            uint32_t* slot = nullptr;
            if (g->batch_groups == 1 && nelem >= (int64_t(1) << 24) && arrival_slots(1, &slot) != QMM_OK) slot = nullptr;
            absmax_flat_bf16<<<dim3(p.flat_blocks, (unsigned)x->batch), kThreads, 0, s>>>(
                static_cast<const uint16_t*>(x->data), x->batch_stride, x->rows * x->cols / 8, partial, slot, qmax, delta_out);
            if (slot) return launch_status();
            break;
        }
        case Plan::ROWS: {
            const int64_t total = x->batch * x->rows;
            float* direct = rows_are_groups ? delta_out : nullptr;
            const unsigned nb = (unsigned)((total + kThreads / kWave - 1) / (kThreads / kWave));
            if (p.vec && x->cols <= 256) {
                const uint16_t* xp = static_cast<const uint16_t*>(x->data);
                const int nvec = (int)(x->cols / 8);
                const int lpr = nvec <= 1 ? 1 : nvec <= 2 ? 2 : nvec <= 4 ? 4 : nvec <= 8 ? 8 : nvec <= 16 ? 16 : 32;
                const int64_t waves = (total + kWave / lpr - 1) / (kWave / lpr);
                const unsigned nbs = (unsigned)((waves + kThreads / kWave - 1) / (kThreads / kWave));
#define QMM_ROWS_SHORT(L) absmax_rows_short<L><<<nbs, kThreads, 0, s>>>(xp, x->batch_stride, x->row_stride, x->rows, x->cols, total, partial, qmax, direct)
                if (lpr == 1) QMM_ROWS_SHORT(1); else if (lpr == 2) QMM_ROWS_SHORT(2); else if (lpr == 4) QMM_ROWS_SHORT(4);
                else if (lpr == 8) QMM_ROWS_SHORT(8); else if (lpr == 16) QMM_ROWS_SHORT(16); else QMM_ROWS_SHORT(32);
#undef QMM_ROWS_SHORT
            } else if (bf16)
                absmax_rows<uint16_t><<<nb, kThreads, 0, s>>>(static_cast<const uint16_t*>(x->data), x->batch_stride,
                                                               x->row_stride, x->rows, x->cols, total, partial, qmax, direct);
            else
                absmax_rows<float><<<nb, kThreads, 0, s>>>(static_cast<const float*>(x->data), x->batch_stride,
                                                            x->row_stride, x->rows, x->cols, total, partial, qmax, direct);
            break;
        }
        case Plan::COLS_VEC:
            absmax_cols_bf16<<<dim3((unsigned)((x->cols / 8 + 31) / 32), (unsigned)P, (unsigned)x->batch), kThreads, 0, s>>>(
                static_cast<const uint16_t*>(x->data), x->batch_stride, x->row_stride, x->rows, x->cols, partial);
            break;
        case Plan::COLS_GENERIC: {
            const dim3 grid((unsigned)((x->cols + kThreads - 1) / kThreads), (unsigned)P, (unsigned)x->batch);
            if (bf16)
                absmax_cols_generic<uint16_t><<<grid, kThreads, 0, s>>>(static_cast<const uint16_t*>(x->data),
                                                                        x->batch_stride, x->row_stride, x->rows, x->cols, partial);
            else
                absmax_cols_generic<float><<<grid, kThreads, 0, s>>>(static_cast<const float*>(x->data), x->batch_stride,
                                                                     x->row_stride, x->rows, x->cols, partial);
            break;
        }
        }
        if (hipGetLastError() != hipSuccess) return QMM_ERR_LAUNCH;
        if (rows_are_groups) return launch_status();
    }
    // An empty tensor has no partials: fold over zero matrices so every group gets delta = 1.
    const int64_t fold_batch = nelem > 0 ? x->batch : 0;
    if (nelem == 0) P = 0;
    const int64_t G = g->batch_groups, inner = g->batch_inner > 0 ? g->batch_inner : 1;
    if (C == 1)
        finalize_single<<<(unsigned)G, kThreads, 0, s>>>(partial, fold_batch, P, G, inner, qmax, delta_out);
    else
        finalize_channels<<<dim3((unsigned)((C + 31) / 32), (unsigned)G), kThreads, 0, s>>>(
            partial, fold_batch, P, C, G, inner, qmax, delta_out);
    return launch_status();
}

// ---- qmm_scale_static: the same kernels with their partial maxima in a scratch array of the device image.
// `scratch` below is the host-side stand-in of the device array; its device address differs per GPU and is looked
// up once per device (kept in scratch_addr), and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[QMM_SCALE_STATIC_BYTES];
namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> scratch_addr[kMaxDevices];

qmm_status static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return QMM_ERR_LAUNCH;
    if (dev < 0 || dev >= kMaxDevices) return QMM_ERR_UNSUPPORTED;
    void* p = scratch_addr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return QMM_ERR_LAUNCH;
        scratch_addr[dev].store(p, std::memory_order_release);      // two first callers store the same address
    }
    *out = p;
    return QMM_OK;
}
}  // namespace

extern "C" qmm_status qmm_scale_static(const qmm_tensor* x, qmm_format fmt, const qmm_granularity* g, float* delta_out,
                                       void* stream)
{
    // argument errors first, exactly as qmm_scale reports them (the workspace checks cannot fail with a dummy of full size)
    const qmm_status chk = scale_check(x, fmt, g, delta_out, reinterpret_cast<const void*>(uintptr_t(256)), ~size_t(0));
    if (chk != QMM_OK) return chk;
    if (qmm_scale_workspace_size(x, g) > QMM_SCALE_STATIC_BYTES) return QMM_ERR_LIMIT;
    void* ws = nullptr;
    const qmm_status st = static_scratch(&ws);
    if (st != QMM_OK) return st;
    return qmm_scale(x, fmt, g, delta_out, ws, QMM_SCALE_STATIC_BYTES, stream);
}

namespace {
size_t multi_slice(const qmm_tensor* x, const qmm_granularity* g)
{
    return (qmm_scale_workspace_size(x, g) + 15u) & ~(size_t)15u;
}
// the tensors absmax_flat_multi takes: one matrix, dense, bfloat16 in whole 16-byte vectors, one step size
bool multi_flat_ok(const qmm_tensor* x, const qmm_granularity* g)
{
    qmm_status st;
    if (!valid_tensor(x, &st) || !x->data) return false;
    return x->dtype == QMM_DT_BF16 && x->batch == 1 && !g->per_channel && g->batch_groups == 1 && g->batch_inner >= 0 &&
           x->row_stride == x->cols && x->rows * x->cols >= 8 && (x->cols % 8 == 0) && aligned16(x->data) &&
           make_plan(x, g).kind == Plan::FLAT;
}
}  // namespace

extern "C" size_t qmm_scale_multi_workspace_size(int32_t count, const qmm_tensor* x, const qmm_granularity* g)
{
    if (count <= 0 || !x || !g) return 0;
    size_t total = 0;
    for (int32_t t = 0; t < count; ++t) total += multi_slice(x + t, g + t);
    return total;
}

extern "C" qmm_status qmm_scale_multi(int32_t count, const qmm_tensor* x, qmm_format fmt, const qmm_granularity* g,
                                      float* const* delta_out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (count < 0) return QMM_ERR_SHAPE;
    if (count == 0) return QMM_OK;
    if (!x || !g || !delta_out) return QMM_ERR_NULL;
    if (fmt != QMM_FMT_INT8 && fmt != QMM_FMT_E4M3 && fmt != QMM_FMT_E5M2) return QMM_ERR_ENUM;
    if (!workspace || workspace_bytes < qmm_scale_multi_workspace_size(count, x, g)) return QMM_ERR_WORKSPACE;
    if (!aligned16(workspace)) return QMM_ERR_ALIGN;
    bool one_launch = count <= kMaxMulti;
    for (int32_t t = 0; t < count && one_launch; ++t) one_launch = delta_out[t] && multi_flat_ok(x + t, g + t);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    if (!one_launch) {
        uint8_t* probe = ws;
        for (int32_t t = 0; t < count; ++t) {      // every tensor's arguments before the first launch
            const size_t slice = multi_slice(x + t, g + t);
            const qmm_status st = scale_check(x + t, fmt, g + t, delta_out[t], probe, slice);
            if (st != QMM_OK) return st;
            probe += slice;
        }
        for (int32_t t = 0; t < count; ++t) {
            const size_t slice = multi_slice(x + t, g + t);
            const qmm_status st = qmm_scale(x + t, fmt, g + t, delta_out[t], ws, slice, stream);
            if (st != QMM_OK) return st;
            ws += slice;
        }
        return QMM_OK;
    }
    MultiFlat a{};
    int max_blk = 1;
    for (int32_t t = 0; t < count; ++t) {
        const Plan p = make_plan(x + t, g + t);          // FLAT for these tensors: the same workgroup count as qmm_scale
        a.x[t] = static_cast<const uint16_t*>(x[t].data);
        a.nvec[t] = x[t].rows * x[t].cols / 8;
        a.partial[t] = reinterpret_cast<uint32_t*>(ws);
        a.delta[t] = delta_out[t];
        a.nblk[t] = p.flat_blocks;
        max_blk = std::max(max_blk, p.flat_blocks);
        ws += multi_slice(x + t, g + t);
    }
    a.qmax = fmt == QMM_FMT_INT8 ? 127.0f : (fmt == QMM_FMT_E4M3 ? 448.0f : 57344.0f);
    const qmm_status sl = arrival_slots(count, &a.slots);
    if (sl != QMM_OK) return sl;
    hipStream_t s = as_stream(stream);
    absmax_flat_multi<<<dim3((unsigned)max_blk, (unsigned)count), kThreads, 0, s>>>(a);
    return launch_status();
}
