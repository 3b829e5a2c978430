// Kernels on a stored sparsity pattern (Sec. 4.2: the pattern of the sparse term is kept for S
// iterations and only its values are recomputed) and for the sparse term H_Omega itself
// (Sec. 3.1, eq. (7)):
//
//   H_Omega = (1/eta) [ diag(T 1_m)          T^Omega_{-m}        ]     x = (x_alpha[n], x_beta[m-1])
//                     [ (T^Omega_{-m})^T     diag(T_{-m}^T 1_n)  ]
//
// The pattern is the CSR the sparsify calls produce (all m columns, ascending inside a row);
// "-m" drops the last column, so its entries are skipped here.  All of this is O(nnz) work on
// data that is a few MB: one wave per row (or column), lanes over the entries, sums in a fixed
// order (bit-reproducible), no floating-point atomics -- the product with the transposed block
// reads the pattern by columns, which regot_pattern_transpose prepares once per pattern.
#pragma once

#include "regot_device.hpp"

namespace regot {

constexpr int kRowsPerScanBlock = 32;  // rows per block in the prefix count of dropped entries (a power of two <= 64)
static_assert(kThreads % kRowsPerScanBlock == 0 && kRowsPerScanBlock <= kLanes, "row blocks");

struct PatternArgs {
    int n, m;
    int64_t ldM;
    const double *M;
    const double *alpha;
    const double *beta;
    const int64_t *row_ptr;
    const int32_t *col_idx;
    const int64_t *csc_pos;  // optional
    int64_t capacity;        // length of col_idx / val: no entry beyond it is touched
    double *val;
    double *val_csc;         // optional
    ExpParams ex;
};

// entries [p0, p1) of row i, clamped to the arrays
__device__ __forceinline__ void row_range(const int64_t *row_ptr, int64_t i, int64_t capacity, int64_t &p0, int64_t &p1)
{
    p0 = row_ptr[i];
    p1 = row_ptr[i + 1];
    if (p0 < 0) p0 = 0;
    if (p1 > capacity) p1 = capacity;
}

// val[p] = T_{i, col_idx[p]}: one wave per row, a random 8-byte read of M per entry.
__global__ __launch_bounds__(kThreads) void pattern_values_kernel(PatternArgs A)
{
    const int lane = threadIdx.x & (kLanes - 1);
    const int64_t wave = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * kWaves;
    for (int64_t i = wave; i < A.n; i += nwaves) {
        int64_t p0, p1;
        row_range(A.row_ptr, i, A.capacity, p0, p1);
        const double al = A.alpha[i];
        const double *Mrow = A.M + i * A.ldM;
        // four entries per lane in flight (the longest rows set the duration of the kernel)
        constexpr int kDepth = 4;
        for (int64_t p = p0 + lane; p < p1; p += kDepth * kLanes) {
            int32_t j[kDepth];
            double mij[kDepth], be[kDepth];
            bool ok[kDepth];
#pragma unroll
            for (int d = 0; d < kDepth; ++d) {
                const int64_t q = p + d * kLanes;
                j[d] = q < p1 ? A.col_idx[q] : -1;
                ok[d] = (uint32_t)j[d] < (uint32_t)A.m;  // anything else is not a column: the entry is left alone
            }
#pragma unroll
            for (int d = 0; d < kDepth; ++d) {
                mij[d] = ok[d] ? __builtin_nontemporal_load(Mrow + j[d]) : 0.0;
                be[d] = ok[d] ? A.beta[j[d]] : 0.0;
            }
#pragma unroll
            for (int d = 0; d < kDepth; ++d) {
                if (!ok[d]) continue;
                const int64_t q = p + d * kLanes;
                const double t = exp_eta_any((al + be[d]) - mij[d], A.ex);
                A.val[q] = t;
                if (A.val_csc) {
                    const int64_t c = A.csc_pos[q];
                    if (c >= 0 && c < A.capacity) A.val_csc[c] = t;
                }
            }
        }
    }
}

struct MatvecArgs {
    int n, m;
    double eta, tau;
    const int64_t *row_ptr;
    const int32_t *col_idx;
    const double *val;
    const int64_t *col_ptr;
    const int32_t *row_idx;
    const double *val_csc;
    int64_t capacity;
    const double *row_sum;
    const double *col_sum;
    const double *x;
    double *y;
    int64_t row_waves;  // waves that take rows; the rest take columns
};

// R vectors side by side: element t of vector k sits at [t * R + k], so one gather fetches the entry of
// every vector (R = 1: a plain array; R = 2: pairs, 16 bytes).
template <int R>
struct Pack {
    double v[R];
};
template <int R>
__device__ __forceinline__ Pack<R> load_pack(const double *a, int64_t t)
{
    static_assert(R == 1 || R == 2, "one vector or a pair");
    Pack<R> q;
    if constexpr (R == 2) {
        const dbl2 w = *reinterpret_cast<const dbl2 *>(a + 2 * t);
        q.v[0] = w.x;
        q.v[1] = w.y;
    } else {
        q.v[0] = a[t];
    }
    return q;
}
template <int R>
__device__ __forceinline__ void store_pack(double *a, int64_t t, const Pack<R> &q)
{
    if constexpr (R == 2) {
        *reinterpret_cast<dbl2 *>(a + 2 * t) = dbl2{q.v[0], q.v[1]};
    } else {
        a[t] = q.v[0];
    }
}

// This lane's share of sum_p val[p] * x[idx[p]] over entries [p0, p1) with idx[p] < limit.  Four
// entries per lane are loaded before the first is used: the longest rows (ten times the average)
// set the duration of the kernel, and their trips would otherwise each wait for a full memory latency.
template <int R>
__device__ __forceinline__ Pack<R> gather_dot(const int32_t *idx, const double *val, const double *x, int limit,
                                              int64_t p0, int64_t p1, int lane)
{
    constexpr int kDepth = 4;
    Pack<R> s;
#pragma unroll
    for (int k = 0; k < R; ++k) s.v[k] = 0.0;
    for (int64_t p = p0 + lane; p < p1; p += kDepth * kLanes) {
        int32_t j[kDepth];
        double v[kDepth];
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            const int64_t q = p + d * kLanes;
            j[d] = q < p1 ? idx[q] : -1;
            v[d] = q < p1 ? val[q] : 0.0;
        }
        Pack<R> xv[kDepth];
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            if ((uint32_t)j[d] < (uint32_t)limit) {
                xv[d] = load_pack<R>(x, j[d]);
            } else {
#pragma unroll
                for (int k = 0; k < R; ++k) xv[d].v[k] = 0.0;
            }
        }
#pragma unroll
        for (int d = 0; d < kDepth; ++d)
#pragma unroll
            for (int k = 0; k < R; ++k) s.v[k] += v[d] * xv[d].v[k];
    }
    return s;
}

// NR rows (or columns) at once, for the product inside the iteration: the loads of all NR rows go out before the
// first value is used, so a wave waits for one memory latency per NR rows instead of per row.  Row r covers
// entries [p0[r], p1[r]); per row the operations and their order are those of gather_dot, hence the same bits
// (trips beyond a row's end add +0, which changes nothing).  The first `nl` entries of x are read from a copy in LDS
// (`xl`), the others from memory; ALL: every index below `limit` is in xl.
template <int R, int NR, bool ALL>
__device__ __forceinline__ void gather_dot_rows(const int32_t *idx, const double *val, const double *x, const double *xl,
                                                int nl, int limit, const int64_t (&p0)[NR], const int64_t (&p1)[NR],
                                                int lane, Pack<R> (&s)[NR])
{
    constexpr int kDepth = 4;
    int longest = 0;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
#pragma unroll
        for (int k = 0; k < R; ++k) s[r].v[k] = 0.0;
        const int len = __builtin_amdgcn_readfirstlane((int)(p1[r] - p0[r]));
        longest = len > longest ? len : longest;
    }
    for (int t = 0; t < longest; t += kDepth * kLanes) {
        int32_t j[NR][kDepth];
        double v[NR][kDepth];
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int d = 0; d < kDepth; ++d) {
                const int64_t q = p0[r] + t + d * kLanes + lane;
                j[r][d] = q < p1[r] ? idx[q] : -1;
                v[r][d] = q < p1[r] ? val[q] : 0.0;
            }
        Pack<R> xv[NR][kDepth];
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int d = 0; d < kDepth; ++d) {
                if (ALL ? (uint32_t)j[r][d] < (uint32_t)limit : (uint32_t)j[r][d] < (uint32_t)nl) {
                    xv[r][d] = load_pack<R>(xl, j[r][d]);
                } else if (!ALL && (uint32_t)j[r][d] < (uint32_t)limit) {
                    xv[r][d] = load_pack<R>(x, j[r][d]);
                } else {
#pragma unroll
                    for (int k = 0; k < R; ++k) xv[r][d].v[k] = 0.0;
                }
            }
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int d = 0; d < kDepth; ++d)
#pragma unroll
                for (int k = 0; k < R; ++k) s[r].v[k] += v[r][d] * xv[r][d].v[k];
    }
}

// y = (H_Omega + tau I) x.  Waves [0, row_waves) take the alpha block row by row from the CSR, the others
// the beta block column by column from the pattern by columns; one wave per row or column where the grid
// allows.  (The call on its own; the conjugate-gradient iteration uses hessian_matvec_lds_kernel.)
__global__ __launch_bounds__(kThreads) void hessian_matvec_kernel(MatvecArgs A)
{
    const int lane = threadIdx.x & (kLanes - 1);
    const int64_t wave = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * kWaves;
    const int mb = A.m - 1;  // beta variables
    const double inv_eta = 1.0 / A.eta;
    if (wave < A.row_waves) {
        for (int64_t i = wave; i < A.n; i += A.row_waves) {
            int64_t p0, p1;
            row_range(A.row_ptr, i, A.capacity, p0, p1);
            const double s = wave_reduce1<OpSum>(gather_dot<1>(A.col_idx, A.val, A.x + A.n, mb, p0, p1, lane).v[0]);
            if (lane == 0) A.y[i] = (A.row_sum[i] * A.x[i] + s) * inv_eta + A.tau * A.x[i];
        }
    } else {
        const int64_t col_waves = nwaves - A.row_waves;
        for (int64_t j = wave - A.row_waves; j < mb; j += col_waves) {
            int64_t q0, q1;
            row_range(A.col_ptr, j, A.capacity, q0, q1);
            const double s = wave_reduce1<OpSum>(gather_dot<1>(A.row_idx, A.val_csc, A.x, A.n, q0, q1, lane).v[0]);
            if (lane == 0) A.y[A.n + j] = (A.col_sum[j] * A.x[A.n + j] + s) * inv_eta + A.tau * A.x[A.n + j];
        }
    }
}

// The product inside the conjugate-gradient iteration, for R vectors at once (x, y: R vectors side by side,
// see Pack), with the half of x that is gathered kept in LDS: workgroups of 16 waves, one per compute unit;
// the first row_blocks of them take the alpha block (they hold x's beta half, m - 1 entries), the others the
// beta block (they hold the alpha half, n entries).  What bounds the kernel above is not the bytes of the
// pattern but the gathers of x, each of which moves a cache line from L2 to a first-level cache far smaller
// than the vector; from LDS a gather costs a few cycles.  When a half has more than kMatvecLdsCap / R
// entries only its first entries are kept and the gathers of the others go to memory.
// The result does not depend on R or on what is kept in LDS: a row is summed by the same lanes in the same
// order as in the kernel above, wave W of the grid takes rows W, W + row waves, ..., and the workgroup writes
// its share of x_k^T y_k (for p^T A p) per group of kWaves waves to dot_part[k * dot_stride + ...], each the
// sum of its waves' shares in wave order.  Does nothing at all if *skip is set.
constexpr int kMatvecLdsCap = 20000;
constexpr int kMatvecLdsWaves = 16;
constexpr int kMatvecLdsThreads = kMatvecLdsWaves * kLanes;
constexpr int kMatvecRows = 2;                             // rows (columns) a wave has in flight
constexpr int kMatvecLdsGroup = kMatvecLdsWaves / kWaves;  // workgroups of the other kernel per workgroup of this one
static_assert(kMatvecLdsWaves % kWaves == 0, "whole workgroups of the other kernel");

// the first xlen doubles of src -> LDS; all loads of a thread go out before the first value is stored
// (16 bytes per load where src allows it)
__device__ __forceinline__ void lds_fill(double *xs, const double *src, int xlen)
{
    if ((reinterpret_cast<uintptr_t>(src) & 15) == 0) {
        constexpr int kPer = (kMatvecLdsCap / 2 + kMatvecLdsThreads - 1) / kMatvecLdsThreads;
        const int pairs = xlen / 2;
        dbl2 t[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int i = j * kMatvecLdsThreads + (int)threadIdx.x;
            t[j] = i < pairs ? reinterpret_cast<const dbl2 *>(src)[i] : dbl2{0.0, 0.0};
        }
        double last = 0.0;
        if ((xlen & 1) && threadIdx.x == 0) last = src[xlen - 1];
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int i = j * kMatvecLdsThreads + (int)threadIdx.x;
            if (i < pairs) reinterpret_cast<dbl2 *>(xs)[i] = t[j];
        }
        if ((xlen & 1) && threadIdx.x == 0) xs[xlen - 1] = last;
        return;
    }
    constexpr int kPer = (kMatvecLdsCap + kMatvecLdsThreads - 1) / kMatvecLdsThreads;
    double t[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int i = j * kMatvecLdsThreads + (int)threadIdx.x;
        t[j] = i < xlen ? src[i] : 0.0;
    }
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int i = j * kMatvecLdsThreads + (int)threadIdx.x;
        if (i < xlen) xs[i] = t[j];
    }
}

// One sweep of a wave over its items (rows of a CSR block or columns of the pattern by columns): items first,
// first + stride, ... below count.  A wave takes its items in batches of 64, lane l holding everything about item
// b0 + l * stride that one load can fetch (its range of entries and whatever `item.fetch` asks for), so the only
// memory latency left per group of kMatvecRows items is that of the entries themselves; the sums
// sum_p val[p] x[idx[p]] of an item are formed by the whole wave (gather_dot_rows), lane l keeps item l's and
// `item.finish` turns it into the item's result, stores it and returns the item's term of an inner product (or 0);
// dot[] (the same in every lane) grows by these terms item by item in ascending order.
//   Item: void fetch(int64_t t);  Pack<R> finish(int64_t t, bool have, const Pack<R> &sum)
// (the loads of a batch's first part: the kernels ask for those of their first batch before they fill the LDS)
struct SweepHead {
    int64_t q0, q1;
};
template <typename Item>
__device__ __forceinline__ SweepHead lds_sweep_head(const int64_t *ptr, int64_t capacity, int64_t count, int64_t b0,
                                                    int64_t stride, int lane, Item &item)
{
    SweepHead h{0, 0};
    const int64_t mine = b0 + lane * stride;
    if (mine < count) {
        row_range(ptr, mine, capacity, h.q0, h.q1);
        item.fetch(mine);
    }
    return h;
}

template <int R, bool ALL, typename Item>
__device__ __forceinline__ void lds_sweep(const int64_t *ptr, const int32_t *idx, const double *val, int64_t capacity,
                                          const double *xsrc, const double *xs, int nl, int limit, int64_t count,
                                          int64_t first, int64_t stride, int lane, Item &item, double (&dot)[R],
                                          SweepHead head /* of the batch at `first` */)
{
    for (int64_t b0 = first; b0 < count; b0 += kLanes * stride) {
        const int64_t mine = b0 + lane * stride;
        const bool have = mine < count;
        if (b0 != first) head = lds_sweep_head(ptr, capacity, count, b0, stride, lane, item);
        const int64_t q0 = head.q0, q1 = head.q1;
        Pack<R> sum;
#pragma unroll
        for (int k = 0; k < R; ++k) sum.v[k] = 0.0;
        const int64_t left = (count - b0 + stride - 1) / stride;
        const int items = __builtin_amdgcn_readfirstlane((int)(left < kLanes ? left : kLanes));
        for (int r0 = 0; r0 < items; r0 += kMatvecRows) {
            int64_t p0[kMatvecRows], p1[kMatvecRows];
#pragma unroll
            for (int r = 0; r < kMatvecRows; ++r) {
                const int src = r0 + r < items ? r0 + r : r0;  // (a surplus slot repeats item r0 with an empty range)
                p0[r] = read_lane_i64(q0, src);
                p1[r] = r0 + r < items ? read_lane_i64(q1, src) : p0[r];
            }
            Pack<R> s[kMatvecRows];
            gather_dot_rows<R, kMatvecRows, ALL>(idx, val, xsrc, xs, nl, limit, p0, p1, lane, s);
#pragma unroll
            for (int r = 0; r < kMatvecRows; ++r)
#pragma unroll
                for (int k = 0; k < R; ++k) {
                    const double t = wave_reduce1<OpSum>(s[r].v[k]);
                    if (lane == r0 + r) sum.v[k] = t;
                }
        }
        const Pack<R> term = item.finish(mine, have, sum);
        for (int r = 0; r < items; ++r)
#pragma unroll
            for (int k = 0; k < R; ++k) dot[k] += read_lane(term.v[k], r);
    }
}

// the waves' shares of an inner product -> one partial sum per group of kWaves waves, added up in wave order
// (the order block_sum uses): dot_part[k * dot_stride + blockIdx.x * kMatvecLdsGroup + g]
template <int R>
__device__ __forceinline__ void lds_leave_dots(const double (&dot)[R], double (*wave_dot)[kMatvecLdsWaves],
                                               double *dot_part, int dot_stride, int lane, int w)
{
#pragma unroll
    for (int k = 0; k < R; ++k)
        if (lane == 0) wave_dot[k][w] = dot[k];
    __syncthreads();
    if (threadIdx.x < kMatvecLdsGroup) {
        const int g = threadIdx.x;
#pragma unroll
        for (int k = 0; k < R; ++k) {
            double r = wave_dot[k][g * kWaves];
#pragma unroll
            for (int q = 1; q < kWaves; ++q) r += wave_dot[k][g * kWaves + q];
            dot_part[(size_t)k * dot_stride + (size_t)blockIdx.x * kMatvecLdsGroup + g] = r;
        }
    }
}

// item of the full product: y_t = (diag_t x_t + sum) / eta + tau x_t, and its term x_t y_t of x^T y
template <int R>
struct ProductItem {
    const double *diag;   // row or column sums of the plan
    const double *x;      // the vector(s), offset to this half
    double *y;
    double inv_eta, tau;
    double dg;
    Pack<R> xt;
    __device__ __forceinline__ void fetch(int64_t t)
    {
        dg = diag[t];
        xt = load_pack<R>(x, t);
    }
    __device__ __forceinline__ Pack<R> finish(int64_t t, bool have, const Pack<R> &sum)
    {
        Pack<R> yt, term;
#pragma unroll
        for (int k = 0; k < R; ++k) {
            yt.v[k] = have ? (dg * xt.v[k] + sum.v[k]) * inv_eta + tau * xt.v[k] : 0.0;
            term.v[k] = have ? yt.v[k] * xt.v[k] : 0.0;
        }
        if (have) store_pack<R>(y, t, yt);
        return term;
    }
};

// ALL: both halves fit entirely (the host has checked), so no gather needs the test for where its entry is.
template <bool DOT, int R, bool ALL>
__global__ __launch_bounds__(kMatvecLdsThreads) void hessian_matvec_lds_kernel(MatvecArgs A, double *dot_part,
                                                                               int dot_stride, const int *skip,
                                                                               int row_blocks)
{
    __shared__ __attribute__((aligned(16))) double xs[kMatvecLdsCap];
    __shared__ double wave_dot[R][kMatvecLdsWaves];
    static_assert(sizeof(double) * (kMatvecLdsCap + R * kMatvecLdsWaves) <= 160 * 1024, "LDS per CU");
    if (DOT && *skip) return;
    const int lane = threadIdx.x & (kLanes - 1), w = threadIdx.x >> 6;
    const int mb = A.m - 1;  // beta variables
    const bool rows = (int)blockIdx.x < row_blocks;
    const double *xsrc = rows ? A.x + (int64_t)A.n * R : A.x;
    const int limit = rows ? mb : A.n;                                         // entries the gathers may ask for
    const int nl = limit < kMatvecLdsCap / R ? limit : kMatvecLdsCap / R;      // of which the first nl sit in LDS
    double dot[R];  // the wave's share of x^T y (the same in every lane)
#pragma unroll
    for (int k = 0; k < R; ++k) dot[k] = 0.0;
    ProductItem<R> item;
    item.inv_eta = 1.0 / A.eta;
    item.tau = A.tau;
    item.diag = rows ? A.row_sum : A.col_sum;
    item.x = rows ? A.x : A.x + (int64_t)A.n * R;
    item.y = rows ? A.y : A.y + (int64_t)A.n * R;
    const int64_t *ptr = rows ? A.row_ptr : A.col_ptr;
    const int64_t count = rows ? A.n : mb;
    const int64_t first = (int64_t)(rows ? (int)blockIdx.x : (int)blockIdx.x - row_blocks) * kMatvecLdsWaves + w;
    const int64_t stride = (int64_t)(rows ? row_blocks : (int)gridDim.x - row_blocks) * kMatvecLdsWaves;
    const SweepHead head = lds_sweep_head(ptr, A.capacity, count, first, stride, lane, item);
    lds_fill(xs, xsrc, nl * R);
    __syncthreads();
    lds_sweep<R, ALL>(ptr, rows ? A.col_idx : A.row_idx, rows ? A.val : A.val_csc, A.capacity, xsrc, xs, nl, limit, count,
                      first, stride, lane, item, dot, head);
    if constexpr (DOT) lds_leave_dots<R>(dot, wave_dot, dot_part, dot_stride, lane, w);
}

struct LowerArgs {
    int n, m;
    double eta, tau;
    const int64_t *row_ptr;
    const int32_t *col_idx;
    const double *val;
    int64_t capacity;
    const double *row_sum;
    const double *col_sum;
    int64_t *h_col_ptr;   // [n + m]
    int32_t *h_row_idx;
    double *h_val;
    int64_t h_capacity;
    int64_t *info;        // [2]: entries, overflow
    int64_t *blk;         // [nblk + 1] workspace: dropped entries per block of rows, then their prefix
    int nblk;
    int values_only;
};

// does row i end with an entry in the dropped column (columns ascend, so it can only be the last one)
__device__ __forceinline__ int row_drops(const LowerArgs &A, int64_t i)
{
    int64_t p0, p1;
    row_range(A.row_ptr, i, A.capacity, p0, p1);
    return (p1 > p0 && A.col_idx[p1 - 1] == A.m - 1) ? 1 : 0;
}

// step 1: dropped entries per block of kRowsPerScanBlock rows; a thread per row, a 32-lane group per block
__global__ __launch_bounds__(kThreads) void lower_count_kernel(LowerArgs A)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    int c = i < A.n ? row_drops(A, i) : 0;
#pragma unroll
    for (int off = kRowsPerScanBlock / 2; off >= 1; off >>= 1) c += __shfl_xor(c, off, kLanes);
    const int64_t rb = i / kRowsPerScanBlock;
    if ((threadIdx.x & (kRowsPerScanBlock - 1)) == 0 && rb < A.nblk) A.blk[rb] = c;
}

// step 2: exclusive prefix over the blocks (one workgroup)
__global__ __launch_bounds__(kThreads) void lower_scan_kernel(LowerArgs A)
{
    __shared__ int64_t part[kThreads + 1];
    const int per = (A.nblk + kThreads - 1) / kThreads;
    const int64_t b0 = (int64_t)threadIdx.x * per;
    int64_t s = 0;
    for (int64_t b = b0; b < b0 + per && b < A.nblk; ++b) s += A.blk[b];
    part[threadIdx.x + 1] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        part[0] = 0;
        for (int t = 1; t <= kThreads; ++t) part[t] += part[t - 1];
    }
    __syncthreads();
    int64_t run = part[threadIdx.x];
    for (int64_t b = b0; b < b0 + per && b < A.nblk; ++b) {
        const int64_t c = A.blk[b];
        A.blk[b] = run;
        run += c;
    }
    if (threadIdx.x == kThreads - 1) A.blk[A.nblk] = part[kThreads];  // all dropped entries
}

// step 3: column i < n of the lower triangle = diagonal, then row i of T^Omega_{-m} as rows n + j;
// columns n + j hold their diagonal only.  A workgroup takes one block of rows: it works out where
// each of its columns starts, then all its threads walk the block's pattern entries together
// (coalesced), finding each entry's row by bisection in LDS.  Workgroups beyond the row blocks write
// the beta diagonal.
__global__ __launch_bounds__(kThreads) void lower_fill_kernel(LowerArgs A)
{
    __shared__ int64_t rp[kRowsPerScanBlock + 1];
    __shared__ int64_t base[kRowsPerScanBlock];
    const int mb = A.m - 1;
    const double inv_eta = 1.0 / A.eta;
    if ((int64_t)blockIdx.x < A.nblk) {
        const int64_t r0 = (int64_t)blockIdx.x * kRowsPerScanBlock;
        const int rows = (int)(A.n - r0 < kRowsPerScanBlock ? A.n - r0 : kRowsPerScanBlock);
        const int t = threadIdx.x;
        if (t <= rows) {
            int64_t v = A.row_ptr[r0 + t];
            rp[t] = v < 0 ? 0 : v > A.capacity ? A.capacity : v;
        }
        __syncthreads();
        if (t < kLanes) {  // first wave: lanes 0 .. rows-1 own a row each
            const bool live = t < rows;
            int64_t start = 0;
            if (A.values_only) {
                if (live) start = A.h_col_ptr[r0 + t];
            } else {
                // i diagonals and row_ptr[i] pattern entries come before column i, minus the dropped ones
                const int flag = live ? row_drops(A, r0 + t) : 0;
                int incl = flag;
#pragma unroll
                for (int off = 1; off < kRowsPerScanBlock; off <<= 1) {
                    const int up = __shfl_up(incl, off, kLanes);
                    if (t >= off) incl += up;
                }
                if (live) start = (r0 + t) + rp[t] - (A.blk[blockIdx.x] + (incl - flag));
            }
            if (live) {
                base[t] = start;
                if (!A.values_only) A.h_col_ptr[r0 + t] = start;
                if (start >= 0 && start < A.h_capacity) {
                    if (!A.values_only) A.h_row_idx[start] = (int32_t)(r0 + t);
                    A.h_val[start] = A.row_sum[r0 + t] * inv_eta + A.tau;
                }
            }
        }
        __syncthreads();
        for (int64_t p = rp[0] + t; p < rp[rows]; p += kThreads) {
            int lo = 0, hi = rows;  // rp[lo] <= p < rp[hi]
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (rp[mid] <= p) lo = mid;
                else hi = mid;
            }
            const int32_t j = A.col_idx[p];
            const int64_t q = base[lo] + 1 + (p - rp[lo]);
            if ((uint32_t)j < (uint32_t)mb && q >= 0 && q < A.h_capacity) {
                if (!A.values_only) A.h_row_idx[q] = A.n + j;
                A.h_val[q] = A.val[p] * inv_eta;
            }
        }
    } else {
        // total entries: n + (m-1) diagonals + pattern entries outside the dropped column
        int64_t pn = A.row_ptr[A.n];
        if (pn > A.capacity) pn = A.capacity;
        if (pn < 0) pn = 0;
        const int64_t first_beta = A.values_only ? A.h_col_ptr[A.n + mb] - mb : (int64_t)A.n + pn - A.blk[A.nblk];
        const int64_t j = ((int64_t)blockIdx.x - A.nblk) * kThreads + threadIdx.x;
        if (j < mb) {
            const int64_t q = first_beta + j;
            if (!A.values_only) A.h_col_ptr[A.n + j] = q;
            if (q >= 0 && q < A.h_capacity) {
                if (!A.values_only) A.h_row_idx[q] = (int32_t)(A.n + j);
                A.h_val[q] = A.col_sum[j] * inv_eta + A.tau;
            }
        }
        if ((int64_t)blockIdx.x == A.nblk && threadIdx.x == 0) {
            const int64_t total = first_beta + mb;
            if (!A.values_only) A.h_col_ptr[A.n + mb] = total;
            A.info[0] = total;
            A.info[1] = total > A.h_capacity ? 1 : 0;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Optimality measures of a dual point from its row and column sums (App. A.5), and the choice
// between two candidate iterates (Sec. 4.3).
// ---------------------------------------------------------------------------------------------

constexpr int kMetricParts = 256;   // workgroups of the first stage
constexpr int kMetricSums = 5;

struct MetricArgs {
    int64_t n, m;
    const double *a, *b, *alpha, *beta, *row_sum, *col_sum;
    double eta;
    double *part;     // [kMetricParts][kMetricSums]
    double *metrics;  // [4]: L_p, L_p - L_d, marginal error, || grad f ||_2
    int parts;
};

// sums over a slice of the n + m entries: alpha^T r + beta^T c, alpha^T (r - a) + beta^T (c - b),
// sum r, sum |r - a| + sum |c - b|, sum (r - a)^2 + sum_{j < m-1} (c - b)^2
__global__ __launch_bounds__(kThreads) void metric_parts_kernel(MetricArgs A)
{
    __shared__ double wsum[kWaves][kMetricSums];
    double s[kMetricSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
    const int64_t total = A.n + A.m;
    for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < total; t += (int64_t)gridDim.x * kThreads) {
        const bool row = t < A.n;
        const int64_t k = row ? t : t - A.n;
        const double dual = row ? A.alpha[k] : A.beta[k];
        const double sum = row ? A.row_sum[k] : A.col_sum[k];
        const double d = sum - (row ? A.a[k] : A.b[k]);
        s[0] += dual * sum;
        s[1] += dual * d;
        if (row) s[2] += sum;
        s[3] += fabs(d);
        if (row || k < A.m - 1) s[4] += d * d;
    }
#pragma unroll
    for (int e = 0; e < kMetricSums; ++e) s[e] = wave_reduce1<OpSum>(s[e]);
    if ((threadIdx.x & (kLanes - 1)) == 0)
        for (int e = 0; e < kMetricSums; ++e) wsum[threadIdx.x >> 6][e] = s[e];
    __syncthreads();
    if (threadIdx.x < kMetricSums) {
        double v = 0.0;
        for (int w = 0; w < kWaves; ++w) v += wsum[w][threadIdx.x];
        A.part[(size_t)blockIdx.x * kMetricSums + threadIdx.x] = v;
    }
}

__global__ void metric_final_kernel(MetricArgs A)
{
    if (threadIdx.x != 0) return;
    double s[kMetricSums] = {0.0, 0.0, 0.0, 0.0, 0.0};
    for (int p = 0; p < A.parts; ++p)
        for (int e = 0; e < kMetricSums; ++e) s[e] += A.part[(size_t)p * kMetricSums + e];
    // L_p = <T, M> + eta sum T log T - eta sum T = sum_ij T_ij (alpha_i + beta_j) - eta sum T
    A.metrics[0] = s[0] - A.eta * s[2];
    A.metrics[1] = s[1];
    A.metrics[2] = s[3];
    A.metrics[3] = sqrt(s[4]);
}

struct ChooseArgs {
    int64_t n, m;
    const double *obj_q, *obj_s;
    const double *alpha_q, *beta_q, *alpha_s, *beta_s;
    double *alpha_out, *beta_out;
    int64_t *choice;
};

// keep the candidate with the larger dual objective (the quasi-Newton one unless the other is strictly better)
__global__ __launch_bounds__(kThreads) void choose_candidate_kernel(ChooseArgs A)
{
    const bool take_s = A.obj_s[0] > A.obj_q[0];
    const double *al = take_s ? A.alpha_s : A.alpha_q;
    const double *be = take_s ? A.beta_s : A.beta_q;
    const int64_t total = A.n + A.m;
    for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < total; t += (int64_t)gridDim.x * kThreads) {
        if (t < A.n) A.alpha_out[t] = al[t];
        else A.beta_out[t - A.n] = be[t - A.n];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) A.choice[0] = take_s ? 1 : 0;
}

}  // namespace regot
