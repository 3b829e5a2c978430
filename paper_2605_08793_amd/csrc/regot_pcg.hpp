// The quasi-Newton direction d = -B^{-1} g, B = H_Omega + R + tau I (Algorithm 1, lines 3-7;
// eq. (5), (6)), by an iterative solve on the GPU.
//
// The paper factorises H_Omega with a sparse Cholesky code whose symbolic phase runs on the host
// (Sec. 3.2) and names iterative solvers as future work; this is that alternative, built from
// regot_hessian_matvec: conjugate gradients on A = H_Omega + tau I (symmetric positive definite by
// Theorem 1) preconditioned with its diagonal, and the Sherman-Morrison-Woodbury identity for the
// rank-two term R = xi u u^T + zeta v v^T.  Because v = A s^-, A^{-1} v = s^- is known, so two solves
// with A (for g and for u = y^-) give B^{-1} g.
//
// One iteration is three kernels (product + p^T A p | x, r, z and their dot products | p).  Dot
// products are summed in two stages in a fixed order: every workgroup leaves a partial sum, and
// every workgroup of the next kernel adds all partials up for itself.  The scalars live on the
// device; after convergence the remaining kernels return at once.
//
// The kernels are written for R right-hand sides at once (R = 1 or 2), the vectors of the R systems
// side by side (see Pack): the product then reads the pattern once and fetches the entries of both
// vectors with one gather, so the two solves of a direction cost little more than one.  Each system
// keeps its own scalars and stops on its own: once it has converged its vectors are left alone, and
// the arithmetic of a system does not depend on the other one being there.
//
// Further down: the same solve through the Schur complement of the first diagonal block (half the
// iterations; regot_pcg_solve_reduced), which reuses the vector kernels on the second block alone.
#pragma once

#include "regot_sparse.hpp"

namespace regot {

constexpr int kPcgParts = 1024;   // most workgroups whose partial sums a later kernel adds up
constexpr int kPcgMaxRhs = 2;

template <int R>
struct PcgScalars {
    double rz[R];        // r^T z
    double bb[R];        // ||rhs||^2 (reduced solves: of the right-hand side of the whole system)
    double rr[R];        // ||r||^2
    long long iters[R];
    int done[R];         // converged (or nothing to do)
    int all_done;        // every system is
    int pad;
};

struct PcgArgs {
    MatvecArgs mv;    // mv.x = p, mv.y = Ap
    int64_t N;
    const double *rhs[kPcgMaxRhs];  // one plain array per system
    double *x_out[kPcgMaxRhs];      // one plain array per system
    double *x, *r, *z, *p, *Ap;     // R vectors side by side (R = 1: x is x_out[0] itself)
    double *part;     // [4][R][kPcgParts]: p^T A p | r^T z | r^T r | (reduced solves) ||rhs||^2
    void *sc;         // PcgScalars<R>[2], alternating by iteration
    double rtol;
    int mv_blocks, vec_blocks;
    double *info;     // [4 R]: per system iterations, converged, ||r||, ||rhs||
};

template <int R>
__device__ __forceinline__ PcgScalars<R> *pcg_scalars(const PcgArgs &A, int slot)
{
    return static_cast<PcgScalars<R> *>(A.sc) + slot;
}

__device__ __forceinline__ double pcg_diag(const MatvecArgs &M, int64_t t)
{
    return (t < M.n ? M.row_sum[t] : M.col_sum[t - M.n]) / M.eta + M.tau;
}

// a thread's share of the sum of part[0 .. count) (asked for early where the sum is needed behind other loads)
__device__ __forceinline__ double part_share(const double *part, int count)
{
    double v = 0.0;
    for (int k = threadIdx.x; k < count; k += kThreads) v += part[k];
    return v;
}

// sum of part[0 .. count) in a fixed order; every thread of the workgroup gets it
__device__ __forceinline__ double sum_parts(const double *part, int count, double *lds)
{
    return block_sum(part_share(part, count), lds);
}

// a workgroup's partial sums of r^T z and r^T r of every system
template <int R>
__device__ __forceinline__ void pcg_leave_partials(const PcgArgs &A, const double (&rz)[R], const double (&rr)[R],
                                                   double *lds)
{
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const double a = block_sum(rz[k], lds), b = block_sum(rr[k], lds);
        if (threadIdx.x == 0) {
            A.part[(size_t)(R + k) * kPcgParts + blockIdx.x] = a;
            A.part[(size_t)(2 * R + k) * kPcgParts + blockIdx.x] = b;
        }
    }
}

// x = 0, r = rhs, z = r / diag, p = z; partial sums of r^T z and r^T r
template <int R>
__global__ __launch_bounds__(kThreads) void pcg_start_kernel(PcgArgs A)
{
    __shared__ double lds[kWaves];
    double rz[R], rr[R];
#pragma unroll
    for (int k = 0; k < R; ++k) rz[k] = rr[k] = 0.0;
    for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < A.N; t += (int64_t)gridDim.x * kThreads) {
        const double dg = pcg_diag(A.mv, t);
        Pack<R> r, z, zero;
#pragma unroll
        for (int k = 0; k < R; ++k) {
            r.v[k] = A.rhs[k][t];
            z.v[k] = r.v[k] / dg;
            zero.v[k] = 0.0;
            rz[k] += r.v[k] * z.v[k];
            rr[k] += r.v[k] * r.v[k];
        }
        store_pack<R>(A.x, t, zero);
        store_pack<R>(A.r, t, r);
        store_pack<R>(A.z, t, z);
        store_pack<R>(A.p, t, z);
    }
    pcg_leave_partials<R>(A, rz, rr, lds);
}

// norm_blocks > 0: the tolerance is relative to the norm whose squares' partial sums are in row 3R + k of
// `part` (the right-hand side of a larger system this one was reduced from), and a residual that is already
// below it needs no iteration.
template <int R>
__global__ __launch_bounds__(kThreads) void pcg_start_scalars_kernel(PcgArgs A, int norm_blocks)
{
    __shared__ double lds[kWaves];
    PcgScalars<R> s;
    s.all_done = 1;
    s.pad = 0;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const double rz = sum_parts(A.part + (size_t)(R + k) * kPcgParts, A.vec_blocks, lds);
        const double rr = sum_parts(A.part + (size_t)(2 * R + k) * kPcgParts, A.vec_blocks, lds);
        s.rz[k] = rz;
        s.bb[k] = rr;
        s.rr[k] = rr;
        s.iters[k] = 0;
        s.done[k] = rr == 0.0 ? 1 : 0;
        if (norm_blocks > 0) {
            s.bb[k] = sum_parts(A.part + (size_t)(3 * R + k) * kPcgParts, norm_blocks, lds);
            if (rr <= A.rtol * A.rtol * s.bb[k]) s.done[k] = 1;
        }
        s.all_done &= s.done[k];
    }
    if (threadIdx.x == 0) *pcg_scalars<R>(A, 0) = s;
}

// x += step p, r -= step Ap, z = r / diag; partial sums of the new r^T z and r^T r
template <int R>
__global__ __launch_bounds__(kThreads) void pcg_update_kernel(PcgArgs A, int it)
{
    __shared__ double lds[kWaves];
    // the vectors of the thread's first element are asked for before the scalars they will be combined with
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    double dg = 1.0;
    Pack<R> x, r, z, p, Ap;
    auto fetch = [&]() {
        dg = pcg_diag(A.mv, t);
        x = load_pack<R>(A.x, t);
        r = load_pack<R>(A.r, t);
        z = load_pack<R>(A.z, t);
        p = load_pack<R>(A.p, t);
        Ap = load_pack<R>(A.Ap, t);
    };
    if (t < A.N) fetch();
    double share[R];  // (likewise the partial sums, which are there whether or not the scalars say "done")
#pragma unroll
    for (int k = 0; k < R; ++k) share[k] = part_share(A.part + (size_t)k * kPcgParts, A.mv_blocks);
    const PcgScalars<R> cur = *pcg_scalars<R>(A, it & 1);
    if (cur.all_done) return;
    double step[R];
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const double pAp = block_sum(share[k], lds);
        step[k] = cur.rz[k] / pAp;
    }
    double rz[R], rr[R];
#pragma unroll
    for (int k = 0; k < R; ++k) rz[k] = rr[k] = 0.0;
    while (t < A.N) {
#pragma unroll
        for (int k = 0; k < R; ++k) {
            if (!cur.done[k]) {   // a system that has converged keeps its vectors
                x.v[k] += step[k] * p.v[k];
                r.v[k] = r.v[k] - step[k] * Ap.v[k];
                z.v[k] = r.v[k] / dg;
            }
            rz[k] += r.v[k] * z.v[k];
            rr[k] += r.v[k] * r.v[k];
        }
        store_pack<R>(A.x, t, x);
        store_pack<R>(A.r, t, r);
        store_pack<R>(A.z, t, z);
        t += stride;
        if (t < A.N) fetch();
    }
    pcg_leave_partials<R>(A, rz, rr, lds);
}

// p = z + (new r^T z / old r^T z) p; the scalars of the next iteration
template <int R>
__global__ __launch_bounds__(kThreads) void pcg_direction_kernel(PcgArgs A, int it)
{
    __shared__ double lds[kWaves];
    // (as in the kernel above: the first element's vectors are on their way while the scalars are worked out)
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    Pack<R> p, z;
    if (t < A.N) {
        p = load_pack<R>(A.p, t);
        z = load_pack<R>(A.z, t);
    }
    double share_rz[R], share_rr[R];
#pragma unroll
    for (int k = 0; k < R; ++k) {
        share_rz[k] = part_share(A.part + (size_t)(R + k) * kPcgParts, A.vec_blocks);
        share_rr[k] = part_share(A.part + (size_t)(2 * R + k) * kPcgParts, A.vec_blocks);
    }
    const PcgScalars<R> cur = *pcg_scalars<R>(A, it & 1);
    if (cur.all_done) {
        if (blockIdx.x == 0 && threadIdx.x == 0) *pcg_scalars<R>(A, (it + 1) & 1) = cur;
        return;
    }
    PcgScalars<R> nx = cur;
    double ratio[R];
    nx.all_done = 1;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const double rz = block_sum(share_rz[k], lds);
        const double rr = block_sum(share_rr[k], lds);
        ratio[k] = rz / cur.rz[k];
        if (!cur.done[k]) {
            nx.rz[k] = rz;
            nx.rr[k] = rr;
            nx.iters[k] = cur.iters[k] + 1;
            nx.done[k] = rr <= A.rtol * A.rtol * cur.bb[k] ? 1 : 0;
        }
        nx.all_done &= nx.done[k];
    }
    while (t < A.N) {
#pragma unroll
        for (int k = 0; k < R; ++k)
            if (!cur.done[k]) p.v[k] = z.v[k] + ratio[k] * p.v[k];
        store_pack<R>(A.p, t, p);
        t += stride;
        if (t < A.N) {
            p = load_pack<R>(A.p, t);
            z = load_pack<R>(A.z, t);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) *pcg_scalars<R>(A, (it + 1) & 1) = nx;
}

// After the last iteration of a call: the scalars go back to slot 0 (a later call continues from
// there), and with more than one system the solutions go to the callers' arrays.
template <int R>
__global__ __launch_bounds__(kThreads) void pcg_finish_kernel(PcgArgs A, int its)
{
    if constexpr (R > 1) {
        for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < A.N; t += (int64_t)gridDim.x * kThreads) {
            const Pack<R> x = load_pack<R>(A.x, t);
#pragma unroll
            for (int k = 0; k < R; ++k) A.x_out[k][t] = x.v[k];
        }
    }
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    const PcgScalars<R> s = *pcg_scalars<R>(A, its & 1);
    *pcg_scalars<R>(A, 0) = s;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        A.info[4 * k + 0] = (double)s.iters[k];
        A.info[4 * k + 1] = (double)s.done[k];
        A.info[4 * k + 2] = sqrt(s.rr[k]);
        A.info[4 * k + 3] = sqrt(s.bb[k]);
    }
}

// ---------------------------------------------------------------------------------------------
// The same system through its Schur complement (regot_pcg_solve_reduced).  With
//     H_Omega + tau I = [ D1   B  ]     D1 = diag(T 1) / eta + tau        (n)
//                       [ B^T  D2 ]     D2 = diag(T_{-m}^T 1) / eta + tau (m - 1),   B = T^Omega_{-m} / eta
// (eq. (7)) and rhs = (g1, g2), eliminating the first block leaves S x2 = g2 - B^T D1^{-1} g1 with
// S = D2 - B^T D1^{-1} B (symmetric positive definite as the whole matrix is, Theorem 1), and
// x1 = D1^{-1} (g1 - B x2).  Conjugate gradients on S preconditioned with D2 take about half the iterations
// of the iteration on the whole matrix (the classical result for matrices whose diagonal blocks are diagonal) at
// the same cost per iteration: one product with B (by rows) and one with B^T (by columns), now one after the
// other, each by all compute units.  The vector kernels above run on the second block alone.
// ---------------------------------------------------------------------------------------------
// R systems at once as in the kernels above: the vectors the iteration itself produces (u, p, S p, the iterate) are
// "packed", R side by side (see Pack); what the caller hands over or gets back (the right-hand sides, the solutions)
// and the right-hand sides of the reduced systems are plain arrays, one per system.
enum SchurMode {
    kSchurRows = 0,       // out_i = (sum_j T_ij in_j / eta) / D1_i             u = D1^{-1} B p      out packed
    kSchurRowsFinal = 1,  // out_i = (own_i - sum_j T_ij in_j / eta) / D1_i     x1, own = g1         own, out plain
    kSchurCols = 2,       // out_j = D2_j own_j - sum_i T_ij in_i / eta         S p, own = p         own, out packed;
                          //                                                    and own^T out
    kSchurColsRhs = 3     // out_j = own_j - sum_i T_ij in_i / eta              own = g2             own, out plain
};
constexpr int kPcgPartRows = 4 * kPcgMaxRhs;  // rows of `part`: p^T A p | r^T z | r^T r | ||rhs||^2, R of each

template <int R>
struct SchurArgs {
    MatvecArgs mv;       // pattern, values, sums, eta, tau (x, y, row_waves unused)
    const double *in;    // packed: the vectors the entries are multiplied with, m - 1 entries (rows) or n (columns)
    const double *own[R];  // see SchurMode; a packed vector is own[0]
    double *out[R];        // a packed vector is out[0]
    double *dot_part;    // kSchurCols: partial sums of own^T out, one per system and group of kWaves waves
    const int *skip;     // the kernel does nothing if *skip is set (may be NULL)
};

template <int MODE, int R>
struct SchurItem {
    static constexpr bool kPacked = MODE == kSchurRows || MODE == kSchurCols;
    const double *sums;
    const double *own[R];
    double *out[R];
    double eta, inv_eta, tau;
    double dg;
    Pack<R> mine;
    __device__ __forceinline__ void fetch(int64_t t)
    {
        dg = sums[t] / eta + tau;
        if (MODE == kSchurCols) {
            mine = load_pack<R>(own[0], t);
        } else {
#pragma unroll
            for (int k = 0; k < R; ++k) mine.v[k] = MODE == kSchurRows ? 0.0 : own[k][t];
        }
    }
    __device__ __forceinline__ Pack<R> finish(int64_t t, bool have, const Pack<R> &sum)
    {
        Pack<R> term, o;
#pragma unroll
        for (int k = 0; k < R; ++k) {
            term.v[k] = 0.0;
            const double bs = sum.v[k] * inv_eta;
            if (MODE == kSchurRows) o.v[k] = bs / dg;
            else if (MODE == kSchurRowsFinal) o.v[k] = (mine.v[k] - bs) / dg;
            else if (MODE == kSchurCols) o.v[k] = dg * mine.v[k] - bs;
            else o.v[k] = mine.v[k] - bs;
            if (MODE == kSchurCols && have) term.v[k] = o.v[k] * mine.v[k];
        }
        if (have) {
            if (kPacked) {
                store_pack<R>(out[0], t, o);
            } else {
#pragma unroll
                for (int k = 0; k < R; ++k) out[k][t] = o.v[k];
            }
        }
        return term;
    }
};

template <int MODE, int R, bool ALL>
__global__ __launch_bounds__(kMatvecLdsThreads) void schur_half_kernel(SchurArgs<R> S)
{
    __shared__ __attribute__((aligned(16))) double xs[kMatvecLdsCap];
    __shared__ double wave_dot[R][kMatvecLdsWaves];
    if (S.skip != nullptr && *S.skip) return;
    const MatvecArgs &A = S.mv;
    constexpr bool ROWS = MODE == kSchurRows || MODE == kSchurRowsFinal;
    const int lane = threadIdx.x & (kLanes - 1), w = threadIdx.x >> 6;
    const int mb = A.m - 1;
    const int limit = ROWS ? mb : A.n;
    const int nl = limit < kMatvecLdsCap / R ? limit : kMatvecLdsCap / R;
    double dot[R];
    SchurItem<MODE, R> item;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        dot[k] = 0.0;
        item.own[k] = S.own[k];
        item.out[k] = S.out[k];
    }
    item.sums = ROWS ? A.row_sum : A.col_sum;
    item.eta = A.eta;
    item.inv_eta = 1.0 / A.eta;
    item.tau = A.tau;
    const int64_t *ptr = ROWS ? A.row_ptr : A.col_ptr;
    const int64_t count = ROWS ? A.n : mb;
    const int64_t first = (int64_t)blockIdx.x * kMatvecLdsWaves + w, stride = (int64_t)gridDim.x * kMatvecLdsWaves;
    const SweepHead head = lds_sweep_head(ptr, A.capacity, count, first, stride, lane, item);
    lds_fill(xs, S.in, nl * R);
    __syncthreads();
    lds_sweep<R, ALL>(ptr, ROWS ? A.col_idx : A.row_idx, ROWS ? A.val : A.val_csc, A.capacity, S.in, xs, nl, limit, count,
                      first, stride, lane, item, dot, head);
    if constexpr (MODE == kSchurCols) lds_leave_dots<R>(dot, wave_dot, S.dot_part, (int)kPcgParts, lane, w);
}

// start of a reduced solve: u = D1^{-1} g1 (packed), and partial sums of ||rhs||^2 over both blocks -> rows 3R + k
// of `part`
template <int R>
struct SchurPrepareArgs {
    int64_t n, N;
    const double *rhs[R];
    const double *row_sum;
    double eta, tau;
    double *u;
    double *part;
};
template <int R>
__global__ __launch_bounds__(kThreads) void schur_prepare_kernel(SchurPrepareArgs<R> A)
{
    __shared__ double lds[kWaves];
    double gg[R];
#pragma unroll
    for (int k = 0; k < R; ++k) gg[k] = 0.0;
    for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < A.N; t += (int64_t)gridDim.x * kThreads) {
        Pack<R> g;
#pragma unroll
        for (int k = 0; k < R; ++k) {
            g.v[k] = A.rhs[k][t];
            gg[k] += g.v[k] * g.v[k];
        }
        if (t < A.n) {
            const double d1 = A.row_sum[t] / A.eta + A.tau;
#pragma unroll
            for (int k = 0; k < R; ++k) g.v[k] = g.v[k] / d1;
            store_pack<R>(A.u, t, g);
        }
    }
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const double s = block_sum(gg[k], lds);
        if (threadIdx.x == 0) A.part[(size_t)(3 * R + k) * kPcgParts + blockIdx.x] = s;
    }
}

// ---------------------------------------------------------------------------------------------
// d = -B^{-1} g from p = A^{-1} g, q = A^{-1} y, s = s^- (= A^{-1} v), y = y^-, v = A s^-.
// Two kernels: partial sums of the seven inner products, one set per workgroup; then every workgroup
// adds the partials up for itself (fixed order), solves the 2 x 2 system and writes its share of d.
// Without a previous step, or when (y^-)^T s^- <= 1e-6 ||y^-||^2 (Algorithm 1, line 5), R = 0 and
// d = -p.
// ---------------------------------------------------------------------------------------------
constexpr int kCombineDots = 7;  // y.s, y.y, y.q, v.q, v.s, y.p, v.p

struct CombineArgs {
    int64_t N;
    const double *p, *q, *s, *y, *v;  // q, s, y, v may be NULL together: no previous step
    double *d;
    double *info;  // [2]: 1 if the rank-two term was used, (y^-)^T s^-
    double *part;  // [kCombineDots][kPcgParts]
    int blocks;    // workgroups of both kernels
};

__global__ __launch_bounds__(kThreads) void splr_dots_kernel(CombineArgs A)
{
    __shared__ double lds[kWaves];
    double acc[kCombineDots];
#pragma unroll
    for (int k = 0; k < kCombineDots; ++k) acc[k] = 0.0;
    for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < A.N; t += (int64_t)gridDim.x * kThreads) {
        const double y = A.y[t], s = A.s[t], v = A.v[t], q = A.q[t], p = A.p[t];
        acc[0] += y * s;
        acc[1] += y * y;
        acc[2] += y * q;
        acc[3] += v * q;
        acc[4] += v * s;
        acc[5] += y * p;
        acc[6] += v * p;
    }
#pragma unroll
    for (int k = 0; k < kCombineDots; ++k) {
        const double t = block_sum(acc[k], lds);
        if (threadIdx.x == 0) A.part[(size_t)k * kPcgParts + blockIdx.x] = t;
    }
}

__global__ __launch_bounds__(kThreads) void splr_combine_kernel(CombineArgs A)
{
    __shared__ double lds[kWaves];
    bool use = A.s != nullptr;
    double c0 = 0.0, c1 = 0.0, ys_out = 0.0;
    if (use) {
        double dot[kCombineDots];
#pragma unroll
        for (int k = 0; k < kCombineDots; ++k) dot[k] = sum_parts(A.part + (size_t)k * kPcgParts, A.blocks, lds);
        const double ys = dot[0], yy = dot[1], yq = dot[2], vq = dot[3], vs = dot[4], yp = dot[5], vp = dot[6];
        ys_out = ys;
        use = ys > 1e-6 * yy;
        if (use) {
            // (C^{-1} + U^T A^{-1} U) c = U^T p with U = [y v], C^{-1} = diag(y^T s, -v^T s), A^{-1} U = [q s]
            const double k00 = ys + yq, k01 = ys, k10 = vq, k11 = -vs + vs;
            const double det = k00 * k11 - k01 * k10;
            c0 = (yp * k11 - k01 * vp) / det;
            c1 = (k00 * vp - k10 * yp) / det;
        }
    }
    for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < A.N; t += (int64_t)gridDim.x * kThreads)
        A.d[t] = use ? -(A.p[t] - c0 * A.q[t] - c1 * A.s[t]) : -A.p[t];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        A.info[0] = use ? 1.0 : 0.0;
        A.info[1] = ys_out;
    }
}

}  // namespace regot
