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
#pragma once

#include "regot_sparse.hpp"

namespace regot {

constexpr int kPcgParts = 1024;   // most workgroups whose partial sums a later kernel adds up

struct PcgScalars {
    double rz;        // r^T z
    double bb;        // ||rhs||^2
    double rr;        // ||r||^2
    long long iters;
    int done;         // converged (or nothing to do)
    int pad;
};

struct PcgArgs {
    MatvecArgs mv;    // mv.x = p, mv.y = Ap
    int64_t N;
    const double *rhs;
    double *x, *r, *z, *p, *Ap;
    double *part;     // [3][kPcgParts]: p^T A p | r^T z | r^T r
    PcgScalars *sc;   // [2], alternating by iteration
    double rtol;
    int mv_blocks, vec_blocks;
    double *info;     // [4]: iterations, converged, ||r||, ||rhs||
};

__device__ __forceinline__ double pcg_diag(const MatvecArgs &M, int64_t t)
{
    return (t < M.n ? M.row_sum[t] : M.col_sum[t - M.n]) / M.eta + M.tau;
}

// sum of part[0 .. count) in a fixed order; every thread of the workgroup gets it
__device__ __forceinline__ double sum_parts(const double *part, int count, double *lds)
{
    double v = 0.0;
    for (int k = threadIdx.x; k < count; k += kThreads) v += part[k];
    return block_sum(v, lds);
}

// x = 0, r = rhs, z = r / diag, p = z; partial sums of r^T z and r^T r
__global__ __launch_bounds__(kThreads) void pcg_start_kernel(PcgArgs A)
{
    __shared__ double lds[kWaves];
    double rz = 0.0, rr = 0.0;
    for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < A.N; t += (int64_t)gridDim.x * kThreads) {
        const double r = A.rhs[t];
        const double z = r / pcg_diag(A.mv, t);
        A.x[t] = 0.0;
        A.r[t] = r;
        A.z[t] = z;
        A.p[t] = z;
        rz += r * z;
        rr += r * r;
    }
    rz = block_sum(rz, lds);
    rr = block_sum(rr, lds);
    if (threadIdx.x == 0) {
        A.part[kPcgParts + blockIdx.x] = rz;
        A.part[2 * kPcgParts + blockIdx.x] = rr;
    }
}

__global__ __launch_bounds__(kThreads) void pcg_start_scalars_kernel(PcgArgs A)
{
    __shared__ double lds[kWaves];
    const double rz = sum_parts(A.part + kPcgParts, A.vec_blocks, lds);
    const double rr = sum_parts(A.part + 2 * kPcgParts, A.vec_blocks, lds);
    if (threadIdx.x == 0) {
        PcgScalars s;
        s.rz = rz;
        s.bb = rr;
        s.rr = rr;
        s.iters = 0;
        s.done = rr == 0.0 ? 1 : 0;
        s.pad = 0;
        A.sc[0] = s;
    }
}

// x += step p, r -= step Ap, z = r / diag; partial sums of the new r^T z and r^T r
__global__ __launch_bounds__(kThreads) void pcg_update_kernel(PcgArgs A, int it)
{
    __shared__ double lds[kWaves];
    const PcgScalars cur = A.sc[it & 1];
    if (cur.done) return;
    const double pAp = sum_parts(A.part, A.mv_blocks, lds);
    const double step = cur.rz / pAp;
    double rz = 0.0, rr = 0.0;
    for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < A.N; t += (int64_t)gridDim.x * kThreads) {
        A.x[t] += step * A.p[t];
        const double r = A.r[t] - step * A.Ap[t];
        const double z = r / pcg_diag(A.mv, t);
        A.r[t] = r;
        A.z[t] = z;
        rz += r * z;
        rr += r * r;
    }
    rz = block_sum(rz, lds);
    rr = block_sum(rr, lds);
    if (threadIdx.x == 0) {
        A.part[kPcgParts + blockIdx.x] = rz;
        A.part[2 * kPcgParts + blockIdx.x] = rr;
    }
}

// p = z + (new r^T z / old r^T z) p; the scalars of the next iteration
__global__ __launch_bounds__(kThreads) void pcg_direction_kernel(PcgArgs A, int it)
{
    __shared__ double lds[kWaves];
    const PcgScalars cur = A.sc[it & 1];
    if (cur.done) {
        if (blockIdx.x == 0 && threadIdx.x == 0) A.sc[(it + 1) & 1] = cur;
        return;
    }
    const double rz = sum_parts(A.part + kPcgParts, A.vec_blocks, lds);
    const double rr = sum_parts(A.part + 2 * kPcgParts, A.vec_blocks, lds);
    const double ratio = rz / cur.rz;
    for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < A.N; t += (int64_t)gridDim.x * kThreads)
        A.p[t] = A.z[t] + ratio * A.p[t];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        PcgScalars nx = cur;
        nx.rz = rz;
        nx.rr = rr;
        nx.iters = cur.iters + 1;
        nx.done = rr <= A.rtol * A.rtol * cur.bb ? 1 : 0;
        A.sc[(it + 1) & 1] = nx;
    }
}

// after the last iteration of a call: the scalars go back to slot 0 (a later call continues from there)
__global__ void pcg_finish_kernel(PcgArgs A, int its)
{
    if (threadIdx.x != 0) return;
    const PcgScalars s = A.sc[its & 1];
    A.sc[0] = s;
    A.info[0] = (double)s.iters;
    A.info[1] = (double)s.done;
    A.info[2] = sqrt(s.rr);
    A.info[3] = sqrt(s.bb);
}

// ---------------------------------------------------------------------------------------------
// d = -B^{-1} g from p = A^{-1} g, q = A^{-1} y, s = s^- (= A^{-1} v), y = y^-, v = A s^-.
// One workgroup.  Without a previous step, or when (y^-)^T s^- <= 1e-6 ||y^-||^2 (Algorithm 1,
// line 5), R = 0 and d = -p.
// ---------------------------------------------------------------------------------------------
struct CombineArgs {
    int64_t N;
    const double *p, *q, *s, *y, *v;  // q, s, y, v may be NULL together: no previous step
    double *d;
    double *info;  // [2]: 1 if the rank-two term was used, (y^-)^T s^-
};

__global__ __launch_bounds__(kThreads) void splr_combine_kernel(CombineArgs A)
{
    __shared__ double lds[kWaves];
    bool use = A.s != nullptr;
    double c0 = 0.0, c1 = 0.0, ys_out = 0.0;
    if (use) {
        double ys = 0, yy = 0, yq = 0, vq = 0, vs = 0, yp = 0, vp = 0;
        for (int64_t t = threadIdx.x; t < A.N; t += kThreads) {
            const double y = A.y[t], s = A.s[t], v = A.v[t], q = A.q[t], p = A.p[t];
            ys += y * s;
            yy += y * y;
            yq += y * q;
            vq += v * q;
            vs += v * s;
            yp += y * p;
            vp += v * p;
        }
        ys = block_sum(ys, lds);
        yy = block_sum(yy, lds);
        yq = block_sum(yq, lds);
        vq = block_sum(vq, lds);
        vs = block_sum(vs, lds);
        yp = block_sum(yp, lds);
        vp = block_sum(vp, lds);
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
    for (int64_t t = threadIdx.x; t < A.N; t += kThreads)
        A.d[t] = use ? -(A.p[t] - c0 * A.q[t] - c1 * A.s[t]) : -A.p[t];
    if (threadIdx.x == 0) {
        A.info[0] = use ? 1.0 : 0.0;
        A.info[1] = ys_out;
    }
}

}  // namespace regot
