// Streaming kernels over the cost matrix M (gfx950).
//
// Work decomposition (all stage-1 kernels): the n x m matrix is cut into column
// panels of kPanel = 512 columns and row chunks of `rows_per_chunk` rows.  One
// workgroup (4 waves) owns one (row chunk, panel) pair for its whole life.  Inside
// a panel a lane owns 8 fixed columns (4 x 16-byte loads per row, lanes adjacent in
// memory), so column reductions stay in the lane's registers for all rows of the
// chunk and only row reductions cross lanes.  Waves take groups of kRB = 4 rows
// round-robin.  Each matrix entry is read once and nothing is accumulated with
// floating-point atomics: partial results go to a workspace and a small second
// kernel combines them in a fixed order.
//
// This replaces the tiling of the paper's fused gradient kernel (Sec. 4.4: 32 x D
// thread blocks, one column per thread, shuffle tree per 32-column segment, shared-
// memory atomics for the column sums): the same single-read fusion, re-cut for
// 64-wide waves and 128-bit loads.
#pragma once

#include <type_traits>

#include "regot_device.hpp"

namespace regot {

// ints at the start of the workspace
enum { HDR_POOL_NEXT = 0, HDR_TICKET = 1, HDR_POOL_OVERFLOW = 2, HDR_INTS = 64 };

struct Stage1Args {
    int n, m;
    int64_t ldM;
    const double *M;
    const double *alpha;
    const double *beta;
    int g_c;             // number of column panels
    int rows_per_chunk;  // rows per row chunk (multiple of kRB * kWaves)
    double *rowpart;     // [g_c][n]   (LSE kernels: [g_c][n][2])
    double *colpart;     // [g_r][m]   (LSE kernels: [g_r][m][2])
    // sparsify
    double delta;
    int *seg_count;      // [g_c][n]: entries >= delta of row i inside panel p
    int *header;
    int pool_chunks;
    int *chunk_used;     // [pool_chunks]
    int2 *pool_rc;       // [pool_chunks * kChunk] (row, column)
    double *pool_val;    // [pool_chunks * kChunk]
    int *pool_rank;      // [pool_chunks * kChunk] rank of the record inside its (row, panel) segment
    ExpParams ex;
};

__global__ void init_header_kernel(int *header)
{
    if (threadIdx.x < HDR_INTS) header[threadIdx.x] = 0;
}

// Per-wave cursor into the staging pool of selected entries.
struct EmitState {
    int chunk;  // -1: none yet
    int used;
};

// Stage the entries of one (row, panel) segment that passed the threshold.
// mk[u][e]: wave-wide hit masks.  Records of a segment are contiguous in the pool and
// carry their rank in ascending column order, so the scatter kernel can place each
// one independently of where in the pool it landed.
__device__ __forceinline__ void emit_segment(const Stage1Args &A, EmitState &st, int lane, int row, int col0,
                                             const uint64_t (&mk)[kU][2], const double (&T)[kU][2], int cnt)
{
    if (st.chunk < 0 || st.used + cnt > kChunk) {
        int c = 0;
        if (lane == 0) {
            if (st.chunk >= 0) A.chunk_used[st.chunk] = st.used;
            c = atomicAdd(&A.header[HDR_POOL_NEXT], 1);
        }
        c = __builtin_amdgcn_readfirstlane(c);
        st.used = 0;
        if (c >= A.pool_chunks) {
            if (lane == 0) A.header[HDR_POOL_OVERFLOW] = 1;
            st.chunk = -1;
            return;
        }
        st.chunk = c;
    }
    const int64_t base = (int64_t)st.chunk * kChunk + st.used;
    int off = 0;
#pragma unroll
    for (int u = 0; u < kU; ++u) {
        const uint64_t m0 = mk[u][0], m1 = mk[u][1];
        if ((m0 | m1) != 0) {
            const int below = lanes_below(m0) + lanes_below(m1);
            const bool h0 = (m0 >> lane) & 1, h1 = (m1 >> lane) & 1;
            const int c = col0 + u * (2 * kLanes) + 2 * lane;
            if (h0) {
                const int rk = off + below;
                A.pool_rc[base + rk] = make_int2(row, c);
                A.pool_val[base + rk] = T[u][0];
                A.pool_rank[base + rk] = rk;
            }
            if (h1) {
                const int rk = off + below + (h0 ? 1 : 0);
                A.pool_rc[base + rk] = make_int2(row, c + 1);
                A.pool_val[base + rk] = T[u][1];
                A.pool_rank[base + rk] = rk;
            }
        }
        off += __builtin_popcountll(m0) + __builtin_popcountll(m1);
    }
    st.used += cnt;
}

// ---------------------------------------------------------------------------
// Fused pass: plan entries -> row partials, column partials, threshold hits.
// REDUCE: produce row / column partial sums.  SPARSIFY: count and stage T_ij >= delta.
// ---------------------------------------------------------------------------
template <bool REDUCE, bool SPARSIFY, bool ALIGNED, bool FULL>
__device__ __forceinline__ void plan_pass(const Stage1Args &A, double (*lds_col)[kPanel])
{
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int p = blockIdx.x % A.g_c;
    const int g = blockIdx.x / A.g_c;
    const int col0 = p * kPanel;
    const int ncol = min(kPanel, A.m - col0);
    const int r_begin = g * A.rows_per_chunk;
    const int r_end = min(A.n, r_begin + A.rows_per_chunk);

    bool cv[kU][2];
    double bet[kU][2];
    double cacc[kU][2];
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int c = u * (2 * kLanes) + 2 * lane + e;
            cv[u][e] = FULL || c < ncol;
            bet[u][e] = cv[u][e] ? A.beta[col0 + c] : 0.0;
            cacc[u][e] = 0.0;
        }
    const double *Mlane = A.M + col0 + 2 * lane;
    EmitState st{-1, 0};

    auto one_row = [&](int row, double al, const double (&v)[kU][2]) {
        double T[kU][2];
        double racc = 0.0;
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const double s = (al + bet[u][e]) - v[u][e];
                double t = exp_eta(s, A.ex);
                if constexpr (!FULL) t = cv[u][e] ? t : 0.0;
                T[u][e] = t;
                if constexpr (REDUCE) {
                    racc += t;
                    cacc[u][e] += t;
                }
            }
        if constexpr (REDUCE) {
            const double rs = wave_sum(racc);
            if (lane == 0) A.rowpart[(size_t)p * A.n + row] = rs;
        }
        if constexpr (SPARSIFY) {
            uint64_t mk[kU][2];
            int cnt = 0;
#pragma unroll
            for (int u = 0; u < kU; ++u)
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    bool hit = T[u][e] >= A.delta;
                    if constexpr (!FULL) hit = hit && cv[u][e];
                    mk[u][e] = __ballot(hit);
                    cnt += __builtin_popcountll(mk[u][e]);
                }
            if (lane == 0) A.seg_count[(size_t)p * A.n + row] = cnt;
            if (cnt > 0) emit_segment(A, st, lane, row, col0, mk, T, cnt);
        }
    };

    const int nrows = r_end - r_begin;
    const int ngroups = nrows / kRB;
    for (int q = w; q < ngroups; q += kWaves) {
        const int row0 = r_begin + q * kRB;
        double v[kRB][kU][2];
        load_rows<ALIGNED, FULL, kRB>(Mlane, A.ldM, row0, cv, v);
        double al[kRB];
#pragma unroll
        for (int r = 0; r < kRB; ++r) al[r] = A.alpha[row0 + r];
#pragma unroll
        for (int r = 0; r < kRB; ++r) one_row(row0 + r, al[r], v[r]);
    }
    // leftover rows (fewer than kRB), one at a time, spread over the waves
    for (int t = w; t < nrows - ngroups * kRB; t += kWaves) {
        const int row = r_begin + ngroups * kRB + t;
        double v[1][kU][2];
        load_rows<ALIGNED, FULL, 1>(Mlane, A.ldM, row, cv, v);
        one_row(row, A.alpha[row], v[0]);
    }
    if constexpr (SPARSIFY) {
        if (st.chunk >= 0 && lane == 0) A.chunk_used[st.chunk] = st.used;
    }
    if constexpr (REDUCE) {
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            lds_col[w][u * (2 * kLanes) + 2 * lane] = cacc[u][0];
            lds_col[w][u * (2 * kLanes) + 2 * lane + 1] = cacc[u][1];
        }
        __syncthreads();
        for (int c = threadIdx.x; c < ncol; c += kThreads) {
            double s = lds_col[0][c];
#pragma unroll
            for (int ww = 1; ww < kWaves; ++ww) s += lds_col[ww][c];
            A.colpart[(size_t)g * A.m + col0 + c] = s;
        }
    }
}

template <bool REDUCE, bool SPARSIFY, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void plan_pass_kernel(Stage1Args A)
{
    __shared__ double lds_col[REDUCE ? kWaves : 1][kPanel];
    const int p = blockIdx.x % A.g_c;
    if (A.m - p * kPanel >= kPanel)
        plan_pass<REDUCE, SPARSIFY, ALIGNED, true>(A, lds_col);
    else
        plan_pass<REDUCE, SPARSIFY, ALIGNED, false>(A, lds_col);
}

// ---------------------------------------------------------------------------
// Second stage of the fused pass: combine partials, objective, gradient, CSR offsets.
// ---------------------------------------------------------------------------
struct FinalizeArgs {
    int n, m, g_c, g_r;
    const double *rowpart;
    const double *colpart;
    const double *a, *b, *alpha, *beta;
    double eta;
    double *obj, *grad_alpha, *grad_beta, *row_sum, *col_sum;
    double *objpart;  // [gridDim.x][3]
    int nblk_rows;    // blocks [0, nblk_rows) own rows, the rest own columns
    int *header;
    int *seg_count;   // in: counts; out: exclusive prefix over panels inside the row
    int *row_nnz;     // [n]
    int64_t *row_ptr;
    int64_t capacity;
    int64_t *info;
};

// sum of one value per thread over the workgroup, fixed order, result valid in thread 0
__device__ __forceinline__ double block_sum(double v, double *lds /* [kThreads] */)
{
    lds[threadIdx.x] = v;
    __syncthreads();
    for (int s = kThreads / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) lds[threadIdx.x] += lds[threadIdx.x + s];
        __syncthreads();
    }
    double r = lds[0];
    __syncthreads();
    return r;
}

template <bool REDUCE, bool SPARSIFY>
__global__ __launch_bounds__(kThreads) void finalize_kernel(FinalizeArgs F)
{
    __shared__ double lds[kThreads];
    __shared__ long long lds_scan[kThreads];
    __shared__ int lds_flag;
    const int tid = threadIdx.x;
    double pS = 0.0, pA = 0.0, pB = 0.0;
    if ((int)blockIdx.x < F.nblk_rows) {
        const int64_t i = (int64_t)blockIdx.x * kThreads + tid;
        if (i < F.n) {
            if constexpr (REDUCE) {
                double r = 0.0;
                for (int p = 0; p < F.g_c; ++p) r += F.rowpart[(size_t)p * F.n + i];
                const double ai = F.a[i];
                if (F.row_sum) F.row_sum[i] = r;
                F.grad_alpha[i] = ai - r;
                pS = r;
                pA = F.alpha[i] * ai;
            }
            if constexpr (SPARSIFY) {
                int run = 0;
                for (int p = 0; p < F.g_c; ++p) {
                    const size_t k = (size_t)p * F.n + i;
                    const int c = F.seg_count[k];
                    F.seg_count[k] = run;
                    run += c;
                }
                F.row_nnz[i] = run;
            }
        }
    } else if constexpr (REDUCE) {
        const int64_t j = (int64_t)((int)blockIdx.x - F.nblk_rows) * kThreads + tid;
        if (j < F.m) {
            double c = 0.0;
            for (int g = 0; g < F.g_r; ++g) c += F.colpart[(size_t)g * F.m + j];
            const double bj = F.b[j];
            if (F.col_sum) F.col_sum[j] = c;
            F.grad_beta[j] = bj - c;
            pB = F.beta[j] * bj;
        }
    }
    if constexpr (REDUCE) {
        const double bS = block_sum(pS, lds), bA = block_sum(pA, lds), bB = block_sum(pB, lds);
        if (tid == 0) {
            F.objpart[(size_t)blockIdx.x * 3 + 0] = bS;
            F.objpart[(size_t)blockIdx.x * 3 + 1] = bA;
            F.objpart[(size_t)blockIdx.x * 3 + 2] = bB;
        }
    }
    // the workgroup that finishes last does the global epilogue
    __threadfence();
    __syncthreads();  // every thread's results are written and fenced before the ticket is taken
    if (tid == 0) {
        const int t = atomicAdd(&F.header[HDR_TICKET], 1);
        lds_flag = (t == (int)gridDim.x - 1);
    }
    __syncthreads();
    if (!lds_flag) return;
    __threadfence();
    if constexpr (REDUCE) {
        double S = 0.0, dA = 0.0, dB = 0.0;
        for (int k = tid; k < (int)gridDim.x; k += kThreads) {
            S += F.objpart[(size_t)k * 3 + 0];
            dA += F.objpart[(size_t)k * 3 + 1];
            dB += F.objpart[(size_t)k * 3 + 2];
        }
        S = block_sum(S, lds);
        dA = block_sum(dA, lds);
        dB = block_sum(dB, lds);
        if (tid == 0) *F.obj = -F.eta * S + (dA + dB);
    }
    if constexpr (SPARSIFY) {
        // exclusive scan of row_nnz -> row_ptr; each thread owns a contiguous range of rows
        const int64_t per = ((int64_t)F.n + kThreads - 1) / kThreads;
        const int64_t lo = min((int64_t)F.n, per * tid), hi = min((int64_t)F.n, per * (tid + 1));
        long long mine = 0;
        for (int64_t i = lo; i < hi; ++i) mine += F.row_nnz[i];
        lds_scan[tid] = mine;
        __syncthreads();
        if (tid == 0) {
            long long run = 0;
            for (int k = 0; k < kThreads; ++k) {
                const long long c = lds_scan[k];
                lds_scan[k] = run;
                run += c;
            }
            F.row_ptr[0] = 0;
            F.info[0] = run;
            F.info[1] = (run > F.capacity || F.header[HDR_POOL_OVERFLOW] != 0) ? 1 : 0;
        }
        __syncthreads();
        long long run = lds_scan[tid];
        for (int64_t i = lo; i < hi; ++i) {
            run += F.row_nnz[i];
            F.row_ptr[i + 1] = run;
        }
    }
}

// Place every staged record at its CSR position.
struct ScatterArgs {
    int n;
    const int *header;
    int pool_chunks;
    const int *chunk_used;
    const int2 *pool_rc;
    const double *pool_val;
    const int *pool_rank;
    const int *seg_rel;  // [g_c][n] exclusive prefix inside the row
    const int64_t *row_ptr;
    const int64_t *info;
    int32_t *col_idx;
    double *val;
};

__global__ __launch_bounds__(kThreads) void scatter_kernel(ScatterArgs S)
{
    if (S.info[1] != 0) return;
    const int n_alloc = min(S.header[HDR_POOL_NEXT], S.pool_chunks);
    for (int chunk = blockIdx.x; chunk < n_alloc; chunk += gridDim.x) {
        const int used = S.chunk_used[chunk];
        for (int k = threadIdx.x; k < used; k += kThreads) {
            const int64_t idx = (int64_t)chunk * kChunk + k;
            const int2 rc = S.pool_rc[idx];
            const int64_t dest =
                S.row_ptr[rc.x] + S.seg_rel[(size_t)(rc.y / kPanel) * S.n + rc.x] + S.pool_rank[idx];
            S.col_idx[dest] = rc.y;
            S.val[dest] = S.pool_val[idx];
        }
    }
}

// ---------------------------------------------------------------------------
// Sinkhorn half-steps in the log domain.  Quantities are kept in units of s
// (= eta * x): a partial log-sum-exp is the pair (smax, sum exp((s - smax)/eta)).
// ---------------------------------------------------------------------------

// which = 0: per row i, over the columns of one panel, s_ij = beta_j - M_ij.
template <bool ALIGNED, bool FULL>
__device__ __forceinline__ void row_lse_pass(const Stage1Args &A)
{
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int p = blockIdx.x % A.g_c;
    const int g = blockIdx.x / A.g_c;
    const int col0 = p * kPanel;
    const int ncol = min(kPanel, A.m - col0);
    const int r_begin = g * A.rows_per_chunk;
    const int r_end = min(A.n, r_begin + A.rows_per_chunk);

    bool cv[kU][2];
    double bet[kU][2];
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int c = u * (2 * kLanes) + 2 * lane + e;
            cv[u][e] = FULL || c < ncol;
            bet[u][e] = cv[u][e] ? A.beta[col0 + c] : 0.0;
        }
    const double *Mlane = A.M + col0 + 2 * lane;

    auto one_row = [&](int row, const double (&v)[kU][2]) {
        double s[kU][2];
        double lmax = -INFINITY;
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                s[u][e] = bet[u][e] - v[u][e];
                if (FULL || cv[u][e]) lmax = fmax(lmax, s[u][e]);
            }
        const double wmax = wave_max(lmax);  // finite: column col0 of the panel always exists
        double acc = 0.0;
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                double t = exp_eta(s[u][e] - wmax, A.ex);
                if constexpr (!FULL) t = cv[u][e] ? t : 0.0;
                acc += t;
            }
        const double wsum = wave_sum(acc);
        if (lane == 0) {
            const size_t k = ((size_t)p * A.n + row) * 2;
            A.rowpart[k] = wmax;
            A.rowpart[k + 1] = wsum;
        }
    };

    const int nrows = r_end - r_begin;
    const int ngroups = nrows / kRB;
    for (int q = w; q < ngroups; q += kWaves) {
        const int row0 = r_begin + q * kRB;
        double v[kRB][kU][2];
        load_rows<ALIGNED, FULL, kRB>(Mlane, A.ldM, row0, cv, v);
#pragma unroll
        for (int r = 0; r < kRB; ++r) one_row(row0 + r, v[r]);
    }
    for (int t = w; t < nrows - ngroups * kRB; t += kWaves) {
        const int row = r_begin + ngroups * kRB + t;
        double v[1][kU][2];
        load_rows<ALIGNED, FULL, 1>(Mlane, A.ldM, row, cv, v);
        one_row(row, v[0]);
    }
}

template <bool ALIGNED>
__global__ __launch_bounds__(kThreads) void row_lse_kernel(Stage1Args A)
{
    const int p = blockIdx.x % A.g_c;
    if (A.m - p * kPanel >= kPanel)
        row_lse_pass<ALIGNED, true>(A);
    else
        row_lse_pass<ALIGNED, false>(A);
}

// which = 1: per column j, over the rows of one chunk, s_ij = alpha_i - M_ij.
// Each lane carries a running (cmax, csum) per owned column; the sum is rescaled
// only in the rare groups of rows where some column's maximum moves.
template <bool ALIGNED, bool FULL>
__device__ __forceinline__ void col_lse_pass(const Stage1Args &A, double (*lds_max)[kPanel],
                                             double (*lds_sum)[kPanel])
{
    const int lane = threadIdx.x & (kLanes - 1);
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int p = blockIdx.x % A.g_c;
    const int g = blockIdx.x / A.g_c;
    const int col0 = p * kPanel;
    const int ncol = min(kPanel, A.m - col0);
    const int r_begin = g * A.rows_per_chunk;
    const int r_end = min(A.n, r_begin + A.rows_per_chunk);

    bool cv[kU][2];
    double cmax[kU][2], csum[kU][2];
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int c = u * (2 * kLanes) + 2 * lane + e;
            cv[u][e] = FULL || c < ncol;
            cmax[u][e] = 0.0;
            csum[u][e] = 0.0;  // csum == 0 marks "no row seen yet"
        }
    const double *Mlane = A.M + col0 + 2 * lane;
    bool first = true;

    auto group = [&](auto nr_tag, int row0) {
        constexpr int NR = decltype(nr_tag)::value;
        double v[NR][kU][2];
        load_rows<ALIGNED, FULL, NR>(Mlane, A.ldM, row0, cv, v);
        double al[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) al[r] = A.alpha[row0 + r];
        bool moved = false;
        double nmax[kU][2];
#pragma unroll
        for (int u = 0; u < kU; ++u)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                double mx = al[0] - v[0][u][e];
                v[0][u][e] = mx;
#pragma unroll
                for (int r = 1; r < NR; ++r) {
                    v[r][u][e] = al[r] - v[r][u][e];
                    mx = fmax(mx, v[r][u][e]);
                }
                if (!first) mx = fmax(mx, cmax[u][e]);
                nmax[u][e] = mx;
                moved = moved || (mx != cmax[u][e]);
            }
        if (first) {
#pragma unroll
            for (int u = 0; u < kU; ++u)
#pragma unroll
                for (int e = 0; e < 2; ++e) cmax[u][e] = nmax[u][e];
            first = false;
        } else if (__ballot(moved) != 0) {
#pragma unroll
            for (int u = 0; u < kU; ++u)
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    csum[u][e] *= exp_eta(cmax[u][e] - nmax[u][e], A.ex);  // exactly 1 where unchanged
                    cmax[u][e] = nmax[u][e];
                }
        }
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int u = 0; u < kU; ++u)
#pragma unroll
                for (int e = 0; e < 2; ++e) csum[u][e] += exp_eta(v[r][u][e] - cmax[u][e], A.ex);
    };

    const int nrows = r_end - r_begin;
    const int ngroups = nrows / kRB;
    for (int q = w; q < ngroups; q += kWaves) group(std::integral_constant<int, kRB>{}, r_begin + q * kRB);
    for (int t = w; t < nrows - ngroups * kRB; t += kWaves)
        group(std::integral_constant<int, 1>{}, r_begin + ngroups * kRB + t);

#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            lds_max[w][u * (2 * kLanes) + 2 * lane + e] = cmax[u][e];
            lds_sum[w][u * (2 * kLanes) + 2 * lane + e] = csum[u][e];
        }
    __syncthreads();
    for (int c = threadIdx.x; c < ncol; c += kThreads) {
        double mx = 0.0;
        bool any = false;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww)
            if (lds_sum[ww][c] > 0.0) {
                mx = any ? fmax(mx, lds_max[ww][c]) : lds_max[ww][c];
                any = true;
            }
        double sum = 0.0;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww)
            if (lds_sum[ww][c] > 0.0) sum += lds_sum[ww][c] * exp_eta(lds_max[ww][c] - mx, A.ex);
        const size_t k = ((size_t)g * A.m + col0 + c) * 2;
        A.colpart[k] = mx;
        A.colpart[k + 1] = sum;
    }
}

template <bool ALIGNED>
__global__ __launch_bounds__(kThreads) void col_lse_kernel(Stage1Args A)
{
    __shared__ double lds_max[kWaves][kPanel];
    __shared__ double lds_sum[kWaves][kPanel];
    const int p = blockIdx.x % A.g_c;
    if (A.m - p * kPanel >= kPanel)
        col_lse_pass<ALIGNED, true>(A, lds_max, lds_sum);
    else
        col_lse_pass<ALIGNED, false>(A, lds_max, lds_sum);
}

// Merge the partial (smax, sum) pairs of one row / column and finish the update:
// out = eta*log(marginal) - (smax + eta*log(sum)).
struct LseFinalizeArgs {
    int64_t len;        // n for which = 0, m for which = 1
    int parts;          // g_c for which = 0, g_r for which = 1
    const double *part; // [parts][len][2]
    const double *marginal;
    double eta;
    double *out;
    ExpParams ex;
};

__global__ __launch_bounds__(kThreads) void lse_finalize_kernel(LseFinalizeArgs L)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= L.len) return;
    double mx = 0.0;
    bool any = false;
    for (int q = 0; q < L.parts; ++q) {
        const size_t k = ((size_t)q * L.len + i) * 2;
        if (L.part[k + 1] > 0.0) {
            mx = any ? fmax(mx, L.part[k]) : L.part[k];
            any = true;
        }
    }
    double sum = 0.0;
    for (int q = 0; q < L.parts; ++q) {
        const size_t k = ((size_t)q * L.len + i) * 2;
        if (L.part[k + 1] > 0.0) sum += L.part[k + 1] * exp_eta(L.part[k] - mx, L.ex);
    }
    L.out[i] = L.eta * log(L.marginal[i]) - (mx + L.eta * log(sum));
}

}  // namespace regot
