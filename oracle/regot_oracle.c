/*
 * regot_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, fp64 CPU statement of what the dense streaming pass of the
 * entropic-OT dual computes.  It exists so that the GPU library can be checked
 * against something written independently from the paper's formulas.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it; the
 * GPU library shares no code, header, table or constant with this file.
 *
 * Every function is the definition written out (the method is exact, there is
 * no approximation to follow step by step):
 *
 *   plan entry      T_ij = exp{ (alpha_i + beta_j - M_ij) / eta }      Sec. 3.1
 *   dual objective  L = -eta * sum_ij T_ij + alpha^T a + beta^T b      Sec. 1, display after eq. (3)
 *   gradient of L   (a - T 1_m ,  b - T^T 1_n)                         Sec. 3.1 (the paper prints grad f = -grad L)
 *   sparsified plan T^Omega keeps T_ij on Omega, zero elsewhere        Sec. 3.1, eq. (7)
 *   Omega           positions of the k largest entries of T            Sec. 3.1 (top-k rule)
 *   Sinkhorn        exact block-coordinate ascent on L                 Sec. 1 (paragraph after eq. (3))
 *   sparse term     H_Omega of the quasi-Newton matrix, its product    Sec. 3.1, eq. (7); eq. (6) (v = (H_Omega + tau I) s)
 *                   with a vector and its lower triangle by columns
 *   stored pattern  values recomputed on a pattern kept from before    Sec. 4.2
 *
 * Conventions fixed here where the paper is silent:
 *   - M is row-major with leading dimension ldM >= m; everything is fp64.
 *   - the argument of exp is formed as ((alpha_i + beta_j) - M_ij) / eta, in
 *     that association order, with one rounding per operation (the build
 *     forbids contraction into fused multiply-adds).
 *   - sums are accumulated in long double (64-bit mantissa on x86-64), rows in
 *     ascending j, columns in ascending i.
 *   - an entry belongs to the threshold pattern iff T_ij >= delta; CSR columns
 *     are 0-based and strictly ascending inside a row; row_ptr is int64.
 *   - a half-step maximises L exactly in one block of variables:
 *       d L / d alpha_i = a_i - sum_j T_ij = 0
 *         <=>  alpha_i = eta*log a_i - eta*log sum_j exp{(beta_j - M_ij)/eta}
 *     (and the mirror image for beta_j), evaluated as a two-pass,
 *     max-subtracted log-sum-exp so that small eta cannot underflow the sum.
 *
 * OpenMP only splits independent rows / column ranges between threads; the
 * per-thread column partials of dual_eval are merged in thread order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <omp.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ALLOC (-1)
#define ORACLE_ERR_ARG (-2)

/* T_ij as defined in Sec. 3.1; the one place the plan entry is computed. */
static double plan_entry(double alpha_i, double beta_j, double M_ij, double eta)
{
    double s = (alpha_i + beta_j) - M_ij;
    double x = s / eta;
    return exp(x);
}

void oracle_set_threads(int threads)
{
    if (threads > 0) omp_set_num_threads(threads);
}

int oracle_get_max_threads(void)
{
    return omp_get_max_threads();
}

/* Dense T (row-major, leading dimension m).  For small checks only. */
int oracle_plan_dense(int64_t n, int64_t m, const double *M, int64_t ldM,
                      const double *alpha, const double *beta, double eta,
                      double *T)
{
    if (n < 0 || m < 0 || ldM < m) return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < m; ++j)
            T[i * m + j] = plan_entry(alpha[i], beta[j], M[i * ldM + j], eta);
    return ORACLE_OK;
}

/*
 * L(alpha,beta), its gradient (a - T1, b - T^T 1), and the row / column sums
 * of T themselves.  Any output pointer may be NULL.
 */
int oracle_dual_eval(int64_t n, int64_t m, const double *M, int64_t ldM,
                     const double *a, const double *b,
                     const double *alpha, const double *beta, double eta,
                     double *obj, double *grad_alpha, double *grad_beta,
                     double *row_sum, double *col_sum)
{
    if (n < 0 || m < 0 || ldM < m) return ORACLE_ERR_ARG;
    int nthreads = omp_get_max_threads();
    long double *colacc = (long double *)calloc((size_t)nthreads * (size_t)(m > 0 ? m : 1), sizeof(long double));
    long double *rowacc = (long double *)calloc((size_t)(n > 0 ? n : 1), sizeof(long double));
    if (!colacc || !rowacc) { free(colacc); free(rowacc); return ORACLE_ERR_ALLOC; }

#pragma omp parallel num_threads(nthreads)
    {
        int t = omp_get_thread_num();
        int nt = omp_get_num_threads();
        /* contiguous block of rows per thread */
        int64_t lo = (n * t) / nt, hi = (n * (t + 1)) / nt;
        long double *cacc = colacc + (size_t)t * (size_t)m;
        for (int64_t i = lo; i < hi; ++i) {
            long double r = 0.0L;
            for (int64_t j = 0; j < m; ++j) {
                double T = plan_entry(alpha[i], beta[j], M[i * ldM + j], eta);
                r += (long double)T;
                cacc[j] += (long double)T;
            }
            rowacc[i] = r;
        }
    }

    long double S = 0.0L, dot_a = 0.0L, dot_b = 0.0L;
    for (int64_t i = 0; i < n; ++i) {
        S += rowacc[i];
        dot_a += (long double)alpha[i] * (long double)a[i];
        double r = (double)rowacc[i];
        if (row_sum) row_sum[i] = r;
        if (grad_alpha) grad_alpha[i] = (double)((long double)a[i] - rowacc[i]);
    }
    for (int64_t j = 0; j < m; ++j) {
        long double c = 0.0L;
        for (int t = 0; t < nthreads; ++t) c += colacc[(size_t)t * (size_t)m + j];
        dot_b += (long double)beta[j] * (long double)b[j];
        if (col_sum) col_sum[j] = (double)c;
        if (grad_beta) grad_beta[j] = (double)((long double)b[j] - c);
    }
    if (obj) *obj = (double)(-(long double)eta * S + dot_a + dot_b);
    free(colacc);
    free(rowacc);
    return ORACLE_OK;
}

/*
 * Threshold pattern, step 1: row_ptr[0..n] with row_ptr[i+1]-row_ptr[i] =
 * #{j : T_ij >= delta}.  Returns nnz in *nnz.
 */
int oracle_sparsify_count(int64_t n, int64_t m, const double *M, int64_t ldM,
                          const double *alpha, const double *beta, double eta,
                          double delta, int64_t *row_ptr, int64_t *nnz)
{
    if (n < 0 || m < 0 || ldM < m || !row_ptr) return ORACLE_ERR_ARG;
    row_ptr[0] = 0;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int64_t cnt = 0;
        for (int64_t j = 0; j < m; ++j)
            if (plan_entry(alpha[i], beta[j], M[i * ldM + j], eta) >= delta) ++cnt;
        row_ptr[i + 1] = cnt;
    }
    for (int64_t i = 0; i < n; ++i) row_ptr[i + 1] += row_ptr[i];
    if (nnz) *nnz = row_ptr[n];
    return ORACLE_OK;
}

/* Threshold pattern, step 2: fill col_idx / val at the offsets of step 1. */
int oracle_sparsify_fill(int64_t n, int64_t m, const double *M, int64_t ldM,
                         const double *alpha, const double *beta, double eta,
                         double delta, const int64_t *row_ptr,
                         int32_t *col_idx, double *val)
{
    if (n < 0 || m < 0 || ldM < m || !row_ptr) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int64_t p = row_ptr[i];
        for (int64_t j = 0; j < m; ++j) {
            double T = plan_entry(alpha[i], beta[j], M[i * ldM + j], eta);
            if (T >= delta) {
                col_idx[p] = (int32_t)j;
                val[p] = T;
                ++p;
            }
        }
    }
    return ORACLE_OK;
}

/*
 * One exact block maximisation of L.
 *   which == 0:  out[i] = eta*log a_i - eta*LSE_j{(beta_j - M_ij)/eta}, i < n
 *   which == 1:  out[j] = eta*log b_j - eta*LSE_i{(alpha_i - M_ij)/eta}, j < m
 * LSE is evaluated with the maximum subtracted (pass 1: max, pass 2: sum).
 * `marginal` is a for which == 0 and b for which == 1.  `out` must not alias
 * alpha or beta.
 */
int oracle_sinkhorn_half_step(int64_t n, int64_t m, const double *M, int64_t ldM,
                              const double *marginal,
                              const double *alpha, const double *beta, double eta,
                              int which, double *out)
{
    if (n < 0 || m < 0 || ldM < m || !out) return ORACLE_ERR_ARG;
    if (which == 0) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < n; ++i) {
            double mx = -INFINITY;
            for (int64_t j = 0; j < m; ++j) {
                double x = (beta[j] - M[i * ldM + j]) / eta;
                if (x > mx) mx = x;
            }
            long double sum = 0.0L;
            for (int64_t j = 0; j < m; ++j) {
                double x = (beta[j] - M[i * ldM + j]) / eta;
                sum += (long double)exp(x - mx);
            }
            double lse = mx + log((double)sum);
            out[i] = eta * log(marginal[i]) - eta * lse;
        }
        return ORACLE_OK;
    }
    if (which == 1) {
        int err = 0;
#pragma omp parallel
        {
            int t = omp_get_thread_num();
            int nt = omp_get_num_threads();
            /* contiguous range of columns per thread; rows in ascending order */
            int64_t lo = (m * t) / nt, hi = (m * (t + 1)) / nt;
            int64_t w = hi - lo;
            double *mx = (double *)malloc((size_t)(w > 0 ? w : 1) * sizeof(double));
            long double *sum = (long double *)malloc((size_t)(w > 0 ? w : 1) * sizeof(long double));
            if (!mx || !sum) {
#pragma omp atomic write
                err = 1;
            } else {
                for (int64_t j = 0; j < w; ++j) { mx[j] = -INFINITY; sum[j] = 0.0L; }
                for (int64_t i = 0; i < n; ++i)
                    for (int64_t j = lo; j < hi; ++j) {
                        double x = (alpha[i] - M[i * ldM + j]) / eta;
                        if (x > mx[j - lo]) mx[j - lo] = x;
                    }
                for (int64_t i = 0; i < n; ++i)
                    for (int64_t j = lo; j < hi; ++j) {
                        double x = (alpha[i] - M[i * ldM + j]) / eta;
                        sum[j - lo] += (long double)exp(x - mx[j - lo]);
                    }
                for (int64_t j = lo; j < hi; ++j) {
                    double lse = mx[j - lo] + log((double)sum[j - lo]);
                    out[j] = eta * log(marginal[j]) - eta * lse;
                }
            }
            free(mx);
            free(sum);
        }
        return err ? ORACLE_ERR_ALLOC : ORACLE_OK;
    }
    return ORACLE_ERR_ARG;
}

/* ---- k-th largest entry of T without storing T ------------------------- */

static int cmp_desc(const void *pa, const void *pb)
{
    double x = *(const double *)pa, y = *(const double *)pb;
    return (x < y) - (x > y);
}

/* T >= 0, so the IEEE bit pattern is monotone in the value. */
static uint32_t top_bits(double T)
{
    uint64_t u;
    memcpy(&u, &T, sizeof u);
    return (uint32_t)(u >> 44); /* sign(0) + 11 exponent + 8 mantissa bits */
}

#define NBUCKET (1u << 20)

/*
 * delta = the k-th largest T_ij (1 <= k <= n*m), so that #{T_ij >= delta} >= k
 * with equality when the k-th and (k+1)-th largest differ.
 * Pass 1 histograms the leading bits of every T_ij; pass 2 gathers the bucket
 * that holds rank k, sorts it and picks the entry.  NaN entries are not
 * supported.
 */
int oracle_topk_threshold(int64_t n, int64_t m, const double *M, int64_t ldM,
                          const double *alpha, const double *beta, double eta,
                          int64_t k, double *delta)
{
    if (n <= 0 || m <= 0 || ldM < m || k < 1 || k > n * m || !delta) return ORACLE_ERR_ARG;
    int64_t *hist = (int64_t *)calloc(NBUCKET, sizeof(int64_t));
    if (!hist) return ORACLE_ERR_ALLOC;
    int err = 0;
#pragma omp parallel
    {
        int64_t *h = (int64_t *)calloc(NBUCKET, sizeof(int64_t));
        if (!h) {
#pragma omp atomic write
            err = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t i = 0; i < n; ++i)
                for (int64_t j = 0; j < m; ++j)
                    h[top_bits(plan_entry(alpha[i], beta[j], M[i * ldM + j], eta))]++;
#pragma omp critical
            for (uint32_t q = 0; q < NBUCKET; ++q) hist[q] += h[q];
        }
        free(h);
    }
    if (err) { free(hist); return ORACLE_ERR_ALLOC; }

    int64_t above = 0;
    uint32_t bucket = NBUCKET - 1;
    for (;; --bucket) {
        if (above + hist[bucket] >= k) break;
        above += hist[bucket];
        if (bucket == 0) { free(hist); return ORACLE_ERR_ARG; }
    }
    int64_t cnt = hist[bucket];
    free(hist);
    double *buf = (double *)malloc((size_t)cnt * sizeof(double));
    if (!buf) return ORACLE_ERR_ALLOC;
    int64_t fill = 0;
    /* gather order does not matter: the bucket is sorted afterwards */
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < m; ++j) {
            double T = plan_entry(alpha[i], beta[j], M[i * ldM + j], eta);
            if (top_bits(T) == bucket) {
                int64_t slot;
#pragma omp atomic capture
                slot = fill++;
                buf[slot] = T;
            }
        }
    qsort(buf, (size_t)cnt, sizeof(double), cmp_desc);
    *delta = buf[k - above - 1];
    free(buf);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------
 * The sparse term of the quasi-Newton matrix (Sec. 3.1, eq. (7)) on a stored
 * pattern (Sec. 4.2: the pattern is kept for S iterations, only the values of
 * its entries are recomputed).
 *
 *   x = (x_alpha[n], x_beta[m-1])   -- the last dual variable beta_m is fixed
 *
 *   H_Omega = (1/eta) [ diag(T 1_m)           T^Omega_{-m}          ]
 *                     [ (T^Omega_{-m})^T      diag(T_{-m}^T 1_n)    ]
 *
 * T^Omega keeps T_ij on the pattern and is zero elsewhere; "-m" drops the last
 * column (0-based column m-1), so pattern entries in that column do not enter.
 * The diagonal blocks use the FULL row sums r = T 1_m and column sums
 * c = T^T 1_n (first m-1 of them), which are inputs here.
 * The pattern comes as CSR over all m columns (0-based, ascending columns).
 * ---------------------------------------------------------------------- */

/* val[p] = T_{i, col_idx[p]} for every entry p of row i of the pattern. */
int oracle_pattern_values(int64_t n, int64_t m, const double *M, int64_t ldM,
                          const double *alpha, const double *beta, double eta,
                          const int64_t *row_ptr, const int32_t *col_idx, double *val)
{
    if (n < 0 || m < 0 || ldM < m) return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            int64_t j = col_idx[p];
            if (j < 0 || j >= m) return ORACLE_ERR_ARG;
            val[p] = plan_entry(alpha[i], beta[j], M[i * ldM + j], eta);
        }
    return ORACLE_OK;
}

/* The pattern by columns: col_ptr[m+1]; row_idx[q] ascending inside a column;
 * csc_pos[p] = position q of CSR entry p in that order. */
int oracle_pattern_transpose(int64_t n, int64_t m, const int64_t *row_ptr, const int32_t *col_idx,
                             int64_t *col_ptr, int32_t *row_idx, int64_t *csc_pos)
{
    if (n < 0 || m < 0) return ORACLE_ERR_ARG;
    for (int64_t j = 0; j <= m; ++j) col_ptr[j] = 0;
    for (int64_t p = 0; p < row_ptr[n]; ++p) col_ptr[col_idx[p] + 1]++;
    for (int64_t j = 0; j < m; ++j) col_ptr[j + 1] += col_ptr[j];
    int64_t *next = (int64_t *)malloc((size_t)(m > 0 ? m : 1) * sizeof(int64_t));
    if (!next) return ORACLE_ERR_ALLOC;
    for (int64_t j = 0; j < m; ++j) next[j] = col_ptr[j];
    for (int64_t i = 0; i < n; ++i)            /* rows in ascending order: so are the rows of a column */
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            int64_t q = next[col_idx[p]]++;
            row_idx[q] = (int32_t)i;
            csc_pos[p] = q;
        }
    free(next);
    return ORACLE_OK;
}

/* y = (H_Omega + tau I) x, x and y of length n + m - 1. */
int oracle_hessian_matvec(int64_t n, int64_t m, double eta, double tau,
                          const int64_t *row_ptr, const int32_t *col_idx, const double *val,
                          const double *row_sum, const double *col_sum,
                          const double *x, double *y)
{
    if (n < 1 || m < 1 || !(eta > 0.0)) return ORACLE_ERR_ARG;
    const int64_t mb = m - 1;                    /* beta variables in x */
    long double *acc = (long double *)calloc((size_t)(mb > 0 ? mb : 1), sizeof(long double));
    if (!acc) return ORACLE_ERR_ALLOC;
    for (int64_t i = 0; i < n; ++i) {
        long double s = (long double)row_sum[i] * x[i];
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            int64_t j = col_idx[p];
            if (j >= mb) continue;               /* the dropped column */
            s += (long double)val[p] * x[n + j];
            acc[j] += (long double)val[p] * x[i];
        }
        y[i] = (double)(s / eta + (long double)tau * x[i]);
    }
    for (int64_t j = 0; j < mb; ++j) {
        long double s = acc[j] + (long double)col_sum[j] * x[n + j];
        y[n + j] = (double)(s / eta + (long double)tau * x[n + j]);
    }
    free(acc);
    return ORACLE_OK;
}

/* H_Omega + tau I as a dense (n+m-1) x (n+m-1) row-major matrix; small sizes only. */
int oracle_hessian_dense(int64_t n, int64_t m, double eta, double tau,
                         const int64_t *row_ptr, const int32_t *col_idx, const double *val,
                         const double *row_sum, const double *col_sum, double *H)
{
    if (n < 1 || m < 1 || !(eta > 0.0)) return ORACLE_ERR_ARG;
    const int64_t N = n + m - 1;
    memset(H, 0, (size_t)(N * N) * sizeof(double));
    for (int64_t i = 0; i < n; ++i) {
        H[i * N + i] = row_sum[i] / eta + tau;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            int64_t j = col_idx[p];
            if (j >= m - 1) continue;
            H[i * N + (n + j)] = val[p] / eta;
            H[(n + j) * N + i] = val[p] / eta;
        }
    }
    for (int64_t j = 0; j < m - 1; ++j) H[(n + j) * N + (n + j)] = col_sum[j] / eta + tau;
    return ORACLE_OK;
}

/* Lower triangle of H_Omega + tau I in compressed-column form, the input of a
 * sparse Cholesky factorisation (Sec. 3.2): column i < n holds its diagonal and
 * the entries of row i of T^Omega_{-m} (as rows n + j, ascending); column n + j
 * holds its diagonal only.  h_col_ptr has n + m entries.  With h_row_idx == NULL
 * only h_col_ptr is written (so the caller can size the arrays). */
int oracle_hessian_lower_csc(int64_t n, int64_t m, double eta, double tau,
                             const int64_t *row_ptr, const int32_t *col_idx, const double *val,
                             const double *row_sum, const double *col_sum,
                             int64_t *h_col_ptr, int32_t *h_row_idx, double *h_val)
{
    if (n < 1 || m < 1 || !(eta > 0.0)) return ORACLE_ERR_ARG;
    int64_t q = 0;
    for (int64_t i = 0; i < n; ++i) {
        h_col_ptr[i] = q;
        if (h_row_idx) {
            h_row_idx[q] = (int32_t)i;
            h_val[q] = row_sum[i] / eta + tau;
        }
        ++q;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            int64_t j = col_idx[p];
            if (j >= m - 1) continue;
            if (h_row_idx) {
                h_row_idx[q] = (int32_t)(n + j);
                h_val[q] = val[p] / eta;
            }
            ++q;
        }
    }
    for (int64_t j = 0; j < m - 1; ++j) {
        h_col_ptr[n + j] = q;
        if (h_row_idx) {
            h_row_idx[q] = (int32_t)(n + j);
            h_val[q] = col_sum[j] / eta + tau;
        }
        ++q;
    }
    h_col_ptr[n + m - 1] = q;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------
 * Optimality measures of a dual point (App. A.5) and the candidate choice of
 * Sec. 4.3.
 *
 *   primal value    L_p = <T, M> + eta * sum T log T - eta * sum T      (direct definition; 0 log 0 = 0)
 *   dual value      L_d = -eta * sum T + alpha^T a + beta^T b
 *   duality gap     L_p - L_d
 *   marginal error  || T 1 - a ||_1 + || T^T 1 - b ||_1
 *   gradient norm   || grad f ||_2 over x = (alpha, beta_1..beta_{m-1})  (Sec. 3.1; Algorithm 1 uses it for tau)
 *
 * out[0] = L_p, out[1] = L_p - L_d, out[2] = marginal error, out[3] = || grad f ||_2.
 * log T_ij is taken as (alpha_i + beta_j - M_ij)/eta, the exponent itself.
 * ---------------------------------------------------------------------- */
int oracle_dual_metrics(int64_t n, int64_t m, const double *M, int64_t ldM,
                        const double *a, const double *b,
                        const double *alpha, const double *beta, double eta, double *out)
{
    if (n < 0 || m < 0 || ldM < m || !out) return ORACLE_ERR_ARG;
    long double *col = (long double *)calloc((size_t)(m > 0 ? m : 1), sizeof(long double));
    if (!col) return ORACLE_ERR_ALLOC;
    long double tm = 0.0L, tlogt = 0.0L, tsum = 0.0L, aa = 0.0L, bb = 0.0L, merr = 0.0L, g2 = 0.0L;
    for (int64_t i = 0; i < n; ++i) {
        long double r = 0.0L;
        for (int64_t j = 0; j < m; ++j) {
            double s = (alpha[i] + beta[j]) - M[i * ldM + j];
            double x = s / eta;
            double T = exp(x);
            r += T;
            col[j] += T;
            tm += (long double)T * M[i * ldM + j];
            if (T > 0.0) tlogt += (long double)T * x;
        }
        tsum += r;
        aa += (long double)alpha[i] * a[i];
        merr += fabsl(r - a[i]);
        g2 += (r - a[i]) * (r - a[i]);
    }
    for (int64_t j = 0; j < m; ++j) {
        bb += (long double)beta[j] * b[j];
        merr += fabsl(col[j] - b[j]);
        if (j < m - 1) g2 += (col[j] - b[j]) * (col[j] - b[j]);
    }
    free(col);
    long double Lp = tm + (long double)eta * tlogt - (long double)eta * tsum;
    long double Ld = -(long double)eta * tsum + aa + bb;
    out[0] = (double)Lp;
    out[1] = (double)(Lp - Ld);
    out[2] = (double)merr;
    out[3] = (double)sqrtl(g2);
    return ORACLE_OK;
}
