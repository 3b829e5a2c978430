/*
 * regot.h -- C ABI of the MI355X (gfx950) streaming kernels for the dual of
 * entropic-regularised optimal transport.
 *
 * Problem statement (Sec. 1): cost matrix M (n x m), probability vectors a (n)
 * and b (m), regularisation eta > 0, dual variables alpha (n), beta (m).
 * The dense calls (dual_eval, sparsify_csr, dual_eval_sparsify, sinkhorn_half_step)
 * make ONE streaming pass over M each and form the plan entry
 *
 *     T_ij = exp{ (alpha_i + beta_j - M_ij) / eta }              (Sec. 3.1)
 *
 * in registers; T is never stored.  Around them: the threshold that keeps k
 * entries (topk_threshold, normally one more pass over M; dual_eval_sparsify_topk
 * finds it inside the fused pass: one pass for both), and calls that work
 * on the sparse pattern only (pattern_*, hessian_*, pcg_solve, pcg_solve2, splr_direction)
 * or on vectors (dual_metrics, choose_candidate).
 *
 * Conventions common to all calls
 *   - All array arguments are DEVICE pointers (HBM of the current HIP device)
 *     unless the parameter comment says "host".  Everything is fp64; indices
 *     are int32 (columns) and int64 (row offsets).
 *   - M is row-major with leading dimension ldM >= m (in elements).  When M is
 *     16-byte aligned and ldM is even the kernels use 128-bit loads; otherwise
 *     a 64-bit-load variant runs (slower, same results).
 *   - The argument of exp is formed as ((alpha_i + beta_j) - M_ij), in that
 *     order, and divided by eta inside the exponential's range reduction.
 *   - Non-finite data is not an error and follows IEEE arithmetic, as a plain
 *     evaluation of the formulas with libm would: an infinite cost M_ij = +inf is a
 *     forbidden assignment, T_ij = exp(-inf) = 0 exactly, which adds nothing to any
 *     sum, is a pattern entry only for delta = 0 and is ignored by the half-steps
 *     (a row or column with no finite cost at all has no half-step update: NaN or
 *     +inf comes back for it); M_ij = -inf gives T_ij = +inf; a NaN makes every sum it
 *     contributes to (and the objective) NaN and never enters a pattern.  Finite
 *     inputs cost nothing extra for this: the kernels look again only at rows whose
 *     sum came out not finite.
 *   - Ownership: the caller owns every buffer, including `workspace`
 *     (regot_workspace_bytes() gives its size for the dense calls, the
 *     *_workspace_bytes function named at a call for that call; it must be
 *     256-byte aligned).
 *     The library allocates and frees no device memory and keeps no state that
 *     a result depends on.  (What it does keep: the event pair of
 *     regot_profile_stage1, per host thread, and the per-device address of the
 *     static workspace of regot_dual_eval_noalloc, looked up once.)  Inputs are
 *     never written.  Outputs must not overlap
 *     inputs or each other, except where a parameter comment allows it.
 *     Two calls that overlap in time must use different workspaces.
 *   - Asynchrony: a call validates its arguments on the host, enqueues its
 *     kernels on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and returns.  No host synchronisation happens inside; results,
 *     including scalars, stay on the device.
 *   - Errors: the return value is REGOT_OK or a negative REGOT_ERR_* code.
 *     Argument errors are detected before any HIP call, so nothing is
 *     enqueued.  REGOT_ERR_HIP reports a failed launch.
 *   - n = 0 or m = 0 is accepted by regot_dual_eval, regot_sparsify_csr and
 *     regot_dual_eval_sparsify (empty sums: T1 = 0, T^T1 = 0, empty CSR) and
 *     rejected by regot_sinkhorn_half_step (the update is undefined).
 */
#ifndef REGOT_H
#define REGOT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *regot_stream_t;

enum {
    REGOT_OK = 0,
    REGOT_ERR_NULL = -1,      /* a required pointer is NULL                         */
    REGOT_ERR_DIM = -2,       /* n or m negative, above 2^31-1, or zero where the
                                 operation is undefined                             */
    REGOT_ERR_ETA = -3,       /* eta not finite or not > 0                          */
    REGOT_ERR_LD = -4,        /* ldM < m                                            */
    REGOT_ERR_ALIGN = -5,     /* a pointer is not aligned to its element size, or
                                 the workspace is not 256-byte aligned              */
    REGOT_ERR_WORKSPACE = -6, /* workspace smaller than regot_workspace_bytes()     */
    REGOT_ERR_ARG = -7,       /* other invalid argument (which, capacity, delta NaN) */
    REGOT_ERR_HIP = -8,       /* a HIP call failed                                  */
    REGOT_ERR_SCRATCH = -9    /* regot_dual_eval_noalloc: the problem needs more
                                 workspace than REGOT_NOALLOC_MAX_WORKSPACE         */
};

/* Human-readable name of a status code; static storage, never NULL. */
const char *regot_status_string(int status);

/*
 * Size in bytes of the workspace any call below needs for an n x m problem.
 * csr_capacity is the `capacity` that will be passed to regot_sparsify_csr /
 * regot_dual_eval_sparsify, or -1 if only regot_dual_eval and
 * regot_sinkhorn_half_step will be called.  `bytes` is a host pointer.
 * The size depends only on (n, m, csr_capacity).
 */
int regot_workspace_bytes(int64_t n, int64_t m, int64_t csr_capacity, size_t *bytes /* host, out */);

/*
 * How the dense calls cut an n x m matrix into tasks (a host-side query; nothing runs on the device).
 * The streaming pass of Sec. 4.4 is run as g_r row chunks x g_c column panels of 512 columns, one
 * workgroup each, in `rounds` rounds of resident workgroups; csr_capacity as for
 * regot_workspace_bytes (-1: a call without sparsify).
 *     geometry[0] = g_r, [1] = g_c, [2] = rounds, [3] = rows of the tallest chunk,
 *     [4] = 0, or the number of extra workgroups that share a narrow last panel (at most 32 columns)
 *           (up to three row chunks each), while the g_r x (g_c - 1) tasks of the full panels fill the chip
 * The tallest chunk never exceeds 16384 rows (a staged CSR entry stores its row relative to its
 * chunk in 14 bits).  Results of the sums depend on (n, m, csr_capacity) only through this cut.
 * One round holds 1216 staged entries per wave, 2 490 368 in all: a capacity above that (or above a multiple of it)
 * costs another round, about a tenth of the pass at 20000 x 20000, so reserve what the pattern needs with a small
 * margin rather than a generous one.  (The candidate pass of regot_dual_eval_sparsify_topk runs in one round where
 * only the margin of its own capacity would ask for two.)
 */
int regot_plan_geometry(int64_t n, int64_t m, int64_t csr_capacity, int64_t *geometry /* host, [5] out */);

/*
 * Dual objective and gradient (Sec. 1, display after eq. (3); Sec. 3.1):
 *     obj        = L(alpha,beta) = -eta * sum_ij T_ij + alpha^T a + beta^T b
 *     grad_alpha = a - T 1_m        (the paper prints grad f = -grad L)
 *     grad_beta  = b - T^T 1_n      (full length m; the paper drops the last
 *                                    entry when it fixes beta_m = 0)
 *     row_sum    = T 1_m,  col_sum = T^T 1_n    (optional, may be NULL)
 * One pass over M (the fused gradient evaluation of Sec. 4.4); sums are
 * accumulated in a fixed order, so results are bit-reproducible run to run
 * (for the same sizes and, in the fused call, the same capacity: they set how
 * the matrix is cut into tasks, see regot_plan_geometry, i.e. the order in
 * which the sums add up).
 */
int regot_dual_eval(int64_t n, int64_t m,
                    const double *M, int64_t ldM,
                    const double *a, const double *b,          /* [n], [m] */
                    const double *alpha, const double *beta,   /* [n], [m] */
                    double eta,
                    double *obj,                               /* [1] out  */
                    double *grad_alpha, double *grad_beta,     /* [n], [m] out */
                    double *row_sum, double *col_sum,          /* [n], [m] out, optional */
                    void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * regot_dual_eval for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels
 * and results (bit for bit) as regot_dual_eval, minus the workspace: the partial sums live in a
 * static device array of REGOT_NOALLOC_MAX_WORKSPACE bytes that is part of the library's code
 * object (every GPU the library runs on holds its own copy until the process ends).  The call
 * allocates and frees nothing and calls no library routine that does.
 *   - Size limit: regot_workspace_bytes(n, m, -1) must not exceed REGOT_NOALLOC_MAX_WORKSPACE
 *     (it is about 16 (g_c n + g_r m) bytes, g_c = ceil(m / 512), g_r <= 2048 / g_c: 20000 x 20000
 *     and 40000 x 10000 fit, 50000 x 50000 does not); otherwise REGOT_ERR_SCRATCH, nothing enqueued.
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU
 *     (different streams or host threads) race.  Calls on one stream, or ordered by events, are safe.
 *     The array keeps what the last call left in it; no call depends on its contents.
 *   - The first call on each device looks up that device's copy of the array
 *     (hipGetSymbolAddress) and keeps the address; make that first call outside graph capture.
 */
#define REGOT_NOALLOC_MAX_WORKSPACE (32u << 20)
int regot_dual_eval_noalloc(int64_t n, int64_t m,
                            const double *M, int64_t ldM,
                            const double *a, const double *b,
                            const double *alpha, const double *beta,
                            double eta,
                            double *obj, double *grad_alpha, double *grad_beta,
                            double *row_sum, double *col_sum,   /* optional */
                            regot_stream_t stream);

/*
 * Threshold-sparsified plan as CSR (Sec. 3.1, eq. (7) and the top-k rule, in
 * threshold form): the pattern is Omega = {(i,j) : T_ij >= delta}.
 *     row_ptr[0..n]   int64, row_ptr[0] = 0, row_ptr[n] = nnz; always written
 *     col_idx[p]      int32, 0-based, strictly ascending inside each row
 *     val[p]          T_ij
 *     info[0]         nnz
 *     info[1]         0, or 1 if nnz > capacity (then col_idx / val hold
 *                     unspecified data; row_ptr and info[0] are still exact, so
 *                     the caller can re-run with a larger capacity)
 * All m columns are candidates (dropping column m, or forcing the first row
 * and column into Omega as the paper's theory assumes, is left to the caller).
 * One pass over M.  A call assembles at most 2^31 - 1 entries: beyond that
 * info[1] = 1 whatever the capacity (row_ptr and info[0] stay exact).
 */
int regot_sparsify_csr(int64_t n, int64_t m,
                       const double *M, int64_t ldM,
                       const double *alpha, const double *beta, double eta,
                       double delta,                            /* may be 0, +inf; not NaN */
                       int64_t *row_ptr,                        /* [n+1] out */
                       int32_t *col_idx, double *val,           /* [capacity] out */
                       int64_t capacity,                        /* >= 0 */
                       int64_t *info,                           /* [2] out */
                       void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * The fused pass: everything regot_dual_eval and regot_sparsify_csr produce,
 * from a single read of M (objective, gradient and pattern of one SPLR
 * iteration, Algorithm 1 lines 1-2).
 */
int regot_dual_eval_sparsify(int64_t n, int64_t m,
                             const double *M, int64_t ldM,
                             const double *a, const double *b,
                             const double *alpha, const double *beta,
                             double eta,
                             double *obj, double *grad_alpha, double *grad_beta,
                             double *row_sum, double *col_sum,  /* optional */
                             double delta,
                             int64_t *row_ptr, int32_t *col_idx, double *val,
                             int64_t capacity, int64_t *info,
                             void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * One Sinkhorn half-step = exact maximisation of L in one block of variables
 * (block coordinate ascent, Sec. 1; run as candidate generator in Sec. 4.3),
 * in the log domain:
 *   which = 0:  out[i] = eta*log a_i - eta*log sum_j exp{(beta_j  - M_ij)/eta},  i < n
 *   which = 1:  out[j] = eta*log b_j - eta*log sum_i exp{(alpha_i - M_ij)/eta},  j < m
 * `marginal` is a (length n) for which = 0 and b (length m) for which = 1.
 * The log-sum-exp is evaluated relative to the running maximum, so no term
 * overflows and the sum cannot underflow to zero.  Only the vector of the
 * other block is read (beta for which = 0, alpha for which = 1); the one
 * being replaced may be NULL, and `out` may alias it.  One pass over M.
 */
int regot_sinkhorn_half_step(int64_t n, int64_t m,
                             const double *M, int64_t ldM,
                             const double *marginal,
                             const double *alpha, const double *beta, double eta,
                             int which,
                             double *out,
                             void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * `sweeps` Sinkhorn sweeps in place: each is the alpha half-step followed by the beta half-step (the order
 * of the block coordinate ascent of Sec. 1; the candidate generator of Sec. 4.3 and the start of the
 * experiments in Sec. 6.1 run a fixed number of them).  alpha [n] and beta [m] are read and replaced;
 * the first half-step does not read alpha, so it need not be initialised.  2 * sweeps passes over M are
 * enqueued; exactly what the same sequence of regot_sinkhorn_half_step calls gives.  sweeps >= 0.
 */
int regot_sinkhorn_sweeps(int64_t n, int64_t m,
                          const double *M, int64_t ldM,
                          const double *a, const double *b,
                          double *alpha, double *beta, double eta,
                          int sweeps,
                          void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * Threshold of the top-k rule (Sec. 3.1: the pattern keeps the k largest entries of T): delta =
 * the k-th largest T_ij over all n x m entries, counted with multiplicity, so that
 * regot_sparsify_csr(..., delta, ...) keeps at least k entries, and exactly k when the k-th
 * largest entry is not tied.  T = exp(s / eta) is increasing in s_ij = (alpha_i + beta_j) - M_ij,
 * so the search runs on s (an exact radix selection on its bit pattern, no exponential) and
 *     delta[0] = exp(s_k / eta),   s_k = the k-th largest s_ij,
 * evaluated by the same exponential the other calls use.
 *     s_k[0]     s_k itself (optional, may be NULL)
 *     info[0]    number of entries with s_ij >  s_k   (< k)
 *     info[1]    number of entries with s_ij == s_k   (info[0] + info[1] >= k); -0 counts as +0
 * Needs n, m >= 1 and 1 <= k <= n*m.  Cost: one pass over M in the usual case (a sample of 65536
 * entries brackets s_k, one pass counts the entries above the bracket and collects those inside it,
 * and the selection finishes on the collected ones); where the sample cannot be used or its bracket
 * fails (fewer than 2^20 entries, a tie of many entries at s_k) a radix selection over M takes over,
 * one pass per 13-bit digit of s_k until the candidates fit the workspace, at most five more passes.
 * The result never depends on the sample.  All kernels (ten launches) are enqueued at once and the
 * host does not wait for any.
 * The workspace is separate from the other calls': regot_topk_workspace_bytes() gives its size
 * (depends on n, m, k; at most 1/16 of the bytes of M plus 2 MB).
 * If an internal count does not add up (possible only with NaNs in the inputs) delta[0] is NaN
 * and info[0] = info[1] = -1.
 */
int regot_topk_workspace_bytes(int64_t n, int64_t m, int64_t k, size_t *bytes /* host, out */);
int regot_topk_threshold(int64_t n, int64_t m,
                         const double *M, int64_t ldM,
                         const double *alpha, const double *beta, double eta,
                         int64_t k,
                         double *delta,                         /* [1] out */
                         double *s_k,                           /* [1] out, optional */
                         int64_t *info,                         /* [2] out */
                         void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * The pattern refresh in one read of M: the top-k threshold (Sec. 3.1) and the fused evaluation together,
 * i.e. what regot_topk_threshold followed by regot_dual_eval_sparsify(delta) computes.  The fused pass runs
 * with the lower end of the bracket that a sample of T puts around the k-th largest entry as its threshold
 * and stages candidates (k plus a fraction of a percent of all entries); the k-th largest staged value is
 * then selected on the device, written to delta[0], and the CSR is built from the staged entries that are
 * not below it.  Outputs as for regot_dual_eval_sparsify, except
 *     info[0]  nnz = number of T_ij >= delta[0]  (>= k; = k without ties)
 *     info[1]  bit 0: nnz > capacity (as in regot_sparsify_csr);
 *              bit 1: the selection could not be made this way (a matrix of fewer than 2^20 entries, a
 *              sample that did not bracket the k-th entry, more candidates than the workspace holds):
 *              delta[0] is NaN, the CSR outputs are unspecified (objective, gradient and sums are valid)
 *              and the caller makes the two calls instead.
 * workspace: regot_workspace_bytes(n, m, c) with c from
 * regot_refresh_candidate_capacity(n, m, k) (candidates, not entries, size the pool); topk_workspace:
 * regot_topk_workspace_bytes(n, m, k).  capacity: entries of col_idx / val.
 */
int regot_refresh_candidate_capacity(int64_t n, int64_t m, int64_t k, int64_t *capacity /* host, out */);
int regot_dual_eval_sparsify_topk(int64_t n, int64_t m,
                                  const double *M, int64_t ldM,
                                  const double *a, const double *b,
                                  const double *alpha, const double *beta, double eta,
                                  int64_t k,
                                  double *obj, double *grad_alpha, double *grad_beta,
                                  double *row_sum, double *col_sum,   /* optional */
                                  double *delta,                      /* [1] out */
                                  int64_t *row_ptr, int32_t *col_idx, double *val, int64_t capacity,
                                  int64_t *info,                      /* [2] out */
                                  void *workspace, size_t workspace_bytes,
                                  void *topk_workspace, size_t topk_workspace_bytes, regot_stream_t stream);

/*
 * ---- Work on a stored sparsity pattern (Sec. 4.2) and the sparse term H_Omega (Sec. 3.1, eq. (7)) ----
 *
 * A pattern is the CSR structure (row_ptr int64 [n+1], col_idx int32, 0-based, strictly ascending
 * inside a row, all m columns) that regot_sparsify_csr / regot_dual_eval_sparsify write.  `capacity`
 * is the length of the entry arrays (col_idx, val, ...) the caller allocated, >= row_ptr[n]: no
 * entry at or beyond it is read or written, and a col_idx outside [0, m) is skipped, so that a
 * damaged pattern cannot make a kernel leave the caller's buffers.  These calls need no workspace
 * unless a parameter says so; they follow the common conventions above (device pointers, async).
 *
 * Values of the plan on a stored pattern: val[p] = T_{i, col_idx[p]} for the entries p of row i.
 * Sec. 4.2 keeps the pattern for S iterations and recomputes only these numbers (one random
 * 8-byte read of M per entry instead of a pass over M).  If val_csc is not NULL the same values are
 * also written in column order, val_csc[csc_pos[p]] = val[p] (csc_pos from regot_pattern_transpose).
 * Values equal those regot_sparsify_csr writes for the same entries, bit for bit.
 */
int regot_pattern_values(int64_t n, int64_t m,
                         const double *M, int64_t ldM,
                         const double *alpha, const double *beta, double eta,
                         const int64_t *row_ptr, const int32_t *col_idx,
                         const int64_t *csc_pos,                /* [capacity], optional */
                         int64_t capacity,
                         double *val,                           /* [capacity] out */
                         double *val_csc,                       /* [capacity] out, optional */
                         regot_stream_t stream);

/*
 * The pattern by columns (symbolic, once per pattern): col_ptr int64 [m+1]; row_idx[q] int32, strictly
 * ascending inside a column; csc_pos[p] = position q of CSR entry p in the column order (-1 for an entry
 * whose col_idx is outside [0, m): it belongs to no column).
 * nnz is a HOST value and must equal row_ptr[n] (the caller has read info[0] of the sparsify call);
 * nnz <= 2^31 - 1.  Workspace: regot_pattern_transpose_workspace_bytes(n, m, nnz), 256-byte aligned
 * (20.5 bytes per entry + a few KB).  The CSR positions, which start out in ascending order, are sorted
 * stably by column (a radix sort of this library, 8 bits per pass: two passes for m < 65536); inside a
 * column ascending position is ascending row.  No atomics on memory: the same bits on every call.
 */
int regot_pattern_transpose_workspace_bytes(int64_t n, int64_t m, int64_t nnz, size_t *bytes /* host, out */);
int regot_pattern_transpose(int64_t n, int64_t m, int64_t nnz /* host */,
                            const int64_t *row_ptr, const int32_t *col_idx,
                            int64_t *col_ptr,                   /* [m+1] out */
                            int32_t *row_idx,                   /* [nnz] out */
                            int64_t *csc_pos,                   /* [nnz] out */
                            void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * y = (H_Omega + tau I) x, the product eq. (6) needs for v = (H_Omega + tau I) s^-, with
 *     H_Omega = (1/eta) [ diag(T 1_m)         T^Omega_{-m}       ]      x = (x_alpha[n], x_beta[m-1])
 *                       [ (T^Omega_{-m})^T    diag(T_{-m}^T 1_n) ]      (Sec. 3.1, eq. (7))
 * T^Omega = the stored pattern with its values; "-m" drops the last column (entries of the pattern in
 * column m-1 are skipped; beta_m is the dual variable the paper fixes).  row_sum = T 1_m [n] and
 * col_sum = T^T 1_n [m] are the FULL sums from regot_dual_eval.  The product with the transposed block
 * reads the pattern by columns (col_ptr, row_idx, val_csc), so every sum has a fixed order and the
 * result is bit-reproducible; no floating-point atomics.  x and y have n + m - 1 entries and must not
 * overlap.  Needs n, m >= 1; tau may be 0.
 */
int regot_hessian_matvec(int64_t n, int64_t m, double eta, double tau,
                         const int64_t *row_ptr, const int32_t *col_idx, const double *val,
                         const int64_t *col_ptr, const int32_t *row_idx, const double *val_csc,
                         int64_t capacity,
                         const double *row_sum, const double *col_sum,
                         const double *x, double *y,
                         regot_stream_t stream);

/*
 * Lower triangle of H_Omega + tau I by columns (compressed sparse column), the matrix a sparse
 * Cholesky factorisation takes (Sec. 3.2): column i < n holds the diagonal row_sum[i]/eta + tau and
 * the entries of row i of T^Omega_{-m} as rows n + j (ascending); column n + j, j < m - 1, holds
 * its diagonal col_sum[j]/eta + tau only.
 *     h_col_ptr int64 [n+m];  h_row_idx int32, h_val fp64 [h_capacity]
 *     info[0] = number of entries = n + m - 1 + (pattern entries outside column m-1),
 *     info[1] = 1 if that exceeds h_capacity (then the arrays are incomplete, h_col_ptr is exact).
 * values_only = 1 rewrites h_val alone on the structure a previous call with values_only = 0 left in
 * h_col_ptr (the amortised iterations of Sec. 4.2).  Workspace: regot_hessian_workspace_bytes(n, m).
 */
int regot_hessian_workspace_bytes(int64_t n, int64_t m, size_t *bytes /* host, out */);
int regot_hessian_lower_csc(int64_t n, int64_t m, double eta, double tau,
                            const int64_t *row_ptr, const int32_t *col_idx, const double *val,
                            int64_t capacity,
                            const double *row_sum, const double *col_sum,
                            int64_t *h_col_ptr, int32_t *h_row_idx, double *h_val,
                            int64_t h_capacity,
                            int64_t *info,                      /* [2] out */
                            int values_only,
                            void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * Optimality measures of a dual point (App. A.5; Algorithm 1 line 6 uses the gradient norm for tau),
 * from the row and column sums regot_dual_eval produced at that point:
 *     metrics[0] = L_p = <T, M> + eta sum T log T - eta sum T   (primal value; evaluated through the
 *                  identity sum_ij T_ij (alpha_i + beta_j) - eta sum T = alpha^T r + beta^T c - eta sum r)
 *     metrics[1] = L_p - L_d = alpha^T (T 1 - a) + beta^T (T^T 1 - b)          (duality gap)
 *     metrics[2] = || T 1 - a ||_1 + || T^T 1 - b ||_1                           (marginal error)
 *     metrics[3] = || grad f ||_2 over x = (alpha, beta_1 .. beta_{m-1})         (Sec. 3.1)
 * O(n + m) work, two small kernels, fixed summation order.  Any workspace of regot_workspace_bytes(n, m, -1)
 * bytes or more will do (not one that a call overlapping in time uses).
 */
int regot_dual_metrics(int64_t n, int64_t m,
                       const double *a, const double *b,
                       const double *alpha, const double *beta, double eta,
                       const double *row_sum, const double *col_sum,  /* [n], [m]: T 1, T^T 1 */
                       double *metrics,                                /* [4] out */
                       void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * Choice between two candidate iterates (Sec. 4.3): the quasi-Newton candidate q and the Sinkhorn
 * candidate s generated meanwhile, each with its dual objective already evaluated (obj_q, obj_s: device
 * scalars written by regot_dual_eval).  The one with the larger L (smaller f = -L) is copied to
 * (alpha_out, beta_out); q unless s is strictly better.  choice[0] = 0 for q, 1 for s.  The outputs may be
 * the buffers of either candidate.  Everything stays on the device: the host need not wait to know.
 */
int regot_choose_candidate(int64_t n, int64_t m,
                           const double *obj_q, const double *obj_s,    /* [1], [1] */
                           const double *alpha_q, const double *beta_q,
                           const double *alpha_s, const double *beta_s,
                           double *alpha_out, double *beta_out,
                           int64_t *choice,                              /* [1] out */
                           regot_stream_t stream);

/*
 * Solve (H_Omega + tau I) x = rhs by conjugate gradients preconditioned with the diagonal, from x = 0:
 * an iterative, GPU-only alternative to the sparse Cholesky solve of Sec. 3.2 (H_Omega + tau I is
 * symmetric positive definite, Theorem 1).  Pattern, values, sums, eta, tau as for regot_hessian_matvec;
 * rhs and x have n + m - 1 entries.  The call enqueues `iterations` iterations (three kernels each);
 * the iteration stops changing x once ||r||_2 <= rtol ||rhs||_2 (the remaining kernels return at once).
 * restart = 1 starts a new solve; restart = 0 continues the one whose state the workspace holds (same
 * arguments), so a caller can enqueue the iterations in portions and read info in between:
 *     info[0] = iterations done, info[1] = 1 if converged, info[2] = ||r||_2, info[3] = ||rhs||_2.
 * Sums are formed in a fixed order: results are bit-reproducible.
 * Workspace: regot_pcg_workspace_bytes(n, m) (ten vectors of n + m - 1 doubles + 64 KB; the same
 * workspace serves regot_pcg_solve2).
 */
int regot_pcg_workspace_bytes(int64_t n, int64_t m, size_t *bytes /* host, out */);
int regot_pcg_solve(int64_t n, int64_t m, double eta, double tau,
                    const int64_t *row_ptr, const int32_t *col_idx, const double *val,
                    const int64_t *col_ptr, const int32_t *row_idx, const double *val_csc,
                    int64_t capacity,
                    const double *row_sum, const double *col_sum,
                    const double *rhs, double *x,
                    double rtol, int iterations, int restart,
                    double *info,                               /* [4] out */
                    void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * The same system, (H_Omega + tau I) x = rhs, solved through the Schur complement of its first block.  In the
 * block form of eq. (7), [D1 B; B^T D2] with diagonal D1 (n) and D2 (m - 1), eliminating the first block leaves
 * S x2 = rhs2 - B^T D1^{-1} rhs1, S = D2 - B^T D1^{-1} B, and x1 = D1^{-1} (rhs1 - B x2).  Conjugate gradients
 * on S preconditioned with D2, from x2 = 0: about half the iterations of regot_pcg_solve at the same cost per
 * iteration (four kernels: the product with B by rows, the product with B^T by columns, two vector kernels).
 * Arguments, restart, info and workspace as for regot_pcg_solve.  The residual of the whole system at
 * (x1, x2) is (0, residual of S), so the stopping rule is the same: ||residual||_2 <= rtol ||rhs||_2, where a
 * residual that satisfies it from the start needs no iteration.  x[n ..] is the iterate while the solve runs
 * (a call with restart = 0 must be given the same x); x[0 .. n) is written by the last kernel of every call.
 */
int regot_pcg_solve_reduced(int64_t n, int64_t m, double eta, double tau,
                            const int64_t *row_ptr, const int32_t *col_idx, const double *val,
                            const int64_t *col_ptr, const int32_t *row_idx, const double *val_csc,
                            int64_t capacity,
                            const double *row_sum, const double *col_sum,
                            const double *rhs, double *x,
                            double rtol, int iterations, int restart,
                            double *info,                               /* [4] out */
                            void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * Two systems with the same matrix at once: (H_Omega + tau I) x_a = rhs_a and (H_Omega + tau I) x_b = rhs_b,
 * the two solves a quasi-Newton direction needs (Algorithm 1, lines 3-7: for the gradient and for y^-).
 * Arguments as for regot_pcg_solve.  The pattern is read once per iteration for both systems, which makes
 * the pair cost little more than one solve.  Each system stops on its own: x_a, x_b and their halves of
 *     info[0..3] (system a), info[4..7] (system b): iterations done, converged, ||r||_2, ||rhs||_2
 * are bit for bit what two calls of regot_pcg_solve give.  x_a and x_b must not be the same array; they
 * are written when the call's last kernel runs.  restart = 0 continues a solve of the same kind (two
 * systems) whose state the workspace holds.
 */
int regot_pcg_solve2(int64_t n, int64_t m, double eta, double tau,
                     const int64_t *row_ptr, const int32_t *col_idx, const double *val,
                     const int64_t *col_ptr, const int32_t *row_idx, const double *val_csc,
                     int64_t capacity,
                     const double *row_sum, const double *col_sum,
                     const double *rhs_a, const double *rhs_b, double *x_a, double *x_b,
                     double rtol, int iterations, int restart,
                     double *info,                              /* [8] out */
                     void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * regot_pcg_solve2 through the Schur complement: two systems in one reduced iteration.  Arguments as for
 * regot_pcg_solve2; x_a, x_b and info are bit for bit what two calls of regot_pcg_solve_reduced give.  The
 * second blocks of the iterates live in the workspace; x_a and x_b are written by the call's last kernels.
 */
int regot_pcg_solve2_reduced(int64_t n, int64_t m, double eta, double tau,
                             const int64_t *row_ptr, const int32_t *col_idx, const double *val,
                             const int64_t *col_ptr, const int32_t *row_idx, const double *val_csc,
                             int64_t capacity,
                             const double *row_sum, const double *col_sum,
                             const double *rhs_a, const double *rhs_b, double *x_a, double *x_b,
                             double rtol, int iterations, int restart,
                             double *info,                              /* [8] out */
                             void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * The quasi-Newton direction d = -B^{-1} g, B = H_Omega + R + tau I (Algorithm 1, lines 3-7), from solves
 * with A = H_Omega + tau I: p = A^{-1} g, q = A^{-1} y^-, and s^- (= A^{-1} v, since v = A s^-, eq. (6)).
 * R = xi u u^T + zeta v v^T (u = y^-, xi = 1/(y^-)^T s^-, zeta = -1/v^T s^-) enters through the
 * Sherman-Morrison-Woodbury identity, and only if (y^-)^T s^- > 1e-6 ||y^-||^2 (line 5); otherwise, or
 * with q = s_prev = y_prev = v = NULL (no previous step), d = -p.  All vectors have n + m - 1 entries.
 *     info[0] = 1 if the rank-two term was used, info[1] = (y^-)^T s^-.
 * The inner products are summed in two stages in a fixed order (bit-reproducible).  Workspace:
 * regot_pcg_workspace_bytes(n, m); the workspace of the solves can be used (their state is not needed
 * any more once p and q are there).
 */
int regot_splr_direction(int64_t n, int64_t m,
                         const double *p, const double *q,
                         const double *s_prev, const double *y_prev, const double *v,
                         double *d,
                         double *info,                          /* [2] out */
                         void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * Measurement aid, not part of the method: one pass over M with the tiling and the loads of the dense
 * calls (the g_r x g_c cut of regot_plan_geometry(n, m, -1), 128-bit non-temporal loads, four rows per
 * wave in flight) that only adds the entries up.  sum[0] = sum of all M_ij (fixed order).  Its duration
 * is the rate at which this tiling can stream M from memory on the device at hand: what the streaming
 * kernels above are measured against besides the nominal peak.  Workspace as for regot_dual_eval;
 * n = 0 or m = 0 gives 0.
 */
int regot_stream_read_probe(int64_t n, int64_t m,
                            const double *M, int64_t ldM,
                            double *sum,                        /* [1] out */
                            void *workspace, size_t workspace_bytes, regot_stream_t stream);

/*
 * Measurement aid, not part of the method: where the device puts the workgroups of a grid launched like the
 * fused pass (256 threads, the same LDS, two workgroups per compute unit).  ids[2b] = the hardware-id register of
 * workgroup b (compute unit in bits 11:8, shader array in bit 12, shader engine in bits 15:13), ids[2b+1] = its
 * die (XCC) id register.  The fused pass lets the two workgroups of a compute unit keep each other's pace and
 * assumes that workgroups b and b + 256 of a 512-workgroup grid are those two (and the scatter kernel that
 * workgroups with equal b mod 8 share a die); a test reads this probe to see whether that holds on the
 * device at hand (only speed depends on it).  1 <= grid <= 65536.
 */
int regot_placement_probe(int grid, uint32_t *ids /* device, [2 * grid] out */, regot_stream_t stream);

/*
 * Profiling aid, not part of the method.  The next call of any entry point above made by the
 * calling host thread records `start_event` on its stream just before, and `stop_event` just
 * after, the launch of its streaming kernel (the single pass over M; the small combine / scatter
 * kernels that follow are outside the pair; for regot_topk_threshold it is the first pass over M).  Both are hipEvent_t handles owned by the caller,
 * created with timing enabled; either may be NULL.  The request is consumed by that one call.
 * The request is state of the calling host thread only.
 */
int regot_profile_stage1(void *start_event /* host handle */, void *stop_event /* host handle */);

#ifdef __cplusplus
}
#endif
#endif /* REGOT_H */
