"""CPU oracle for the dense streaming pass of the entropic-OT dual.

TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the GPU library must never do so and
shares nothing with it.

This module marshals numpy arrays into ``liboracle.so`` (built from
``regot_oracle.c`` by ``oracle/build.py``); the arithmetic of the dense pass, of
the sparse term H_Omega and of the optimality measures is in the C file, which
cites the passages of the paper it follows.  Three things are plain Python loops
over those C functions: ``sinkhorn_sweeps`` ("alpha half-step, then beta
half-step": block coordinate ascent, Sec. 1), ``pcg_solve`` /
``quasi_newton_direction`` (textbook preconditioned conjugate gradients and the
Sherman-Morrison-Woodbury identity for Algorithm 1, lines 3-7) and
``choose_candidate`` (Sec. 4.3).
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

_c_double_p = ctypes.POINTER(ctypes.c_double)
_c_i64_p = ctypes.POINTER(ctypes.c_int64)
_c_i32_p = ctypes.POINTER(ctypes.c_int32)


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(_LIB_PATH)
    i64, dbl, p = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
    lib.oracle_set_threads.argtypes = [ctypes.c_int]
    lib.oracle_set_threads.restype = None
    lib.oracle_get_max_threads.argtypes = []
    lib.oracle_get_max_threads.restype = ctypes.c_int
    lib.oracle_plan_dense.argtypes = [i64, i64, p, i64, p, p, dbl, p]
    lib.oracle_dual_eval.argtypes = [i64, i64, p, i64, p, p, p, p, dbl, p, p, p, p, p]
    lib.oracle_sparsify_count.argtypes = [i64, i64, p, i64, p, p, dbl, dbl, p, p]
    lib.oracle_sparsify_fill.argtypes = [i64, i64, p, i64, p, p, dbl, dbl, p, p, p]
    lib.oracle_sinkhorn_half_step.argtypes = [i64, i64, p, i64, p, p, p, dbl, ctypes.c_int, p]
    lib.oracle_topk_threshold.argtypes = [i64, i64, p, i64, p, p, dbl, i64, p]
    lib.oracle_dual_metrics.argtypes = [i64, i64, p, i64, p, p, p, p, dbl, p]
    lib.oracle_pattern_values.argtypes = [i64, i64, p, i64, p, p, dbl, p, p, p]
    lib.oracle_pattern_transpose.argtypes = [i64, i64, p, p, p, p, p]
    lib.oracle_hessian_matvec.argtypes = [i64, i64, dbl, dbl, p, p, p, p, p, p, p]
    lib.oracle_hessian_dense.argtypes = [i64, i64, dbl, dbl, p, p, p, p, p, p]
    lib.oracle_hessian_lower_csc.argtypes = [i64, i64, dbl, dbl, p, p, p, p, p, p, p, p]
    for name in ("oracle_plan_dense", "oracle_dual_eval", "oracle_sparsify_count",
                 "oracle_sparsify_fill", "oracle_sinkhorn_half_step", "oracle_topk_threshold"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def set_threads(threads: int) -> None:
    _load().oracle_set_threads(int(threads))


def get_max_threads() -> int:
    return int(_load().oracle_get_max_threads())


def _mat(M):
    """Returns (array, n, m, ldM); keeps a row-strided fp64 view as it is, copies anything else."""
    M = np.asarray(M)
    if M.ndim != 2:
        raise ValueError("M must be 2-D")
    n, m = M.shape
    strided_ok = (M.dtype == np.float64 and n > 0 and m > 0 and M.strides[1] == 8
                  and M.strides[0] % 8 == 0 and M.strides[0] >= 8 * m)
    if not strided_ok:
        M = np.ascontiguousarray(M, dtype=np.float64)
        return M, n, m, max(m, 1)
    return M, n, m, M.strides[0] // 8


def _vec(v, length, name):
    v = np.ascontiguousarray(v, dtype=np.float64)
    if v.shape != (length,):
        raise ValueError(f"{name}: expected shape ({length},), got {v.shape}")
    return v


def _ptr(arr):
    return arr.ctypes.data_as(ctypes.c_void_p)


def _check(status, what):
    if status != 0:
        raise RuntimeError(f"{what} failed with status {status}")


def plan_dense(M, alpha, beta, eta):
    """Dense T_ij = exp((alpha_i + beta_j - M_ij)/eta) (Sec. 3.1). Small inputs only."""
    M, n, m, ld = _mat(M)
    alpha, beta = _vec(alpha, n, "alpha"), _vec(beta, m, "beta")
    T = np.empty((n, m), dtype=np.float64)
    _check(_load().oracle_plan_dense(n, m, _ptr(M), ld, _ptr(alpha), _ptr(beta), float(eta), _ptr(T)), "plan_dense")
    return T


def dual_eval(M, a, b, alpha, beta, eta):
    """Returns dict(obj=L, grad_alpha=a-T1, grad_beta=b-T^T1, row_sum=T1, col_sum=T^T1)."""
    M, n, m, ld = _mat(M)
    a, b = _vec(a, n, "a"), _vec(b, m, "b")
    alpha, beta = _vec(alpha, n, "alpha"), _vec(beta, m, "beta")
    obj = np.zeros(1)
    ga, gb = np.empty(n), np.empty(m)
    r, c = np.empty(n), np.empty(m)
    _check(_load().oracle_dual_eval(n, m, _ptr(M), ld, _ptr(a), _ptr(b), _ptr(alpha), _ptr(beta), float(eta),
                                    _ptr(obj), _ptr(ga), _ptr(gb), _ptr(r), _ptr(c)), "dual_eval")
    return dict(obj=float(obj[0]), grad_alpha=ga, grad_beta=gb, row_sum=r, col_sum=c)


def sparsify_csr(M, alpha, beta, eta, delta):
    """CSR (row_ptr int64, col_idx int32, val fp64) of {T_ij >= delta} (Sec. 3.1, eq. (7))."""
    M, n, m, ld = _mat(M)
    alpha, beta = _vec(alpha, n, "alpha"), _vec(beta, m, "beta")
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    nnz = np.zeros(1, dtype=np.int64)
    lib = _load()
    _check(lib.oracle_sparsify_count(n, m, _ptr(M), ld, _ptr(alpha), _ptr(beta), float(eta), float(delta),
                                     _ptr(row_ptr), _ptr(nnz)), "sparsify_count")
    k = int(nnz[0])
    col_idx = np.empty(max(k, 1), dtype=np.int32)
    val = np.empty(max(k, 1), dtype=np.float64)
    _check(lib.oracle_sparsify_fill(n, m, _ptr(M), ld, _ptr(alpha), _ptr(beta), float(eta), float(delta),
                                    _ptr(row_ptr), _ptr(col_idx), _ptr(val)), "sparsify_fill")
    return row_ptr, col_idx[:k], val[:k]


def sinkhorn_half_step(M, marginal, alpha, beta, eta, which):
    """which=0: new alpha from (a, beta); which=1: new beta from (b, alpha)."""
    M, n, m, ld = _mat(M)
    alpha, beta = _vec(alpha, n, "alpha"), _vec(beta, m, "beta")
    length = n if which == 0 else m
    marginal = _vec(marginal, length, "marginal")
    out = np.empty(length)
    _check(_load().oracle_sinkhorn_half_step(n, m, _ptr(M), ld, _ptr(marginal), _ptr(alpha), _ptr(beta),
                                             float(eta), int(which), _ptr(out)), "sinkhorn_half_step")
    return out


def sinkhorn_sweeps(M, a, b, eta, sweeps, alpha0=None, beta0=None):
    """`sweeps` times (alpha half-step, then beta half-step), from alpha=beta=0 by default."""
    M, n, m, _ = _mat(M)
    alpha = np.zeros(n) if alpha0 is None else np.array(alpha0, dtype=np.float64)
    beta = np.zeros(m) if beta0 is None else np.array(beta0, dtype=np.float64)
    for _ in range(int(sweeps)):
        alpha = sinkhorn_half_step(M, a, alpha, beta, eta, 0)
        beta = sinkhorn_half_step(M, b, alpha, beta, eta, 1)
    return alpha, beta


def topk_threshold(M, alpha, beta, eta, k):
    """The k-th largest T_ij (top-k rule of Sec. 3.1, in threshold form)."""
    M, n, m, ld = _mat(M)
    alpha, beta = _vec(alpha, n, "alpha"), _vec(beta, m, "beta")
    delta = np.zeros(1)
    _check(_load().oracle_topk_threshold(n, m, _ptr(M), ld, _ptr(alpha), _ptr(beta), float(eta), int(k),
                                         _ptr(delta)), "topk_threshold")
    return float(delta[0])


# ---------------------------------------------------------------- sparse term of the quasi-Newton matrix

def _pattern(row_ptr, col_idx, n):
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    if row_ptr.shape != (n + 1,):
        raise ValueError("row_ptr must have n + 1 entries")
    nnz = int(row_ptr[-1])
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    if col_idx.shape[0] < nnz:
        raise ValueError("col_idx shorter than row_ptr[n]")
    return row_ptr, col_idx, nnz


def _hessian_args(n, m, row_ptr, col_idx, val, row_sum, col_sum):
    row_ptr, col_idx, nnz = _pattern(row_ptr, col_idx, n)
    val = np.ascontiguousarray(val, dtype=np.float64)
    if val.shape[0] < nnz:
        raise ValueError("val shorter than row_ptr[n]")
    return row_ptr, col_idx, val, _vec(row_sum, n, "row_sum"), _vec(col_sum, m, "col_sum")


def pattern_values(M, alpha, beta, eta, row_ptr, col_idx):
    """T_ij at the entries of a stored CSR pattern (Sec. 4.2: values refreshed, pattern kept)."""
    M, n, m, ld = _mat(M)
    alpha, beta = _vec(alpha, n, "alpha"), _vec(beta, m, "beta")
    row_ptr, col_idx, nnz = _pattern(row_ptr, col_idx, n)
    val = np.empty(max(nnz, 1))
    _check(_load().oracle_pattern_values(n, m, _ptr(M), ld, _ptr(alpha), _ptr(beta), float(eta),
                                         _ptr(row_ptr), _ptr(col_idx), _ptr(val)), "pattern_values")
    return val[:nnz]


def pattern_transpose(n, m, row_ptr, col_idx):
    """(col_ptr int64[m+1], row_idx int32[nnz], csc_pos int64[nnz]) of a CSR pattern."""
    row_ptr, col_idx, nnz = _pattern(row_ptr, col_idx, n)
    col_ptr = np.zeros(m + 1, dtype=np.int64)
    row_idx = np.empty(max(nnz, 1), dtype=np.int32)
    csc_pos = np.empty(max(nnz, 1), dtype=np.int64)
    _check(_load().oracle_pattern_transpose(n, m, _ptr(row_ptr), _ptr(col_idx), _ptr(col_ptr), _ptr(row_idx),
                                            _ptr(csc_pos)), "pattern_transpose")
    return col_ptr, row_idx[:nnz], csc_pos[:nnz]


def hessian_matvec(n, m, eta, tau, row_ptr, col_idx, val, row_sum, col_sum, x):
    """y = (H_Omega + tau I) x of Sec. 3.1, eq. (7); x, y of length n + m - 1."""
    row_ptr, col_idx, val, row_sum, col_sum = _hessian_args(n, m, row_ptr, col_idx, val, row_sum, col_sum)
    x = _vec(x, n + m - 1, "x")
    y = np.empty(n + m - 1)
    _check(_load().oracle_hessian_matvec(n, m, float(eta), float(tau), _ptr(row_ptr), _ptr(col_idx), _ptr(val),
                                         _ptr(row_sum), _ptr(col_sum), _ptr(x), _ptr(y)), "hessian_matvec")
    return y


def hessian_dense(n, m, eta, tau, row_ptr, col_idx, val, row_sum, col_sum):
    """H_Omega + tau I as a dense matrix (small sizes)."""
    row_ptr, col_idx, val, row_sum, col_sum = _hessian_args(n, m, row_ptr, col_idx, val, row_sum, col_sum)
    N = n + m - 1
    H = np.empty((N, N))
    _check(_load().oracle_hessian_dense(n, m, float(eta), float(tau), _ptr(row_ptr), _ptr(col_idx), _ptr(val),
                                        _ptr(row_sum), _ptr(col_sum), _ptr(H)), "hessian_dense")
    return H


def hessian_lower_csc(n, m, eta, tau, row_ptr, col_idx, val, row_sum, col_sum):
    """Lower triangle of H_Omega + tau I, compressed columns: (col_ptr int64[n+m], row_idx int32, val)."""
    row_ptr, col_idx, val, row_sum, col_sum = _hessian_args(n, m, row_ptr, col_idx, val, row_sum, col_sum)
    lib = _load()
    h_col_ptr = np.zeros(n + m, dtype=np.int64)
    args = (n, m, float(eta), float(tau), _ptr(row_ptr), _ptr(col_idx), _ptr(val), _ptr(row_sum), _ptr(col_sum))
    _check(lib.oracle_hessian_lower_csc(*args, _ptr(h_col_ptr), None, None), "hessian_lower_csc")
    nnz = int(h_col_ptr[-1])
    h_row_idx = np.empty(nnz, dtype=np.int32)
    h_val = np.empty(nnz)
    _check(lib.oracle_hessian_lower_csc(*args, _ptr(h_col_ptr), _ptr(h_row_idx), _ptr(h_val)), "hessian_lower_csc")
    return h_col_ptr, h_row_idx, h_val


# ---------------------------------------------------------------- optimality measures, candidate choice

def dual_metrics(M, a, b, alpha, beta, eta):
    """dict(primal=L_p, gap=L_p-L_d, marginal_error, grad_norm) of App. A.5 / Algorithm 1, by the direct definitions."""
    M, n, m, ld = _mat(M)
    a, b = _vec(a, n, "a"), _vec(b, m, "b")
    alpha, beta = _vec(alpha, n, "alpha"), _vec(beta, m, "beta")
    out = np.zeros(4)
    _check(_load().oracle_dual_metrics(n, m, _ptr(M), ld, _ptr(a), _ptr(b), _ptr(alpha), _ptr(beta), float(eta),
                                       _ptr(out)), "dual_metrics")
    return dict(primal=float(out[0]), gap=float(out[1]), marginal_error=float(out[2]), grad_norm=float(out[3]))


def choose_candidate(M, a, b, eta, cand_q, cand_s):
    """Sec. 4.3: of the quasi-Newton candidate and the Sinkhorn candidate (each an (alpha, beta) pair) keep the
    one with the larger dual objective L (the smaller f = -L); the quasi-Newton one on a tie.
    Returns (index 0 = q / 1 = s, L_q, L_s)."""
    Lq = dual_eval(M, a, b, cand_q[0], cand_q[1], eta)["obj"]
    Ls = dual_eval(M, a, b, cand_s[0], cand_s[1], eta)["obj"]
    return (1 if Ls > Lq else 0), Lq, Ls


# ---------------------------------------------------------------- quasi-Newton direction by an iterative solve

def pcg_solve(n, m, eta, tau, row_ptr, col_idx, val, row_sum, col_sum, rhs, rtol=1e-10, max_iter=1000):
    """Solve (H_Omega + tau I) x = rhs by conjugate gradients preconditioned with the diagonal
    (textbook PCG from x = 0; stops when ||r||_2 <= rtol ||rhs||_2).  Returns (x, iterations, ||r|| / ||rhs||).
    An iterative stand-in for the sparse Cholesky solve of Sec. 3.2 (the paper lists iterative solvers as
    future work); H_Omega + tau I is symmetric positive definite (Theorem 1), so the iteration converges."""
    rhs = _vec(rhs, n + m - 1, "rhs")
    diag = np.concatenate([np.asarray(row_sum, dtype=np.float64), np.asarray(col_sum, dtype=np.float64)[:m - 1]]) / eta + tau
    A = lambda x: hessian_matvec(n, m, eta, tau, row_ptr, col_idx, val, row_sum, col_sum, x)
    x = np.zeros_like(rhs)
    r = rhs.copy()
    bb = float(r @ r)
    if bb == 0.0:
        return x, 0, 0.0
    z = r / diag
    p = z.copy()
    rz = float(r @ z)
    it = 0
    while it < max_iter and float(r @ r) > rtol * rtol * bb:
        Ap = A(p)
        step = rz / float(p @ Ap)
        x += step * p
        r -= step * Ap
        z = r / diag
        rz_new = float(r @ z)
        p = z + (rz_new / rz) * p
        rz = rz_new
        it += 1
    return x, it, float(np.sqrt((r @ r) / bb))


def pcg_solve_reduced(n, m, eta, tau, row_ptr, col_idx, val, row_sum, col_sum, rhs, rtol=1e-10, max_iter=1000):
    """The same system as pcg_solve, (H_Omega + tau I) x = rhs, solved through its Schur complement.

    With H_Omega + tau I = [[D1, B], [B^T, D2]] (eq. (7): D1 = diag(T 1)/eta + tau, D2 = diag(T_{-m}^T 1)/eta + tau,
    B = T^Omega_{-m}/eta) and rhs = (g1, g2), eliminating the first block leaves
        S x2 = g2 - B^T D1^{-1} g1,   S = D2 - B^T D1^{-1} B,   x1 = D1^{-1} (g1 - B x2),
    and S is symmetric positive definite because the whole matrix is (Theorem 1).  Conjugate gradients on S,
    preconditioned with D2, from x2 = 0; the residual of the full system at (x1, x2) is (0, residual of S), so the
    iteration stops when that residual is <= rtol ||rhs||_2.  Returns (x, iterations, ||residual|| / ||rhs||).
    (Textbook: the reduced system of a matrix whose two diagonal blocks are themselves diagonal needs about half the
    iterations of the diagonally preconditioned full system, at the same cost per iteration.)"""
    rhs = _vec(rhs, n + m - 1, "rhs")
    d1 = np.asarray(row_sum, dtype=np.float64) / eta + tau
    d2 = np.asarray(col_sum, dtype=np.float64)[:m - 1] / eta + tau
    full = lambda x: hessian_matvec(n, m, eta, tau, row_ptr, col_idx, val, row_sum, col_sum, x)
    # products with the off-diagonal blocks alone: the other half of the vector is zero
    B_times = lambda x2: full(np.concatenate([np.zeros(n), x2]))[:n]
    Bt_times = lambda x1: full(np.concatenate([x1, np.zeros(m - 1)]))[n:]
    g1, g2 = rhs[:n], rhs[n:]
    norm2 = float(rhs @ rhs)
    if norm2 == 0.0:
        return np.zeros_like(rhs), 0, 0.0
    x2 = np.zeros(m - 1)
    res = g2 - Bt_times(g1 / d1)
    zed = res / d2
    q = zed.copy()
    rho = float(res @ zed)
    it = 0
    while it < max_iter and float(res @ res) > rtol * rtol * norm2:
        Sq = d2 * q - Bt_times(B_times(q) / d1)
        a = rho / float(q @ Sq)
        x2 += a * q
        res = res - a * Sq
        zed = res / d2
        rho_new = float(res @ zed)
        q = zed + (rho_new / rho) * q
        rho = rho_new
        it += 1
    x1 = (g1 - B_times(x2)) / d1
    return np.concatenate([x1, x2]), it, float(np.sqrt((res @ res) / norm2))


def quasi_newton_direction(n, m, eta, tau, row_ptr, col_idx, val, row_sum, col_sum, g, s_prev=None, y_prev=None,
                           rtol=1e-10, max_iter=1000, reduced=False):
    """d = -B^{-1} g with B = H_Omega + R + tau I (Algorithm 1, lines 3-7; eq. (5), (6)).

    R = xi u u^T + zeta v v^T with u = y^-, v = (H_Omega + tau I) s^-, xi = 1 / (y^-)^T s^-, zeta = -1 / v^T s^-,
    used only if (y^-)^T s^- > 1e-6 ||y^-||^2.  With A = H_Omega + tau I the rank-two term is handled by the
    Sherman-Morrison-Woodbury identity B^{-1} = A^{-1} - A^{-1} U (C^{-1} + U^T A^{-1} U)^{-1} U^T A^{-1},
    U = [u v], C = diag(xi, zeta); A^{-1} v = s^- by construction, so two solves with A suffice
    (`reduced`: by pcg_solve_reduced instead of pcg_solve).  Returns (d, used_rank_two)."""
    g = _vec(g, n + m - 1, "g")
    inner = pcg_solve_reduced if reduced else pcg_solve   # which iteration performs the two solves
    solve = lambda rhs: inner(n, m, eta, tau, row_ptr, col_idx, val, row_sum, col_sum, rhs, rtol, max_iter)[0]
    p = solve(g)
    if s_prev is None or y_prev is None:
        return -p, False
    s = _vec(s_prev, n + m - 1, "s_prev")
    y = _vec(y_prev, n + m - 1, "y_prev")
    ys = float(y @ s)
    if not ys > 1e-6 * float(y @ y):
        return -p, False
    v = hessian_matvec(n, m, eta, tau, row_ptr, col_idx, val, row_sum, col_sum, s)
    q = solve(y)
    w = s                                   # A^{-1} v
    K = np.array([[ys + float(y @ q), float(y @ w)],
                  [float(v @ q), -float(v @ s) + float(v @ w)]])
    c = np.linalg.solve(K, np.array([float(y @ p), float(v @ p)]))
    return -(p - c[0] * q - c[1] * w), True
