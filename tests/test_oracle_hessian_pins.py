"""Pins of the oracle's sparse-Hessian functions (Sec. 3.1, eq. (7); Sec. 4.2) to facts that do not
come from the oracle itself: finite differences of the gradient, a closed-form product, the
eigenvalue bounds of Theorem 1, and scipy's sparse containers."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2605_08793_amd import workloads as W


def problem(n, m, seed, eta):
    M, a, b, alpha, beta = W.random_small(n, m, seed=seed, eta=eta)
    ev = oracle.dual_eval(M, a, b, alpha, beta, eta)
    return M, a, b, alpha, beta, ev


def full_pattern(n, m):
    row_ptr = np.arange(n + 1, dtype=np.int64) * m
    col_idx = np.tile(np.arange(m, dtype=np.int32), n)
    return row_ptr, col_idx


def grad_f(M, a, b, x, eta):
    """Gradient of f = -L in the variables x = (alpha, beta without its last entry), beta_m = 0 ... kept fixed."""
    n, m = M.shape
    alpha, beta = x[:n], np.concatenate([x[n:], [grad_f.beta_last]])
    ev = oracle.dual_eval(M, a, b, alpha, beta, eta)
    return np.concatenate([-ev["grad_alpha"], -ev["grad_beta"][:-1]])


@pytest.mark.parametrize("n,m,eta", [(5, 4, 0.7), (7, 9, 0.3)])
def test_full_pattern_is_the_hessian_of_f(n, m, eta):
    # Sec. 3.1: with every entry in Omega, H_Omega is the Hessian of f; compare with central
    # differences of the gradient, direction by direction
    M, a, b, alpha, beta, ev = problem(n, m, 21, eta)
    row_ptr, col_idx = full_pattern(n, m)
    val = oracle.pattern_values(M, alpha, beta, eta, row_ptr, col_idx)
    H = oracle.hessian_dense(n, m, eta, 0.0, row_ptr, col_idx, val, ev["row_sum"], ev["col_sum"])
    x = np.concatenate([alpha, beta[:-1]])
    grad_f.beta_last = beta[-1]
    h = 1e-5
    for d in range(n + m - 1):
        e = np.zeros(n + m - 1); e[d] = h
        fd = (grad_f(M, a, b, x + e, eta) - grad_f(M, a, b, x - e, eta)) / (2 * h)
        np.testing.assert_allclose(H[:, d], fd, rtol=2e-6, atol=1e-8 * np.abs(H).max())


def test_closed_form_product_and_symmetry():
    # full Hessian times (1_n, -1_{m-1}) = (1/eta) (last column of T, 0): row sums minus the first
    # m-1 columns leave the last one; the beta block cancels exactly
    n, m, eta = 9, 6, 0.4
    M, a, b, alpha, beta, ev = problem(n, m, 22, eta)
    row_ptr, col_idx = full_pattern(n, m)
    val = oracle.pattern_values(M, alpha, beta, eta, row_ptr, col_idx)
    T = oracle.plan_dense(M, alpha, beta, eta)
    np.testing.assert_array_equal(val.reshape(n, m), T)
    x = np.concatenate([np.ones(n), -np.ones(m - 1)])
    y = oracle.hessian_matvec(n, m, eta, 0.0, row_ptr, col_idx, val, ev["row_sum"], ev["col_sum"], x)
    np.testing.assert_allclose(y[:n], T[:, -1] / eta, rtol=1e-12)
    np.testing.assert_allclose(y[n:], 0.0, atol=1e-12 * ev["col_sum"].max() / eta)
    # tau only adds tau * x
    y2 = oracle.hessian_matvec(n, m, eta, 0.37, row_ptr, col_idx, val, ev["row_sum"], ev["col_sum"], x)
    np.testing.assert_allclose(y2 - y, 0.37 * x, rtol=1e-12, atol=1e-13)
    H = oracle.hessian_dense(n, m, eta, 0.37, row_ptr, col_idx, val, ev["row_sum"], ev["col_sum"])
    np.testing.assert_array_equal(H, H.T)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_eigenvalue_bounds_of_sparsified_hessian(seed):
    # Theorem 1: for Omega containing the first row and column,
    # 0 < lmin(H) <= lmin(H_Omega) <= lmax(H_Omega) <= lmax(H)
    n, m, eta = 12, 10, 0.5
    M, a, b, alpha, beta, ev = problem(n, m, 30 + seed, eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    rng = np.random.default_rng(seed)
    mask = rng.random((n, m)) < 0.3
    mask[0, :] = True; mask[:, 0] = True
    A = sp.csr_matrix(np.where(mask, T, 0.0)); A.sort_indices()
    # scipy drops nothing here: T > 0 everywhere on the mask
    row_ptr, col_idx = A.indptr.astype(np.int64), A.indices.astype(np.int32)
    val = oracle.pattern_values(M, alpha, beta, eta, row_ptr, col_idx)
    np.testing.assert_array_equal(val, A.data)
    H_om = oracle.hessian_dense(n, m, eta, 0.0, row_ptr, col_idx, val, ev["row_sum"], ev["col_sum"])
    fr, fc = full_pattern(n, m)
    H = oracle.hessian_dense(n, m, eta, 0.0, fr, fc, T.ravel(), ev["row_sum"], ev["col_sum"])
    w_om, w = np.linalg.eigvalsh(H_om), np.linalg.eigvalsh(H)
    tol = 1e-12 * w[-1]
    assert 0 < w[0] <= w_om[0] + tol and w_om[-1] <= w[-1] + tol


def test_matvec_csc_and_transpose_against_scipy():
    n, m, eta, tau = 23, 31, 0.2, 0.05
    M, a, b, alpha, beta, ev = problem(n, m, 40, eta)
    beta = beta.copy(); beta[-1] = beta.max() + 0.1      # make sure the last column reaches the pattern
    ev = oracle.dual_eval(M, a, b, alpha, beta, eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    delta = np.quantile(T, 0.8)
    row_ptr, col_idx, val = oracle.sparsify_csr(M, alpha, beta, eta, delta)
    assert np.any(col_idx == m - 1)          # the dropped column is present in the pattern
    np.testing.assert_array_equal(oracle.pattern_values(M, alpha, beta, eta, row_ptr, col_idx), val)
    r, c = ev["row_sum"], ev["col_sum"]
    # reference H_Omega + tau I built with numpy from the dense masked plan
    Tm = np.where(T >= delta, T, 0.0)[:, :-1]
    N = n + m - 1
    Href = np.zeros((N, N))
    Href[:n, :n] = np.diag(r); Href[n:, n:] = np.diag(c[:-1]); Href[:n, n:] = Tm; Href[n:, :n] = Tm.T
    Href = Href / eta + tau * np.eye(N)
    H = oracle.hessian_dense(n, m, eta, tau, row_ptr, col_idx, val, r, c)
    np.testing.assert_allclose(H, Href, rtol=1e-15, atol=0)
    x = np.random.default_rng(4).standard_normal(N)
    y = oracle.hessian_matvec(n, m, eta, tau, row_ptr, col_idx, val, r, c, x)
    np.testing.assert_allclose(y, Href @ x, rtol=1e-13, atol=1e-13 * np.abs(Href).max())
    # lower triangle by columns
    cp, ri, hv = oracle.hessian_lower_csc(n, m, eta, tau, row_ptr, col_idx, val, r, c)
    L = sp.csc_matrix((hv, ri, cp), shape=(N, N)).toarray()
    np.testing.assert_array_equal(L, np.tril(H))
    assert all(np.all(np.diff(ri[cp[j]:cp[j + 1]]) > 0) and ri[cp[j]] == j for j in range(N))
    # the pattern by columns
    col_ptr, row_idx, csc_pos = oracle.pattern_transpose(n, m, row_ptr, col_idx)
    A = sp.csr_matrix((np.arange(1, len(col_idx) + 1, dtype=np.float64), col_idx, row_ptr), shape=(n, m)).tocsc()
    A.sort_indices()
    np.testing.assert_array_equal(col_ptr, A.indptr)
    np.testing.assert_array_equal(row_idx, A.indices)
    np.testing.assert_array_equal(csc_pos[(A.data - 1).astype(np.int64)], np.arange(len(col_idx)))


def test_empty_rows_and_single_column():
    # m = 1: no beta variable at all, H is diag(r)/eta + tau; rows without pattern entries
    n, eta, tau = 6, 0.3, 0.1
    M, a, b, alpha, beta, ev = problem(n, 1, 41, eta)
    row_ptr = np.zeros(n + 1, dtype=np.int64); col_idx = np.zeros(0, dtype=np.int32); val = np.zeros(0)
    x = np.arange(1.0, n + 1)
    y = oracle.hessian_matvec(n, 1, eta, tau, row_ptr, col_idx, val, ev["row_sum"], ev["col_sum"], x)
    np.testing.assert_allclose(y, (ev["row_sum"] / eta + tau) * x, rtol=1e-15)
    cp, ri, hv = oracle.hessian_lower_csc(n, 1, eta, tau, row_ptr, col_idx, val, ev["row_sum"], ev["col_sum"])
    np.testing.assert_array_equal(cp, np.arange(n + 1)); np.testing.assert_array_equal(ri, np.arange(n))


# ------------------------------------------------------------------ optimality measures (App. A.5)

def test_metrics_against_hand_computation_and_identities():
    import math
    n, m, eta = 3, 2, 0.7
    M = np.array([[0.2, 0.9], [0.5, 0.1], [0.8, 0.4]]); a = np.array([0.2, 0.3, 0.5]); b = np.array([0.6, 0.4])
    alpha = np.array([0.1, -0.2, 0.05]); beta = np.array([-0.3, 0.15])
    T = [[math.exp((alpha[i] + beta[j] - M[i, j]) / eta) for j in range(m)] for i in range(n)]
    tm = math.fsum(T[i][j] * M[i, j] for i in range(n) for j in range(m))
    tl = math.fsum(T[i][j] * math.log(T[i][j]) for i in range(n) for j in range(m))
    ts = math.fsum(T[i][j] for i in range(n) for j in range(m))
    Lp = tm + eta * tl - eta * ts
    Ld = -eta * ts + float(alpha @ a) + float(beta @ b)
    r = [math.fsum(T[i]) for i in range(n)]; c = [math.fsum(T[i][j] for i in range(n)) for j in range(m)]
    got = oracle.dual_metrics(M, a, b, alpha, beta, eta)
    assert abs(got["primal"] - Lp) <= 1e-14 * abs(Lp)
    assert abs(got["gap"] - (Lp - Ld)) <= 1e-13 * max(abs(Lp), abs(Ld))
    assert abs(got["marginal_error"] - (sum(abs(r[i] - a[i]) for i in range(n)) + sum(abs(c[j] - b[j]) for j in range(m)))) <= 1e-14
    assert abs(got["grad_norm"] - math.sqrt(sum((r[i] - a[i]) ** 2 for i in range(n)) + (c[0] - b[0]) ** 2)) <= 1e-14
    # a point where the marginal residuals have both signs (absolute values matter)
    alpha2 = np.array([0.1, -2.0, 0.05]); beta2 = np.array([-1.5, 0.15])
    T2 = [[math.exp((alpha2[i] + beta2[j] - M[i, j]) / eta) for j in range(m)] for i in range(n)]
    r2 = [math.fsum(T2[i]) for i in range(n)]; c2 = [math.fsum(T2[i][j] for i in range(n)) for j in range(m)]
    res = [r2[i] - a[i] for i in range(n)] + [c2[j] - b[j] for j in range(m)]
    assert min(res[:n]) < 0 < max(res[:n]) and min(res[n:]) < 0 < max(res[n:])
    got2 = oracle.dual_metrics(M, a, b, alpha2, beta2, eta)
    assert abs(got2["marginal_error"] - math.fsum(abs(x) for x in res)) <= 1e-14
    assert abs(got2["grad_norm"] - math.sqrt(math.fsum(x * x for x in res[:n + m - 1]))) <= 1e-14
    # App. A.5: the gap equals alpha^T (T1 - a) + beta^T (T^T 1 - b); the dual value is dual_eval's objective
    ev = oracle.dual_eval(M, a, b, alpha, beta, eta)
    ident = float(alpha @ (ev["row_sum"] - a) + beta @ (ev["col_sum"] - b))
    assert abs(got["gap"] - ident) <= 1e-13
    assert abs((got["primal"] - got["gap"]) - ev["obj"]) <= 1e-13


def test_metrics_vanish_at_the_optimum_of_a_separable_cost():
    # M_ij = u_i + v_j: the optimum is known in closed form, T = a b^T, primal = dual, all errors zero
    rng = np.random.default_rng(5)
    n, m, eta = 40, 30, 0.05
    u, v = rng.random(n), rng.random(m)
    a = rng.random(n) + 0.1; a /= a.sum(); b = rng.random(m) + 0.1; b /= b.sum()
    M = u[:, None] + v[None, :]
    alpha = eta * np.log(a) + u; beta = eta * np.log(b) + v
    got = oracle.dual_metrics(M, a, b, alpha, beta, eta)
    Lstar = -eta + float(a @ (eta * np.log(a) + u)) + float(b @ (eta * np.log(b) + v))
    assert abs(got["primal"] - Lstar) <= 1e-13 and abs(got["gap"]) <= 1e-13
    assert got["marginal_error"] <= 1e-13 and got["grad_norm"] <= 1e-14


def test_choice_prefers_the_larger_dual_value():
    M, a, b, alpha, beta = W.random_small(30, 40, seed=9, eta=0.2)
    better = oracle.sinkhorn_sweeps(M, a, b, 0.2, 3, alpha, beta)     # ascent steps cannot lower L
    which, Lq, Ls = oracle.choose_candidate(M, a, b, 0.2, (alpha, beta), better)
    assert which == 1 and Ls >= Lq
    which, Lq, Ls = oracle.choose_candidate(M, a, b, 0.2, better, (alpha, beta))
    assert which == 0
    assert oracle.choose_candidate(M, a, b, 0.2, better, better)[0] == 0   # tie: the quasi-Newton candidate


# ------------------------------------------------------------------ quasi-Newton direction (Algorithm 1, lines 3-7)

def _small_splr_problem(seed, n=14, m=11, eta=0.4, tau=0.05):
    M, a, b, alpha, beta, ev = problem(n, m, seed, eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    rng = np.random.default_rng(seed)
    mask = rng.random((n, m)) < 0.4
    mask[0, :] = True; mask[:, 0] = True
    A = sp.csr_matrix(np.where(mask, T, 0.0)); A.sort_indices()
    row_ptr, col_idx, val = A.indptr.astype(np.int64), A.indices.astype(np.int32), A.data.copy()
    g = np.concatenate([ev["row_sum"] - a, (ev["col_sum"] - b)[:-1]])
    return n, m, eta, tau, row_ptr, col_idx, val, ev["row_sum"], ev["col_sum"], g, rng


def test_pcg_solves_the_dense_system():
    n, m, eta, tau, rp, ci, val, r, c, g, rng = _small_splr_problem(51)
    H = oracle.hessian_dense(n, m, eta, tau, rp, ci, val, r, c)
    x, iters, rel = oracle.pcg_solve(n, m, eta, tau, rp, ci, val, r, c, g, rtol=1e-12)
    assert rel <= 1e-12 and 0 < iters <= n + m - 1 + 5       # CG terminates in at most N steps (plus rounding)
    np.testing.assert_allclose(x, np.linalg.solve(H, g), rtol=1e-9, atol=1e-12 * np.abs(x).max())
    x0, it0, _ = oracle.pcg_solve(n, m, eta, tau, rp, ci, val, r, c, np.zeros(n + m - 1))
    assert it0 == 0 and not x0.any()
    # with an empty pattern the matrix is its own diagonal (row / column sums over eta, plus tau): the
    # diagonal preconditioner is then the exact inverse and the first step lands on the solution
    empty_rp = np.zeros(n + 1, dtype=np.int64)
    x1, it1, rel1 = oracle.pcg_solve(n, m, eta, tau, empty_rp, ci[:0], val[:0], r, c, g, rtol=1e-14)
    assert it1 == 1
    np.testing.assert_allclose(x1, g / (np.concatenate([r, c[:-1]]) / eta + tau), rtol=1e-14)


def test_reduced_pcg_solves_the_dense_system():
    """The Schur-complement iteration: same solution as the dense solve, a residual of the FULL system below the
    tolerance, the eliminated block satisfied exactly, and the textbook property that it needs at most about half the
    iterations of the diagonally preconditioned full system."""
    for seed, shape in ((53, (14, 11)), (54, (9, 23)), (55, (30, 2))):
        n, m, eta, tau, rp, ci, val, r, c, g, rng = _small_splr_problem(seed, n=shape[0], m=shape[1])
        H = oracle.hessian_dense(n, m, eta, tau, rp, ci, val, r, c)
        x, iters, rel = oracle.pcg_solve_reduced(n, m, eta, tau, rp, ci, val, r, c, g, rtol=1e-12)
        assert rel <= 1e-12 and 0 < iters <= m - 1 + 3           # CG on the (m-1) x (m-1) Schur complement
        np.testing.assert_allclose(x, np.linalg.solve(H, g), rtol=1e-9, atol=1e-12 * np.abs(x).max())
        res = H @ x - g
        assert np.linalg.norm(res) <= 2e-12 * np.linalg.norm(g)
        assert np.abs(res[:n]).max() <= 1e-14 * np.abs(g).max() * 50     # first block: solved by elimination
        # the Schur complement itself, assembled densely
        D1, Bm, D2 = H[:n, :n], H[:n, n:], H[n:, n:]
        S = D2 - Bm.T @ np.linalg.solve(D1, Bm)
        x2 = np.linalg.solve(S, g[n:] - Bm.T @ np.linalg.solve(D1, g[:n]))
        np.testing.assert_allclose(x[n:], x2, rtol=1e-9, atol=1e-12 * np.abs(x2).max())
        # against the iteration on the full system, at a loose and a tight tolerance
        for rtol in (1e-4, 1e-10):
            xf, itf, _ = oracle.pcg_solve(n, m, eta, tau, rp, ci, val, r, c, g, rtol=rtol)
            xr, itr, relr = oracle.pcg_solve_reduced(n, m, eta, tau, rp, ci, val, r, c, g, rtol=rtol)
            assert itr <= (itf + 1) // 2 + 1, (itr, itf)
            assert relr <= rtol
            np.testing.assert_allclose(xr, xf, rtol=0, atol=50 * rtol * np.abs(xf).max())
    x0, it0, _ = oracle.pcg_solve_reduced(n, m, eta, tau, rp, ci, val, r, c, np.zeros(n + m - 1))
    assert it0 == 0 and not x0.any()
    # empty pattern: the matrix is diagonal, S = D2 and its preconditioner is its inverse
    empty_rp = np.zeros(n + 1, dtype=np.int64)
    x1, it1, rel1 = oracle.pcg_solve_reduced(n, m, eta, tau, empty_rp, ci[:0], val[:0], r, c, g, rtol=1e-14)
    assert it1 == 1
    np.testing.assert_allclose(x1, g / (np.concatenate([r, c[:-1]]) / eta + tau), rtol=1e-14)
    # one column: nothing left to iterate on
    n1, m1, eta1, tau1, rp1, ci1, val1, r1, c1, g1, _ = _small_splr_problem(56, n=8, m=1)
    xs, its, _ = oracle.pcg_solve_reduced(n1, m1, eta1, tau1, rp1, ci1, val1, r1, c1, g1)
    assert its == 0
    np.testing.assert_allclose(xs, g1 / (r1 / eta1 + tau1), rtol=1e-15)


def test_direction_matches_the_dense_quasi_newton_matrix():
    # B = H_Omega + xi u u^T + zeta v v^T + tau I assembled densely (eq. (5), (6)); d = -B^{-1} g
    n, m, eta, tau, rp, ci, val, r, c, g, rng = _small_splr_problem(52)
    H = oracle.hessian_dense(n, m, eta, tau, rp, ci, val, r, c)         # H_Omega + tau I
    N = n + m - 1
    s = 0.1 * rng.standard_normal(N)
    y = H @ s + 0.05 * rng.standard_normal(N)                            # a secant pair with y^T s > 0
    assert y @ s > 1e-6 * (y @ y)
    v = H @ s
    B = H + np.outer(y, y) / (y @ s) - np.outer(v, v) / (v @ s)
    d, used = oracle.quasi_newton_direction(n, m, eta, tau, rp, ci, val, r, c, g, s, y, rtol=1e-13)
    assert used
    np.testing.assert_allclose(d, -np.linalg.solve(B, g), rtol=1e-8, atol=1e-11 * np.abs(d).max())
    # the secant equation of the BFGS-type update: B s = y
    np.testing.assert_allclose(B @ s, y, rtol=1e-10, atol=1e-13)
    # curvature condition violated -> the rank-two term is dropped (Algorithm 1, line 5)
    d0, used0 = oracle.quasi_newton_direction(n, m, eta, tau, rp, ci, val, r, c, g, s, -y, rtol=1e-13)
    assert not used0
    np.testing.assert_allclose(d0, -np.linalg.solve(H, g), rtol=1e-8, atol=1e-11 * np.abs(d0).max())
    d1, used1 = oracle.quasi_newton_direction(n, m, eta, tau, rp, ci, val, r, c, g, rtol=1e-13)
    assert not used1
    np.testing.assert_array_equal(d1, d0)
    # a descent direction for f: g^T d < 0
    assert g @ d < 0 and g @ d0 < 0
    # the same with the two solves done by the reduced iteration
    dr, usedr = oracle.quasi_newton_direction(n, m, eta, tau, rp, ci, val, r, c, g, s, y, rtol=1e-13, reduced=True)
    assert usedr
    np.testing.assert_allclose(dr, -np.linalg.solve(B, g), rtol=1e-8, atol=1e-11 * np.abs(dr).max())
