"""Pins for the CPU oracle: each test ties it to something other than itself.

The paper prints no numeric worked example (all its results are figures), so
the pins are what its formulas and the mathematics fix:

  closed forms      1x1 problem; separable cost M_ij = u_i + v_j (T = a b^T exactly)
  calculus          central differences of L against the gradient output; mixed
                    second differences of L against CSR values (the Hessian's
                    off-diagonal block is T/eta, Sec. 3.1)
  identities        sum of row sums = sum of column sums; gauge invariance
                    (Sec. 1); duality-gap identity (App. A.5)
  optimisation      a half-step zeroes its own block of the gradient, never
                    decreases L, and a converged sweep has vanishing gradient
  library routines  scipy.special.logsumexp for the half-steps, numpy sort for
                    the k-th largest entry, scipy.sparse for the CSR layout
  brute force       pure-Python loops with math.fsum on tiny inputs
"""
import math

import numpy as np
import pytest
import scipy.sparse
import scipy.special

import oracle
from paper_2605_08793_amd import workloads as W


def small(n, m, seed, eta=0.5):
    return W.random_small(n, m, seed, eta)


# ---------------------------------------------------------------- closed forms

def test_one_by_one_closed_form():
    # n = m = 1: T = exp((alpha+beta-M)/eta), L = -eta*T + alpha*a + beta*b   (display after eq. (3))
    M = np.array([[0.3]])
    a = np.array([1.0]); b = np.array([1.0])
    alpha = np.array([0.2]); beta = np.array([-0.05]); eta = 0.7
    T = math.exp((0.2 - 0.05 - 0.3) / 0.7)
    r = oracle.dual_eval(M, a, b, alpha, beta, eta)
    assert r["obj"] == pytest.approx(-0.7 * T + 0.2 - 0.05, rel=1e-15)
    assert r["row_sum"][0] == pytest.approx(T, rel=1e-15)
    assert r["col_sum"][0] == pytest.approx(T, rel=1e-15)
    assert r["grad_alpha"][0] == pytest.approx(1.0 - T, rel=1e-14)
    assert r["grad_beta"][0] == pytest.approx(1.0 - T, rel=1e-14)


def test_two_by_three_hand_case():
    # hand-expanded sums; rectangular so a transposed operand cannot pass
    M = np.array([[0.0, 0.5, 1.0], [0.25, 0.75, 0.125]])
    a = np.array([0.4, 0.6]); b = np.array([0.2, 0.3, 0.5])
    alpha = np.array([0.1, -0.2]); beta = np.array([0.05, 0.0, 0.3]); eta = 0.25
    T = [[math.exp((alpha[i] + beta[j] - M[i, j]) / eta) for j in range(3)] for i in range(2)]
    r = oracle.dual_eval(M, a, b, alpha, beta, eta)
    for i in range(2):
        assert r["row_sum"][i] == pytest.approx(T[i][0] + T[i][1] + T[i][2], rel=1e-15)
        assert r["grad_alpha"][i] == pytest.approx(a[i] - (T[i][0] + T[i][1] + T[i][2]), rel=1e-13)
    for j in range(3):
        assert r["col_sum"][j] == pytest.approx(T[0][j] + T[1][j], rel=1e-15)
        assert r["grad_beta"][j] == pytest.approx(b[j] - (T[0][j] + T[1][j]), rel=1e-13)
    S = sum(sum(row) for row in T)
    assert r["obj"] == pytest.approx(-eta * S + float(alpha @ a) + float(beta @ b), rel=1e-14)


@pytest.mark.parametrize("n,m,eta", [(5, 7, 0.3), (9, 4, 0.05)])
def test_separable_cost_closed_form(n, m, eta):
    # M_ij = u_i + v_j: alpha = eta*log a + u + t, beta = eta*log b + v - t gives T = a b^T exactly,
    # zero gradient and L* = -eta + sum a_i(eta log a_i + u_i) + sum b_j(eta log b_j + v_j).
    rng = np.random.default_rng(7)
    u = rng.uniform(0, 0.5, n); v = rng.uniform(0, 0.5, m)
    M = u[:, None] + v[None, :]
    a = rng.uniform(0.5, 1.5, n); a /= a.sum()
    b = rng.uniform(0.5, 1.5, m); b /= b.sum()
    t = 0.123
    alpha = eta * np.log(a) + u + t
    beta = eta * np.log(b) + v - t
    r = oracle.dual_eval(M, a, b, alpha, beta, eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    np.testing.assert_allclose(T, np.outer(a, b), rtol=1e-13)
    np.testing.assert_allclose(r["row_sum"], a, rtol=1e-13)
    np.testing.assert_allclose(r["col_sum"], b, rtol=1e-13)
    assert np.abs(r["grad_alpha"]).max() < 1e-14 and np.abs(r["grad_beta"]).max() < 1e-14
    Lstar = -eta + float(a @ (eta * np.log(a) + u)) + float(b @ (eta * np.log(b) + v))
    assert r["obj"] == pytest.approx(Lstar, rel=1e-13)
    # Sinkhorn reaches the optimum in ONE sweep from any start (up to the gauge shift)
    a0 = rng.standard_normal(n); b0 = rng.standard_normal(m)
    al, be = oracle.sinkhorn_sweeps(M, a, b, eta, 1, a0, b0)
    r1 = oracle.dual_eval(M, a, b, al, be, eta)
    assert np.abs(r1["grad_alpha"]).max() < 1e-13 and np.abs(r1["grad_beta"]).max() < 1e-13
    shift = (al - alpha)
    np.testing.assert_allclose(shift, shift[0], atol=1e-12)
    np.testing.assert_allclose(be - beta, -shift[0], atol=1e-12)


# ------------------------------------------------------------------- calculus

@pytest.mark.parametrize("n,m", [(4, 6), (7, 3)])
def test_gradient_matches_central_differences(n, m):
    eta = 0.5
    M, a, b, alpha, beta = small(n, m, 11, eta)
    g = oracle.dual_eval(M, a, b, alpha, beta, eta)
    h = 1e-5

    def L(al, be):
        return oracle.dual_eval(M, a, b, al, be, eta)["obj"]

    for i in range(n):
        e = np.zeros(n); e[i] = h
        fd = (L(alpha + e, beta) - L(alpha - e, beta)) / (2 * h)
        assert fd == pytest.approx(g["grad_alpha"][i], rel=1e-7, abs=1e-9)
    for j in range(m):
        e = np.zeros(m); e[j] = h
        fd = (L(alpha, beta + e) - L(alpha, beta - e)) / (2 * h)
        assert fd == pytest.approx(g["grad_beta"][j], rel=1e-7, abs=1e-9)


def test_csr_values_are_mixed_second_differences():
    # d^2 L / d alpha_i d beta_j = -T_ij / eta  (off-diagonal Hessian block, Sec. 3.1)
    n, m, eta = 4, 5, 0.6
    M, a, b, alpha, beta = small(n, m, 21, eta)
    row_ptr, col_idx, val = oracle.sparsify_csr(M, alpha, beta, eta, 0.0)   # keep everything
    assert row_ptr[-1] == n * m
    h = 1e-3

    def L(al, be):
        return oracle.dual_eval(M, a, b, al, be, eta)["obj"]

    for i in range(n):
        for p in range(row_ptr[i], row_ptr[i + 1]):
            j = col_idx[p]
            ei = np.zeros(n); ei[i] = h
            ej = np.zeros(m); ej[j] = h
            d2 = (L(alpha + ei, beta + ej) - L(alpha + ei, beta - ej)
                  - L(alpha - ei, beta + ej) + L(alpha - ei, beta - ej)) / (4 * h * h)
            assert -eta * d2 == pytest.approx(val[p], rel=1e-4)


# ----------------------------------------------------------------- identities

@pytest.mark.parametrize("name,n,m", [("c1", 60, 45), ("c3", 50, 70), ("c4", 80, 30), ("syn2", 32, 32)])
def test_sum_invariants_and_objective_assembly(name, n, m):
    p = W.make_problem(name, n=n, m=m)
    M, a, b = p.host()
    rng = np.random.default_rng(3)
    alpha = 0.05 * rng.standard_normal(n); beta = 0.05 * rng.standard_normal(m)
    eta = max(p.eta, 0.01)
    r = oracle.dual_eval(M, a, b, alpha, beta, eta)
    S_r, S_c = r["row_sum"].sum(), r["col_sum"].sum()
    assert S_r == pytest.approx(S_c, rel=1e-13)
    assert r["obj"] == pytest.approx(-eta * S_r + alpha @ a + beta @ b, rel=1e-12, abs=1e-13 * eta * S_r)
    np.testing.assert_allclose(r["grad_alpha"], a - r["row_sum"], rtol=0, atol=1e-15 * max(1, r["row_sum"].max()))
    np.testing.assert_allclose(r["grad_beta"], b - r["col_sum"], rtol=0, atol=1e-15 * max(1, r["col_sum"].max()))


def test_gauge_invariance():
    # L(alpha + c 1, beta - c 1) = L(alpha, beta) when sum a = sum b  (Sec. 1)
    n, m, eta = 12, 9, 0.2
    M, a, b, alpha, beta = small(n, m, 5, eta)
    r0 = oracle.dual_eval(M, a, b, alpha, beta, eta)
    r1 = oracle.dual_eval(M, a, b, alpha + 0.37, beta - 0.37, eta)
    assert r1["obj"] == pytest.approx(r0["obj"], rel=1e-13)
    np.testing.assert_allclose(r1["row_sum"], r0["row_sum"], rtol=1e-13)
    np.testing.assert_allclose(r1["col_sum"], r0["col_sum"], rtol=1e-13)
    delta = np.median(oracle.plan_dense(M, alpha, beta, eta))
    p0 = oracle.sparsify_csr(M, alpha, beta, eta, delta * (1 + 1e-9))
    p1 = oracle.sparsify_csr(M, alpha + 0.37, beta - 0.37, eta, delta * (1 + 1e-9))
    np.testing.assert_array_equal(p0[0], p1[0])
    np.testing.assert_array_equal(p0[1], p1[1])


def test_duality_gap_identity():
    # L_p - L_d = alpha^T (T1 - a) + beta^T (T^T 1 - b), with L_p = <T,M> + eta sum T log T - eta sum T  (App. A.5)
    n, m, eta = 10, 14, 0.3
    M, a, b, alpha, beta = small(n, m, 9, eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    r = oracle.dual_eval(M, a, b, alpha, beta, eta)
    Lp = (T * M).sum() + eta * (T * np.log(T)).sum() - eta * T.sum()
    gap = alpha @ (r["row_sum"] - a) + beta @ (r["col_sum"] - b)
    assert Lp - r["obj"] == pytest.approx(gap, rel=1e-11)
    # and the same through the gradient outputs (sign check: grad = marginal - sums)
    assert Lp - r["obj"] == pytest.approx(-(alpha @ r["grad_alpha"]) - (beta @ r["grad_beta"]), rel=1e-11)


# --------------------------------------------------------------- optimisation

@pytest.mark.parametrize("name,n,m", [("c1", 40, 50), ("c3", 64, 48), ("c4", 30, 20)])
def test_half_step_is_exact_block_maximiser(name, n, m):
    p = W.make_problem(name, n=n, m=m)
    M, a, b = p.host()
    eta = p.eta
    rng = np.random.default_rng(1)
    alpha = 0.1 * rng.standard_normal(n); beta = 0.1 * rng.standard_normal(m)
    L0 = oracle.dual_eval(M, a, b, alpha, beta, eta)["obj"]
    alpha1 = oracle.sinkhorn_half_step(M, a, alpha, beta, eta, 0)
    r1 = oracle.dual_eval(M, a, b, alpha1, beta, eta)
    np.testing.assert_allclose(r1["row_sum"], a, rtol=1e-11)          # its block of the gradient vanishes
    beta1 = oracle.sinkhorn_half_step(M, b, alpha1, beta, eta, 1)
    r2 = oracle.dual_eval(M, a, b, alpha1, beta1, eta)
    np.testing.assert_allclose(r2["col_sum"], b, rtol=1e-11)
    assert L0 <= r1["obj"] + 1e-15 and r1["obj"] <= r2["obj"] + 1e-15  # ascent
    # a perturbation of the block just maximised cannot increase L
    for _ in range(5):
        dpert = 1e-4 * rng.standard_normal(m)
        assert oracle.dual_eval(M, a, b, alpha1, beta1 + dpert, eta)["obj"] <= r2["obj"] + 1e-15


def test_converged_sinkhorn_has_vanishing_gradient():
    p = W.make_problem("c1", n=30, m=25)
    M, a, b = p.host()
    eta = 0.05
    al, be = oracle.sinkhorn_sweeps(M, a, b, eta, 3000)
    r = oracle.dual_eval(M, a, b, al, be, eta)
    err = np.abs(r["grad_alpha"]).sum() + np.abs(r["grad_beta"]).sum()   # marginal error, Sec. 6.1
    assert err < 1e-12


def test_monotone_ascent_over_sweeps():
    p = W.make_problem("syn2", n=32, m=32)       # the paper's small illustration problem, App. A.2
    M, a, b = p.host()
    eta = 0.001
    al = np.zeros(32); be = np.zeros(32)
    last = -np.inf
    for _ in range(10):
        al = oracle.sinkhorn_half_step(M, a, al, be, eta, 0)
        L1 = oracle.dual_eval(M, a, b, al, be, eta)["obj"]
        be = oracle.sinkhorn_half_step(M, b, al, be, eta, 1)
        L2 = oracle.dual_eval(M, a, b, al, be, eta)["obj"]
        assert last <= L1 + 1e-15 and L1 <= L2 + 1e-15
        last = L2
    assert np.all(np.isfinite(al)) and np.all(np.isfinite(be))


def test_lse_form_equals_ratio_form():
    # alpha_new = alpha + eta (log a - log r) wherever r > 0: ties the half-step to dual_eval's sums
    n, m, eta = 20, 30, 0.1
    M, a, b, alpha, beta = small(n, m, 13, eta)
    r = oracle.dual_eval(M, a, b, alpha, beta, eta)
    np.testing.assert_allclose(oracle.sinkhorn_half_step(M, a, alpha, beta, eta, 0),
                               alpha + eta * (np.log(a) - np.log(r["row_sum"])), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.sinkhorn_half_step(M, b, alpha, beta, eta, 1),
                               beta + eta * (np.log(b) - np.log(r["col_sum"])), rtol=1e-12, atol=1e-14)


# ----------------------------------------------------------- library routines

@pytest.mark.parametrize("n,m,eta", [(17, 33, 0.01), (40, 12, 0.001)])
def test_half_steps_against_scipy_logsumexp(n, m, eta):
    M, a, b, alpha, beta = small(n, m, 17, eta)
    ref_a = eta * np.log(a) - eta * scipy.special.logsumexp((beta[None, :] - M) / eta, axis=1)
    ref_b = eta * np.log(b) - eta * scipy.special.logsumexp((alpha[:, None] - M) / eta, axis=0)
    np.testing.assert_allclose(oracle.sinkhorn_half_step(M, a, alpha, beta, eta, 0), ref_a, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(oracle.sinkhorn_half_step(M, b, alpha, beta, eta, 1), ref_b, rtol=1e-13, atol=1e-15)


def test_small_eta_does_not_underflow_half_step():
    # eta = 0.001 and costs near 1: exp(-M/eta) is exactly 0, the log-domain step must stay finite
    n, m, eta = 6, 8, 0.001
    rng = np.random.default_rng(2)
    M = 0.9 + 0.1 * rng.uniform(size=(n, m))
    a = np.full(n, 1 / n); b = np.full(m, 1 / m)
    al = oracle.sinkhorn_half_step(M, a, np.zeros(n), np.zeros(m), eta, 0)
    assert np.all(np.isfinite(al))
    assert np.all(oracle.dual_eval(M, a, b, np.zeros(n), np.zeros(m), eta)["row_sum"] == 0.0)
    np.testing.assert_allclose(oracle.dual_eval(M, a, b, al, np.zeros(m), eta)["row_sum"], a, rtol=1e-10)


@pytest.mark.parametrize("n,m,k", [(30, 40, 1), (30, 40, 12), (25, 16, 399), (25, 16, 400)])
def test_topk_threshold_against_numpy_sort(n, m, k):
    eta = 0.2
    M, a, b, alpha, beta = small(n, m, 23, eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    ref = np.sort(T.ravel())[::-1][k - 1]
    delta = oracle.topk_threshold(M, alpha, beta, eta, k)
    assert delta == ref
    row_ptr, col_idx, val = oracle.sparsify_csr(M, alpha, beta, eta, delta)
    assert row_ptr[-1] == k                     # no ties in continuous random data


def test_topk_threshold_when_many_entries_share_their_leading_bits():
    # costs that differ in the 9th digit only: all T_ij agree in their leading 20 bits, so the selection
    # has to order a crowded bucket; with exact ties the threshold is the tied value
    rng = np.random.default_rng(41)
    n, m, eta = 40, 50, 0.5
    M = 0.5 + 1e-9 * rng.random((n, m))
    alpha = np.zeros(n); beta = np.zeros(m)
    T = oracle.plan_dense(M, alpha, beta, eta)
    order = np.sort(T.ravel())[::-1]
    assert order[0] / order[-1] < 1 + 1e-8
    for k in (1, 2, 777, n * m - 1, n * m):
        assert oracle.topk_threshold(M, alpha, beta, eta, k) == order[k - 1], k
    M[3, :] = M[3, 0]                          # 50 equal entries
    T = oracle.plan_dense(M, alpha, beta, eta)
    order = np.sort(T.ravel())[::-1]
    for k in (5, 1000, 1999):
        assert oracle.topk_threshold(M, alpha, beta, eta, k) == order[k - 1], k


def test_sweep_is_alpha_step_then_beta_step():
    # the beta half-step comes last, so after any number of sweeps the column marginals are exact and the
    # whole error sits in the row marginals (which the next alpha half-step would remove)
    eta = 0.3
    M, a, b, alpha0, beta0 = small(12, 17, 43, eta)
    for sweeps in (1, 3):
        alpha, beta = oracle.sinkhorn_sweeps(M, a, b, eta, sweeps)
        ev = oracle.dual_eval(M, a, b, alpha, beta, eta)
        np.testing.assert_allclose(ev["col_sum"], b, rtol=1e-13)
        assert np.abs(ev["row_sum"] - a).max() > 1e-6 * a.max()
    one = oracle.sinkhorn_sweeps(M, a, b, eta, 1)
    al = oracle.sinkhorn_half_step(M, a, np.zeros(12), np.zeros(17), eta, 0)
    be = oracle.sinkhorn_half_step(M, b, al, np.zeros(17), eta, 1)
    np.testing.assert_array_equal(one[0], al); np.testing.assert_array_equal(one[1], be)
    cont = oracle.sinkhorn_sweeps(M, a, b, eta, 2, alpha0=one[0], beta0=one[1])
    three = oracle.sinkhorn_sweeps(M, a, b, eta, 3)
    np.testing.assert_array_equal(cont[0], three[0]); np.testing.assert_array_equal(cont[1], three[1])


@pytest.mark.parametrize("n,m", [(13, 29), (31, 8)])
def test_csr_layout_against_scipy_sparse(n, m):
    eta = 0.15
    M, a, b, alpha, beta = small(n, m, 29, eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    delta = np.quantile(T, 0.8)
    ref = scipy.sparse.csr_matrix(np.where(T >= delta, T, 0.0))
    ref.sort_indices()
    row_ptr, col_idx, val = oracle.sparsify_csr(M, alpha, beta, eta, delta)
    np.testing.assert_array_equal(row_ptr, ref.indptr)
    np.testing.assert_array_equal(col_idx, ref.indices)
    np.testing.assert_array_equal(val, ref.data)
    assert row_ptr.dtype == np.int64 and col_idx.dtype == np.int32
    for i in range(n):
        assert np.all(np.diff(col_idx[row_ptr[i]:row_ptr[i + 1]]) > 0)


def test_csr_degenerate_thresholds():
    n, m, eta = 9, 11, 0.3
    M, a, b, alpha, beta = small(n, m, 31, eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    rp, ci, v = oracle.sparsify_csr(M, alpha, beta, eta, T.min())       # keeps everything
    assert rp[-1] == n * m
    np.testing.assert_array_equal(v.reshape(n, m), T)
    np.testing.assert_array_equal(ci.reshape(n, m), np.tile(np.arange(m), (n, 1)))
    r = oracle.dual_eval(M, a, b, alpha, beta, eta)
    np.testing.assert_allclose(np.add.reduceat(v, rp[:-1]), r["row_sum"], rtol=1e-14)
    rp, ci, v = oracle.sparsify_csr(M, alpha, beta, eta, np.inf)        # keeps nothing
    assert rp[-1] == 0 and len(ci) == 0 and np.all(rp == 0)
    rp, ci, v = oracle.sparsify_csr(M, alpha, beta, eta, T.max())       # exactly the maximum (>= is inclusive)
    assert rp[-1] == 1 and v[0] == T.max()


def test_leading_dimension_is_respected():
    n, m, eta = 7, 10, 0.4
    Mfull, a, b, alpha, beta = small(n, m + 5, 37, eta)
    beta = beta[:m]; b = b[:m] / b[:m].sum()
    view = Mfull[:, :m]                        # ldM = m + 5
    packed = np.ascontiguousarray(view)
    r0 = oracle.dual_eval(packed, a, b, alpha, beta, eta)
    r1 = oracle.dual_eval(view, a, b, alpha, beta, eta)
    assert r0["obj"] == r1["obj"]
    np.testing.assert_array_equal(r0["col_sum"], r1["col_sum"])
    np.testing.assert_array_equal(oracle.sinkhorn_half_step(view, b, alpha, beta, eta, 1),
                                  oracle.sinkhorn_half_step(packed, b, alpha, beta, eta, 1))
    np.testing.assert_array_equal(oracle.sinkhorn_half_step(view, a, alpha, beta, eta, 0),
                                  oracle.sinkhorn_half_step(packed, a, alpha, beta, eta, 0))
    # every other function that reads M: the strided view and the packed copy give the same bits, and the
    # packed result is what the dense plan says
    T = oracle.plan_dense(packed, alpha, beta, eta)
    np.testing.assert_array_equal(oracle.plan_dense(view, alpha, beta, eta), T)
    delta = float(np.sort(T.ravel())[-20])
    for got in (oracle.sparsify_csr(view, alpha, beta, eta, delta), oracle.sparsify_csr(packed, alpha, beta, eta, delta)):
        ref = scipy.sparse.csr_matrix(np.where(T >= delta, T, 0.0)); ref.sort_indices()
        np.testing.assert_array_equal(got[0], ref.indptr); np.testing.assert_array_equal(got[1], ref.indices)
        np.testing.assert_array_equal(got[2], ref.data)
    assert oracle.topk_threshold(view, alpha, beta, eta, 20) == delta
    row_ptr = np.arange(n + 1, dtype=np.int64) * 3
    col_idx = np.tile(np.array([0, 4, m - 1], dtype=np.int32), n)
    np.testing.assert_array_equal(oracle.pattern_values(view, alpha, beta, eta, row_ptr, col_idx), T[:, [0, 4, m - 1]].ravel())
    assert oracle.dual_metrics(view, a, b, alpha, beta, eta) == oracle.dual_metrics(packed, a, b, alpha, beta, eta)


# ---------------------------------------------------------------- brute force

@pytest.mark.parametrize("n,m,eta,seed", [(1, 1, 0.5, 0), (3, 8, 0.1, 1), (8, 5, 0.02, 2), (6, 6, 1.0, 3)])
def test_brute_force_tiny(n, m, eta, seed):
    M, a, b, alpha, beta = small(n, m, seed, eta)
    T = [[math.exp(((alpha[i] + beta[j]) - M[i, j]) / eta) for j in range(m)] for i in range(n)]
    r = oracle.dual_eval(M, a, b, alpha, beta, eta)
    rows = [math.fsum(T[i]) for i in range(n)]
    cols = [math.fsum(T[i][j] for i in range(n)) for j in range(m)]
    np.testing.assert_allclose(r["row_sum"], rows, rtol=2e-16)
    np.testing.assert_allclose(r["col_sum"], cols, rtol=2e-16)
    L = math.fsum([-eta * math.fsum(rows)] + [alpha[i] * a[i] for i in range(n)] + [beta[j] * b[j] for j in range(m)])
    assert r["obj"] == pytest.approx(L, rel=1e-14, abs=1e-16)
    flat = sorted((T[i][j] for i in range(n) for j in range(m)), reverse=True)
    delta = flat[(n * m) // 3]
    rp, ci, v = oracle.sparsify_csr(M, alpha, beta, eta, delta)
    exp_cols = [[j for j in range(m) if T[i][j] >= delta] for i in range(n)]
    assert list(rp) == [0] + list(np.cumsum([len(c) for c in exp_cols]))
    assert list(ci) == [j for c in exp_cols for j in c]
    assert list(v) == [T[i][j] for i, c in enumerate(exp_cols) for j in c]
    for i in range(n):
        xs = [(beta[j] - M[i, j]) / eta for j in range(m)]
        mx = max(xs)
        lse = mx + math.log(math.fsum(math.exp(x - mx) for x in xs))
        assert oracle.sinkhorn_half_step(M, a, alpha, beta, eta, 0)[i] == pytest.approx(
            eta * math.log(a[i]) - eta * lse, rel=1e-14, abs=1e-16)
    for j in range(m):
        xs = [(alpha[i] - M[i, j]) / eta for i in range(n)]
        mx = max(xs)
        lse = mx + math.log(math.fsum(math.exp(x - mx) for x in xs))
        assert oracle.sinkhorn_half_step(M, b, alpha, beta, eta, 1)[j] == pytest.approx(
            eta * math.log(b[j]) - eta * lse, rel=1e-14, abs=1e-16)


def test_thread_count_does_not_change_results():
    p = W.make_problem("c1", n=203, m=97)
    M, a, b = p.host()
    rng = np.random.default_rng(4)
    alpha = 0.01 * rng.standard_normal(203); beta = 0.01 * rng.standard_normal(97)
    keep = oracle.get_max_threads()
    try:
        oracle.set_threads(1)
        r1 = oracle.dual_eval(M, a, b, alpha, beta, 0.01)
        h1 = oracle.sinkhorn_half_step(M, b, alpha, beta, 0.01, 1)
        oracle.set_threads(5)
        r5 = oracle.dual_eval(M, a, b, alpha, beta, 0.01)
        h5 = oracle.sinkhorn_half_step(M, b, alpha, beta, 0.01, 1)
    finally:
        oracle.set_threads(keep)
    np.testing.assert_array_equal(r1["row_sum"], r5["row_sum"])
    np.testing.assert_allclose(r1["col_sum"], r5["col_sum"], rtol=3e-16)
    assert r1["obj"] == pytest.approx(r5["obj"], rel=1e-15)
    np.testing.assert_array_equal(h1, h5)
