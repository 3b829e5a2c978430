"""Conjugate gradients on the sparse term and the quasi-Newton direction (Algorithm 1, lines 3-7) on the GPU
against the oracle's iteration and against what the solution must satisfy."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_08793_amd import workloads as W
from paper_2605_08793_amd.driver import DirectionSolver, DualPass, SparseTerm

pytestmark = pytest.mark.gpu


def dev(x, dtype=torch.float64):
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda", dtype=dtype)


def setup(M, a, b, alpha, beta, eta, delta, Md=None):
    n, m = M.shape
    Md = dev(M) if Md is None else Md
    rp, ci, val = oracle.sparsify_csr(M, alpha, beta, eta, delta)
    nnz = int(rp[-1])
    dp = DualPass(n, m, capacity=nnz + 64)
    dp.dual_eval_sparsify(Md, dev(a), dev(b), dev(alpha), dev(beta), eta, delta)
    g_rp, g_ci, g_v, overflow = dp.csr_host()
    np.testing.assert_array_equal(g_rp, rp); np.testing.assert_array_equal(g_ci, ci)
    term = SparseTerm(n, m, dp.row_ptr, dp.col_idx, nnz)
    term.refresh(Md, dev(alpha), dev(beta), eta)
    ev = oracle.dual_eval(M, a, b, alpha, beta, eta)
    g = np.concatenate([ev["row_sum"] - a, (ev["col_sum"] - b)[:-1]])
    return dp, term, (rp, ci, val), ev, g


def solution_tolerance(eta, tau, r, c, g, x, rtol):
    """How far two iterates that both stopped at ||residual|| <= rtol ||g|| can be apart, relative to ||x||.
    A = H_Omega + tau I has its spectrum in [tau, lmax] with lmax <= 2 max(T1, T^T1) / eta + tau (Gershgorin: the
    off-diagonal row sums of H_Omega are at most the diagonal, Theorem 1's argument), so each iterate is within
    ||A^-1|| ||residual|| <= rtol ||g|| / tau of the solution; on top of that fp64 conjugate gradients cannot do
    better than about eps * lmax / tau."""
    lmax = 2.0 * max(np.max(r), np.max(c)) / eta + tau
    return 2.5 * rtol * np.linalg.norm(g) / (tau * np.linalg.norm(x)) + 200 * np.finfo(float).eps * lmax / tau


def check_direction(M, a, b, alpha, beta, eta, delta, tau, rtol, label, Md=None, seed=0, expect_rank_two=True):
    n, m = M.shape
    print(f"[direction] {label} n={n} m={m} eta={eta} tau={tau} rtol={rtol}", flush=True)
    dp, term, (rp, ci, val), ev, g = setup(M, a, b, alpha, beta, eta, delta, Md)
    r, c = ev["row_sum"], ev["col_sum"]
    rd, cd = dev(r), dev(c)
    solver = DirectionSolver(term)
    N = n + m - 1
    # 1. the solve itself
    x = torch.full((N,), float("nan"), dtype=torch.float64, device="cuda")
    its, conv, rel = solver.solve(eta, tau, rd, cd, dev(g), x, rtol=rtol, max_iter=2000)
    o_x, o_its, o_rel = oracle.pcg_solve(n, m, eta, tau, rp, ci, val, r, c, g, rtol=rtol, max_iter=2000)
    assert conv and rel <= rtol
    assert abs(its - o_its) <= 1, (its, o_its)
    xg = x.cpu().numpy()
    # the residual, evaluated by the oracle's product, is what the iteration claims (up to the rounding of r)
    res = np.linalg.norm(oracle.hessian_matvec(n, m, eta, tau, rp, ci, val, r, c, xg) - g) / np.linalg.norm(g)
    assert res <= 1.5 * rtol + 1e-13, res
    x_tol = solution_tolerance(eta, tau, r, c, g, o_x, rtol)
    print(f"[direction] iterations {its} (oracle {o_its}), |x - x_oracle| / |x| = {np.linalg.norm(xg - o_x) / np.linalg.norm(o_x):.2e}"
          f" (bound {x_tol:.2e})", flush=True)
    # the two iterations run the same recurrences on products that agree to rounding: when they stop after the same
    # number of steps the iterates agree to the 1e-10 of the other parity tests (observed: 1e-15); when the stopping
    # test falls on different sides for the two, they are one step apart and only the bound above holds
    if its == o_its:
        x_tol = 1e-10
    assert np.linalg.norm(xg - o_x) <= x_tol * np.linalg.norm(o_x), (np.linalg.norm(xg - o_x) / np.linalg.norm(o_x), x_tol)
    # the same call again gives the same bits (fixed summation order)
    x2 = torch.empty_like(x)
    solver.solve(eta, tau, rd, cd, dev(g), x2, rtol=rtol, max_iter=2000)
    assert torch.equal(x, x2)
    # 1b. the same system through the Schur complement of its first block: the oracle's reduced iteration, the
    # residual of the WHOLE system as the oracle's product sees it, half the iterations, the same bits on a repeated
    # call and when the iterations are enqueued in small portions
    xr = torch.full((N,), float("nan"), dtype=torch.float64, device="cuda")
    r_its, r_conv, r_rel = solver.solve(eta, tau, rd, cd, dev(g), xr, rtol=rtol, max_iter=2000, reduced=True)
    o_xr, o_rits, o_rrel = oracle.pcg_solve_reduced(n, m, eta, tau, rp, ci, val, r, c, g, rtol=rtol, max_iter=2000)
    assert r_conv and r_rel <= rtol
    assert abs(r_its - o_rits) <= 1, (r_its, o_rits)
    assert r_its <= (its + 1) // 2 + 1, (r_its, its)
    xrg = xr.cpu().numpy()
    res_r = np.linalg.norm(oracle.hessian_matvec(n, m, eta, tau, rp, ci, val, r, c, xrg) - g) / np.linalg.norm(g)
    assert res_r <= 1.5 * rtol + 1e-13, res_r
    xr_tol = 1e-10 if r_its == o_rits else solution_tolerance(eta, tau, r, c, g, o_xr, rtol)
    err_r = np.linalg.norm(xrg - o_xr) / np.linalg.norm(o_xr)
    print(f"[direction] reduced: iterations {r_its} (oracle {o_rits}), |x - x_oracle| / |x| = {err_r:.2e} (bound {xr_tol:.2e})", flush=True)
    assert err_r <= xr_tol, (err_r, xr_tol)
    for portion in (24, 3):
        xr2 = torch.full((N,), float("nan"), dtype=torch.float64, device="cuda")
        again = solver.solve(eta, tau, rd, cd, dev(g), xr2, rtol=rtol, max_iter=2000, portion=portion, reduced=True)
        assert again == (r_its, r_conv, r_rel) and torch.equal(xr, xr2), portion
    # two systems in one iteration: bit for bit what two single solves give, each stopping on its own
    # (the iteration on the whole matrix, then the reduced one)
    rng = np.random.default_rng(seed)
    for rhs_b in (dev(rng.standard_normal(N) * np.exp(3 * rng.standard_normal(N))), torch.zeros(N, dtype=torch.float64, device="cuda")):
        for reduced, first, x_first in ((False, (its, conv, rel), x), (True, (r_its, r_conv, r_rel), xr)):
            xb = torch.full((N,), float("nan"), dtype=torch.float64, device="cuda")
            single_b = solver.solve(eta, tau, rd, cd, rhs_b, xb, rtol=rtol, max_iter=2000, reduced=reduced)
            xa2 = torch.full((N,), float("nan"), dtype=torch.float64, device="cuda"); xb2 = xa2.clone()
            pair = solver.solve2(eta, tau, rd, cd, dev(g), rhs_b, xa2, xb2, rtol=rtol, max_iter=2000, reduced=reduced,
                                 portion=24 if not reduced else 5)
            assert pair[0] == first and pair[1] == single_b, (reduced, pair, first, single_b)
            assert torch.equal(xa2, x_first) and torch.equal(xb2, xb), reduced
    # 2. the direction with and without the rank-two term
    s = 0.1 * eta * rng.standard_normal(N)
    As = oracle.hessian_matvec(n, m, eta, tau, rp, ci, val, r, c, s)
    y = As * (1 + 0.2 * rng.random(N))            # a secant pair with positive curvature
    # (with the large plan entries of a perturbed dual point the curvature test of Algorithm 1, line 5, which is
    # not scale-free, rejects even this pair: then the oracle says so and the GPU must agree)
    for label2, sp, yp, expect in (("rank two", s, y, expect_rank_two), ("negative curvature", s, -y, False),
                                   ("first step", None, None, False)):
      for reduced in (False, True):
        o_d, o_used = oracle.quasi_newton_direction(n, m, eta, tau, rp, ci, val, r, c, g, sp, yp, rtol=rtol, max_iter=2000,
                                                    reduced=reduced)
        if expect is None:                        # random cases: whether the pair passes the curvature test is the oracle's call
            expect = o_used
        assert o_used == expect
        solver.direction(eta, tau, rd, cd, dev(g), None if sp is None else dev(sp), None if yp is None else dev(yp),
                         rtol=rtol, max_iter=2000, reduced=reduced)
        torch.cuda.synchronize()
        d = solver.d.cpu().numpy()
        info = solver.info.cpu().numpy()
        assert bool(info[0]) == expect, label2
        # the direction combines two such solves (for g and for y^-) through the 2 x 2 system of the rank-two term,
        # whose conditioning can multiply their errors: ten times the bound of one solve, at most the old 1e-6
        same_steps = (r_its == o_rits) if reduced else (its == o_its)
        d_tol = 1e-9 if same_steps else min(1e-6, 10 * max(x_tol, solution_tolerance(eta, tau, r, c, g if yp is None else yp, o_d, rtol)))
        err_d = np.linalg.norm(d - o_d) / np.linalg.norm(o_d)
        print(f"[direction] {label2}{' (reduced)' if reduced else ''}: |d - d_oracle| / |d| = {err_d:.2e} (bound {d_tol:.2e})", flush=True)
        assert err_d <= d_tol, (label2, reduced, err_d, d_tol)
        assert g @ d < 0                          # a descent direction for f
    return its


# (the last three: sizes at which the product of a single solve keeps its vector in LDS while that of a pair of
# solves gathers from memory, and sizes at which both gather from memory; the pair must still equal the singles)
# (the last two: more rows, or columns, than 64 per wave of the product kernels, whose waves then take their items in
# several batches)
@pytest.mark.parametrize("n,m", [(1, 1), (5, 3), (17, 513), (130, 64), (300, 1537), (1030, 130), (12000, 120),
                                 (150, 12500), (20500, 90), (300_000, 3), (3, 300_000)])
def test_small_shapes(n, m):
    eta = 0.3
    M, a, b, alpha, beta = W.random_small(n, m, seed=900 + n + m, eta=eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    delta = float(np.quantile(T, 0.7)) if n * m > 1 else float(T[0, 0]) * 0.5
    check_direction(M, a, b, alpha, beta, eta, delta, tau=0.05, rtol=1e-11, label="random_small", seed=n)


def test_random_cases():
    rng = np.random.default_rng(31)
    for it in range(16):
        kind = int(rng.integers(0, 3))
        if kind == 0:
            n, m = int(rng.integers(1, 200)), int(rng.integers(2, 2500))
        elif kind == 1:
            n, m = int(rng.integers(2, 2500)), int(rng.integers(1, 200))
        else:
            n, m = int(rng.integers(200, 1200)), int(rng.integers(200, 1200))
        eta = float(rng.choice([0.5, 0.2]))
        M, a, b, alpha, beta = W.random_small(n, m, seed=int(rng.integers(1 << 30)), eta=eta)
        T = oracle.plan_dense(M, alpha, beta, eta)
        delta = float(np.quantile(T, float(rng.choice([0.5, 0.9, 0.98]))))
        check_direction(M, a, b, alpha, beta, eta, delta, tau=float(rng.choice([0.02, 0.2])), rtol=1e-10,
                        label=f"random {it}", seed=it, expect_rank_two=None)


@pytest.mark.parametrize("name,n,m,sweeps", [("c1", None, None, 20), ("c3", 1500, 2300, 10), ("c4", 3000, 700, 5)])
def test_workloads_reduced(name, n, m, sweeps):
    p = W.make_problem(name, device="cuda", n=n, m=m)
    M, a, b = p.host()
    alpha, beta = oracle.sinkhorn_sweeps(M, a, b, p.eta, sweeps)
    if p.noise_alpha is not None:
        alpha = alpha + p.noise_alpha; beta = beta + p.noise_beta
    delta = oracle.topk_threshold(M, alpha, beta, p.eta, p.k_keep()) * (1 - 1e-7)
    ev = oracle.dual_eval(M, a, b, alpha, beta, p.eta)
    gnorm = float(np.sqrt((ev["grad_alpha"] ** 2).sum() + (ev["grad_beta"][:-1] ** 2).sum()))
    tau = min(1e-3, gnorm)                        # Algorithm 1, line 6 with tau_max = 1e-3
    Tmax = oracle.plan_dense(M[:50], alpha[:50], beta, p.eta).max()
    check_direction(M, a, b, alpha, beta, p.eta, delta, tau, rtol=1e-9, label=name, Md=p.M,
                    expect_rank_two=bool(Tmax / p.eta < 1e5))


def test_c3_full_size():
    """The direction solve at the benchmark size (N = 39 999, 2 * 10^6 pattern entries), at the stored dual point:
    iteration count, residual re-evaluated by the oracle's product, and the solution against the oracle's iteration."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "dual_c3.npz")
    if not os.path.exists(path):
        pytest.skip(f"{path} missing")
    z = np.load(path, allow_pickle=False)
    p = W.make_problem("c3", device="cuda")
    M, a, b = p.host()
    alpha, beta = z["alpha"], z["beta"]
    ev = oracle.dual_eval(M, a, b, alpha, beta, p.eta)
    gnorm = float(np.sqrt((ev["grad_alpha"] ** 2).sum() + (ev["grad_beta"][:-1] ** 2).sum()))
    tau = min(1e-3, gnorm)                        # Algorithm 1, line 6 with tau_max = 1e-3
    its = check_direction(M, a, b, alpha, beta, p.eta, float(z["delta"]) * (1 - 1e-7), tau, rtol=1e-8, label="c3 full size",
                          Md=p.M, expect_rank_two=None)
    assert its < 100


def test_zero_right_hand_side_and_iteration_limit():
    n, m, eta, tau = 200, 300, 0.3, 0.01
    M, a, b, alpha, beta = W.random_small(n, m, seed=17, eta=eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    dp, term, (rp, ci, val), ev, g = setup(M, a, b, alpha, beta, eta, float(np.quantile(T, 0.6)))
    rd, cd = dev(ev["row_sum"]), dev(ev["col_sum"])
    solver = DirectionSolver(term)
    N = n + m - 1
    x = torch.full((N,), float("nan"), dtype=torch.float64, device="cuda")
    its, conv, rel = solver.solve(eta, tau, rd, cd, torch.zeros(N, dtype=torch.float64, device="cuda"), x)
    assert (its, conv, rel) == (0, True, 0.0) and not x.any()
    its, conv, rel = solver.solve(eta, tau, rd, cd, dev(g), x, rtol=1e-14, max_iter=3, portion=2)
    o_x, o_its, o_rel = oracle.pcg_solve(n, m, eta, tau, rp, ci, val, ev["row_sum"], ev["col_sum"], g, rtol=1e-14, max_iter=3)
    assert its == 3 == o_its and not conv
    assert abs(rel - o_rel) <= 1e-6 * o_rel
    np.testing.assert_allclose(x.cpu().numpy(), o_x, rtol=1e-9, atol=1e-12 * np.abs(o_x).max())
    # the reduced iteration: the same two cases
    its, conv, rel = solver.solve(eta, tau, rd, cd, torch.zeros(N, dtype=torch.float64, device="cuda"), x, reduced=True)
    assert (its, conv, rel) == (0, True, 0.0) and not x.any()
    # ... and a right-hand side whose solution has a zero second block: the reduced system's residual is rounding
    # noise from the start, below the tolerance relative to the whole right-hand side, so no iteration is needed
    x1 = np.random.default_rng(4).standard_normal(n)
    g0 = oracle.hessian_matvec(n, m, eta, tau, rp, ci, val, ev["row_sum"], ev["col_sum"], np.concatenate([x1, np.zeros(m - 1)]))
    its, conv, rel = solver.solve(eta, tau, rd, cd, dev(g0), x, rtol=1e-10, reduced=True)
    o_x, o_its, _ = oracle.pcg_solve_reduced(n, m, eta, tau, rp, ci, val, ev["row_sum"], ev["col_sum"], g0, rtol=1e-10)
    assert its == 0 == o_its and conv and rel <= 1e-10
    np.testing.assert_allclose(x.cpu().numpy()[:n], x1, rtol=1e-9, atol=1e-12)
    assert np.abs(x.cpu().numpy()[n:]).max() == 0.0
    its, conv, rel = solver.solve(eta, tau, rd, cd, dev(g), x, rtol=1e-14, max_iter=3, portion=2, reduced=True)
    o_x, o_its, o_rel = oracle.pcg_solve_reduced(n, m, eta, tau, rp, ci, val, ev["row_sum"], ev["col_sum"], g, rtol=1e-14, max_iter=3)
    assert its == 3 == o_its and not conv
    assert abs(rel - o_rel) <= 1e-6 * o_rel
    np.testing.assert_allclose(x.cpu().numpy(), o_x, rtol=1e-9, atol=1e-12 * np.abs(o_x).max())
