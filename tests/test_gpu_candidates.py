"""Optimality measures (App. A.5) and candidate generation / choice (Sec. 4.3) on the GPU against the oracle."""
import time

import numpy as np
import pytest
import torch

import oracle
from paper_2605_08793_amd import workloads as W
from paper_2605_08793_amd.driver import CandidateGenerator, DualPass
from parity_utils import assert_half_step_close

pytestmark = pytest.mark.gpu


def dev(x, dtype=torch.float64):
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda", dtype=dtype)


def check_metrics(M, a, b, alpha, beta, eta, Md=None, label=""):
    n, m = M.shape
    print(f"[metrics] {label} n={n} m={m} eta={eta}", flush=True)
    Md = dev(M) if Md is None else Md
    dp = DualPass(n, m)
    ad, bd, ald, bed = dev(a), dev(b), dev(alpha), dev(beta)
    dp.dual_eval(Md, ad, bd, ald, bed, eta)
    got = dp.metrics(ad, bd, ald, bed, eta).cpu().numpy()
    ref = oracle.dual_metrics(M, a, b, alpha, beta, eta)
    ev = oracle.dual_eval(M, a, b, alpha, beta, eta)
    r, c = ev["row_sum"], ev["col_sum"]
    # scales of the sums behind each number (R12-style: relative to what is added up, not to the result)
    s_primal = np.abs(alpha) @ r + np.abs(beta) @ c + eta * r.sum()
    s_gap = np.abs(alpha) @ (r + a) + np.abs(beta) @ (c + b)
    assert abs(got[0] - ref["primal"]) <= 1e-10 * s_primal, (got[0], ref["primal"])
    assert abs(got[1] - ref["gap"]) <= 1e-10 * s_gap, (got[1], ref["gap"])
    assert abs(got[2] - ref["marginal_error"]) <= 1e-10 * (r.sum() + c.sum() + 2.0), (got[2], ref["marginal_error"])
    assert abs(got[3] - ref["grad_norm"]) <= 1e-10 * np.sqrt(((r + a) ** 2).sum() + ((c + b) ** 2).sum())
    return got


@pytest.mark.parametrize("n,m", [(1, 1), (5, 3), (65, 1025), (1030, 130), (300, 1537)])
@pytest.mark.parametrize("eta", [0.5, 0.02])
def test_metrics_small_shapes(n, m, eta):
    M, a, b, alpha, beta = W.random_small(n, m, seed=700 + n + m, eta=eta)
    check_metrics(M, a, b, alpha, beta, eta, label="random_small")


def test_metrics_after_sweeps_go_to_zero():
    p = W.make_problem("c1", device="cuda")
    M, a, b = p.host()
    alpha, beta = oracle.sinkhorn_sweeps(M, a, b, p.eta, 200)
    got = check_metrics(M, a, b, alpha, beta, p.eta, Md=p.M, label="c1 after 200 sweeps")
    far = check_metrics(M, a, b, alpha + p.noise_alpha, beta + p.noise_beta, p.eta, Md=p.M, label="c1 perturbed")
    assert got[2] < 1e-3 * far[2] and abs(got[1]) < 1e-3 * abs(far[1])


@pytest.mark.parametrize("name,n,m", [("c3", 1500, 2300), ("c4", 3000, 700), ("c2", 1201, 999)])
def test_candidate_generation_and_choice(name, n, m):
    p = W.make_problem(name, device="cuda", n=n, m=m)
    M, a, b = p.host()
    eta = p.eta
    alpha0, beta0 = oracle.sinkhorn_sweeps(M, a, b, eta, 3)
    rng = np.random.default_rng(3)
    # two stand-ins for the quasi-Newton candidate: a good one (more ascent than the side stream gets) and a bad one
    good = oracle.sinkhorn_sweeps(M, a, b, eta, 6, alpha0, beta0)
    bad = (alpha0 + 0.5 * eta * rng.standard_normal(n), beta0 + 0.5 * eta * rng.standard_normal(m))
    side_ref = oracle.sinkhorn_sweeps(M, a, b, eta, 2, alpha0, beta0)
    gen = CandidateGenerator(n, m)
    main = DualPass(n, m)
    for label, cand_q in (("good q", good), ("bad q", bad)):
        print(f"[candidates] {name} {label}", flush=True)
        ald, bed = dev(alpha0), dev(beta0)
        gen.launch(p.M, p.a, p.b, ald, bed, eta, sweeps=2)
        time.sleep(0.01)                              # the host's serial work
        aq, bq = dev(cand_q[0]), dev(cand_q[1])
        out_a = torch.full((n,), float("nan"), dtype=torch.float64, device="cuda")
        out_b = torch.full((m,), float("nan"), dtype=torch.float64, device="cuda")
        gen.select(main, p.M, p.a, p.b, eta, aq, bq, out_a, out_b)
        torch.cuda.synchronize()
        which, Lq, Ls = oracle.choose_candidate(M, a, b, eta, cand_q, side_ref)
        assert int(gen.choice.cpu()[0]) == which == (0 if label == "good q" else 1)
        # the side stream's candidate is the oracle's two sweeps
        assert_half_step_close(gen.alpha_s.cpu().numpy(), side_ref[0], eta, "side alpha")
        assert_half_step_close(gen.beta_s.cpu().numpy(), side_ref[1], eta, "side beta")
        assert abs(float(gen.side.obj.cpu()[0]) - Ls) <= 1e-10 * max(abs(Ls), eta)
        assert abs(float(main.obj.cpu()[0]) - Lq) <= 1e-10 * max(abs(Lq), eta)
        chosen = (out_a.cpu().numpy(), out_b.cpu().numpy())
        expect = (gen.alpha_s.cpu().numpy(), gen.beta_s.cpu().numpy()) if which else cand_q
        np.testing.assert_array_equal(chosen[0], expect[0])
        np.testing.assert_array_equal(chosen[1], expect[1])
        # the inputs of the launch were not touched
        np.testing.assert_array_equal(ald.cpu().numpy(), alpha0)


def test_choice_in_place_and_tie():
    n, m, eta = 40, 50, 0.3
    M, a, b, alpha, beta = W.random_small(n, m, seed=8, eta=eta)
    gen = CandidateGenerator(n, m)
    main = DualPass(n, m)
    ald, bed = dev(alpha), dev(beta)
    gen.launch(dev(M), dev(a), dev(b), ald, bed, eta, sweeps=0)      # no sweeps: the same point, a tie
    aq, bq = ald.clone(), bed.clone()
    gen.select(main, dev(M), dev(a), dev(b), eta, aq, bq, aq, bq)    # outputs are q's own buffers
    torch.cuda.synchronize()
    assert int(gen.choice.cpu()[0]) == 0
    np.testing.assert_array_equal(aq.cpu().numpy(), alpha)
