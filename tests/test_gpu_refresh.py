"""regot_dual_eval_sparsify_topk (threshold search and fused evaluation in one read of M) against the oracle:
the threshold is oracle.topk_threshold, the CSR is oracle.sparsify_csr at that threshold, objective and
gradient are oracle.dual_eval."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2605_08793_amd import workloads as W
from paper_2605_08793_amd.driver import PatternRefresh
from parity_utils import assert_csr_close, assert_dual_eval_close

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda")


def run_refresh(Md, M, a, b, alpha, beta, eta, k, label, ref_delta=None, check_csr=True):
    n, m = M.shape
    print(f"[refresh] {label} n={n} m={m} eta={eta} k={k}", flush=True)
    pr = PatternRefresh(n, m, k)
    pr.workspace.fill_(0x3C); pr.topk_workspace.fill_(0xA7)      # the call must not rely on their contents
    for t in (pr.obj, pr.grad_alpha, pr.grad_beta, pr.row_sum, pr.col_sum, pr.val, pr.delta):
        t.fill_(float("nan"))
    pr.row_ptr.fill_(-1); pr.col_idx.fill_(-1); pr.info.fill_(-1)
    pr.refresh(Md, dev(a), dev(b), dev(alpha), dev(beta), eta)
    torch.cuda.synchronize()
    info = pr.info.cpu().tolist()
    delta = float(pr.delta.cpu()[0])
    got = dict(obj=float(pr.obj.cpu()[0]), grad_alpha=pr.grad_alpha.cpu().numpy(), grad_beta=pr.grad_beta.cpu().numpy(),
               row_sum=pr.row_sum.cpu().numpy(), col_sum=pr.col_sum.cpu().numpy())
    return pr, info, delta, got


def check_against_oracle(M, a, b, alpha, beta, eta, k, pr, info, delta, got, ref_delta=None):
    assert info[1] == 0, info
    if ref_delta is None:
        ref_delta = oracle.topk_threshold(M, alpha, beta, eta, k)
    assert abs(delta - ref_delta) <= 1e-12 * ref_delta, (delta, ref_delta)
    assert_dual_eval_close(got, oracle.dual_eval(M, a, b, alpha, beta, eta), a, b, alpha, beta, eta)
    ref_csr = oracle.sparsify_csr(M, alpha, beta, eta, ref_delta)
    rp, ci, v, _ = pr.csr_host()
    assert info[0] == rp[-1] >= k
    assert_csr_close((rp, ci, v), ref_csr, ref_delta, M.shape[1])


# (more than 65536 rows: the per-workgroup counts are then scanned by a launch of its own)
@pytest.mark.parametrize("n,m,frac", [(1100, 1000, 0.01), (1500, 2300, 0.005), (3000, 700, 0.02), (1201, 999, 0.001),
                                       (2048, 1024, 0.05), (40, 30000, 0.003), (70001, 19, 0.004), (131072, 9, 0.01)])
def test_random_problems(n, m, frac):
    eta = 0.05
    M, a, b, alpha, beta = W.random_small(n, m, seed=600 + n, eta=eta)
    k = max(1, int(round(frac * n * m)))
    pr, info, delta, got = run_refresh(dev(M), M, a, b, alpha, beta, eta, k, "random")
    check_against_oracle(M, a, b, alpha, beta, eta, k, pr, info, delta, got)


@pytest.mark.parametrize("name,n,m,sweeps", [("c3", 1500, 2300, 10), ("c4", 3000, 700, 5), ("syn1_diff", 1600, 1200, 5)])
def test_workloads_reduced(name, n, m, sweeps):
    p = W.make_problem(name, device="cuda", n=n, m=m)
    M, a, b = p.host()
    alpha, beta = oracle.sinkhorn_sweeps(M, a, b, p.eta, sweeps)
    k = p.k_keep()
    pr, info, delta, got = run_refresh(p.M, M, a, b, alpha, beta, p.eta, k, name)
    check_against_oracle(M, a, b, alpha, beta, p.eta, k, pr, info, delta, got)


def test_random_cases():
    rng = np.random.default_rng(51)
    for it in range(14):
        kind = int(rng.integers(0, 3))
        if kind == 0:
            n, m = int(rng.integers(20, 300)), int(rng.integers(6000, 60000))
        elif kind == 1:
            n, m = int(rng.integers(6000, 60000)), int(rng.integers(20, 300))
        else:
            n, m = int(rng.integers(1100, 2600)), int(rng.integers(1100, 2600))
        if n * m < (1 << 20) + 4096:
            m = ((1 << 20) + 4096) // n + 1
        eta = float(rng.choice([0.5, 0.05, 0.01]))
        M, a, b, alpha, beta = W.random_small(n, m, seed=int(rng.integers(1 << 30)), eta=eta)
        k = max(1, int(n * m * float(rng.choice([1e-5, 1e-3, 0.01, 0.05]))))
        pr, info, delta, got = run_refresh(dev(M), M, a, b, alpha, beta, eta, k, f"random {it}")
        check_against_oracle(M, a, b, alpha, beta, eta, k, pr, info, delta, got)


def test_ties_at_the_threshold():
    # a block of equal costs around rank k: every tied entry is kept, nnz > k
    rng = np.random.default_rng(7)
    n, m, eta = 1200, 1100, 0.1
    M = rng.random((n, m))
    M[100:140, 200:260] = 0.02                       # 2400 equal entries near the top of the order
    alpha = np.zeros(n); beta = np.zeros(m)
    a = np.full(n, 1.0 / n); b = np.full(m, 1.0 / m)
    T = oracle.plan_dense(M, alpha, beta, eta)
    order = np.sort(T.ravel())[::-1]
    tied = float(np.exp(-0.02 / eta))
    first = int(np.searchsorted(-order, -tied, side="left"))
    k = first + 1000                                  # in the middle of the tie
    pr, info, delta, got = run_refresh(dev(M), M, a, b, alpha, beta, eta, k, "ties")
    check_against_oracle(M, a, b, alpha, beta, eta, k, pr, info, delta, got)
    assert info[0] == first + 2400


def test_small_matrix_asks_for_the_two_calls():
    n, m, eta = 300, 400, 0.1                         # fewer than 2^20 entries: no usable sample
    M, a, b, alpha, beta = W.random_small(n, m, seed=3, eta=eta)
    pr, info, delta, got = run_refresh(dev(M), M, a, b, alpha, beta, eta, 500, "too small")
    assert info[1] & 2 and np.isnan(delta)
    assert_dual_eval_close(got, oracle.dual_eval(M, a, b, alpha, beta, eta), a, b, alpha, beta, eta)


@pytest.mark.parametrize("name", ["c2", "c3", "c4"])
def test_full_size_configs(name):
    path = os.path.join(GOLDEN, f"dual_{name}.npz")
    if not os.path.exists(path):
        pytest.skip(f"{path} missing")
    z = np.load(path, allow_pickle=False)
    alpha, beta, ref_delta, k = z["alpha"], z["beta"], float(z["delta"]), int(z["k"])
    p = W.make_problem(name, device="cuda")
    M, a, b = p.host()
    pr, info, delta, got = run_refresh(p.M, M, a, b, alpha, beta, p.eta, k, name + " full size")
    check_against_oracle(M, a, b, alpha, beta, p.eta, k, pr, info, delta, got, ref_delta=ref_delta)


def test_c5_against_the_two_calls():
    """Configuration 5 (50000^2: three rounds of workgroups, 12.5 * 10^6 candidates, thousands of keys in the bin that
    holds the k-th value): the one-read refresh must give the stored threshold and, bit for bit, the CSR and the sums
    of regot_dual_eval_sparsify at that threshold, which the parity tests check against the oracle at this size."""
    from paper_2605_08793_amd.driver import DualPass
    path = os.path.join(GOLDEN, "dual_c5.npz")
    if not os.path.exists(path):
        pytest.skip(f"{path} missing")
    z = np.load(path, allow_pickle=False)
    alpha, beta, ref_delta, k = dev(z["alpha"]), dev(z["beta"]), float(z["delta"]), int(z["k"])
    p = W.make_problem("c5", device="cuda")
    print(f"[refresh] c5 n={p.n} m={p.m} k={k}", flush=True)
    pr = PatternRefresh(p.n, p.m, k)
    pr.refresh(p.M, p.a, p.b, alpha, beta, p.eta)
    torch.cuda.synchronize()
    info = pr.info.cpu().tolist()
    delta = float(pr.delta.cpu()[0])
    assert info[1] == 0 and info[0] >= k, info
    assert abs(delta - ref_delta) <= 1e-12 * ref_delta, (delta, ref_delta)
    dp = DualPass(p.n, p.m, capacity=int(pr.col_idx.numel()))
    dp.dual_eval_sparsify(p.M, p.a, p.b, alpha, beta, p.eta, delta)
    torch.cuda.synchronize()
    assert dp.info.cpu().tolist() == [info[0], 0]
    nnz = info[0]
    assert torch.equal(dp.row_ptr, pr.row_ptr)
    assert torch.equal(dp.col_idx[:nnz], pr.col_idx[:nnz]) and torch.equal(dp.val[:nnz], pr.val[:nnz])
    torch.testing.assert_close(dp.row_sum, pr.row_sum, rtol=1e-13, atol=0)   # (the two calls may cut the matrix differently)
    torch.testing.assert_close(dp.col_sum, pr.col_sum, rtol=1e-13, atol=0)
