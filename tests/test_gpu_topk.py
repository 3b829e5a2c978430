"""regot_topk_threshold on the GPU against the oracle's threshold and against the plain definition.

delta is compared with oracle.topk_threshold (the k-th largest T_ij, from the T values themselves).
s_k and the two counts are integers / exact bit patterns: they are compared with a full sort of
s = (alpha_i + beta_j) - M_ij done by numpy.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2605_08793_amd import workloads as W
from paper_2605_08793_amd.driver import DualPass, TopK

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
TINY = 2e-323   # a few units in the last place of the subnormal range


def dev(x, dtype=torch.float64):
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda", dtype=dtype)


def s_matrix(M, alpha, beta):
    return ((alpha[:, None] + beta[None, :]) - M) + 0.0


def definition(s_sorted_desc, k):
    s_k = s_sorted_desc[k - 1]
    n_all = s_sorted_desc.size
    asc = s_sorted_desc[::-1]
    above = n_all - int(np.searchsorted(asc, s_k, side="right"))
    equal = n_all - int(np.searchsorted(asc, s_k, side="left")) - above
    return s_k, above, equal


def check_topk(Md, M, alpha, beta, eta, ks, label="", topk_ws=None):
    n, m = M.shape
    s_sorted = np.sort(s_matrix(M, alpha, beta), axis=None)[::-1]
    ald, bed = dev(alpha), dev(beta)
    for k in ks:
        print(f"[topk] {label} n={n} m={m} eta={eta} k={k}", flush=True)
        tk = TopK(n, m, k)
        if topk_ws is not None:
            assert topk_ws.numel() >= tk.workspace.numel()
            tk.workspace = topk_ws
        tk.delta.fill_(float("nan")); tk.s_k.fill_(float("nan")); tk.info.fill_(-7)
        tk.threshold(Md, ald, bed, eta)
        delta, s_k, above, equal = tk.result_host()
        ref_s, ref_above, ref_equal = definition(s_sorted, k)
        assert s_k == ref_s and np.signbit(s_k) == np.signbit(ref_s), (k, s_k, ref_s)
        assert (above, equal) == (ref_above, ref_equal), (k, above, equal, ref_above, ref_equal)
        assert above < k <= above + equal
        ref_delta = oracle.topk_threshold(M, alpha, beta, eta, k)
        if np.isinf(ref_delta):
            assert delta == ref_delta, (k, delta, ref_delta)
        else:
            assert abs(delta - ref_delta) <= 1e-12 * ref_delta + TINY, (k, delta, ref_delta)
    return delta


SHAPES = [(1, 1), (1, 700), (5, 3), (17, 513), (65, 1025), (130, 64), (300, 1537), (1030, 130)]


@pytest.mark.parametrize("n,m", SHAPES)
@pytest.mark.parametrize("eta", [0.5, 0.02])
def test_small_shapes(n, m, eta):
    M, a, b, alpha, beta = W.random_small(n, m, seed=300 + n + m, eta=eta)
    nm = n * m
    ks = sorted({1, nm, (nm + 1) // 2, max(1, nm // 100), max(1, nm - 1), min(nm, 2)})
    check_topk(dev(M), M, alpha, beta, eta, ks, label="random_small")


@pytest.mark.parametrize("n,m", [(3_000_000, 1), (1, 3_000_000), (5, 300_000)])
def test_extreme_aspect_ratios(n, m):
    eta = 0.4
    M, a, b, alpha, beta = W.random_small(n, m, seed=43 + (n % 97), eta=eta)
    nm = n * m
    check_topk(dev(M), M, alpha, beta, eta, [1, nm // 1000, nm // 3, nm], label="extreme aspect")


@pytest.mark.parametrize("pad,shift", [(3, 0), (1, 1), (4, 2)])
def test_leading_dimension_and_misalignment(pad, shift):
    n, m, eta = 77, 1100, 0.1
    M, a, b, alpha, beta = W.random_small(n, m, seed=6, eta=eta)
    buf = torch.zeros(n * (m + pad) + 8, dtype=torch.float64, device="cuda")
    Md = buf[shift:shift + n * (m + pad)].view(n, m + pad)[:, :m]
    Md.copy_(dev(M))
    check_topk(Md, M, alpha, beta, eta, [1, 847, n * m // 3], label=f"ld=m+{pad} shift={shift}")


def test_all_entries_tied_never_fits_the_pool():
    # 1.3 million equal keys: the bucket never shrinks below the pool, so all five digits are
    # resolved by passes over M
    n, m, eta = 1100, 1200, 0.05
    M = np.full((n, m), 0.375)
    alpha = np.zeros(n); beta = np.zeros(m)
    check_topk(dev(M), M, alpha, beta, eta, [1, 65537, n * m], label="all tied")


def test_few_distinct_values_and_a_tied_block():
    rng = np.random.default_rng(11)
    n, m, eta = 900, 1300, 0.1
    M = rng.choice([0.0, 0.25, 0.5, 0.75], size=(n, m))
    alpha = np.zeros(n); beta = np.zeros(m)
    # 4 distinct keys, ~290k copies each
    ks = [1, 200000, 292500, 600000, n * m]
    check_topk(dev(M), M, alpha, beta, eta, ks, label="4 values")
    # distinct values with a block of 100k ties in the middle of the order
    M2 = rng.random((n, m))
    M2[100:300, 200:700] = 0.5
    check_topk(dev(M2), M2, alpha, beta, eta, [5, 585000 - 60000, 585000, 585000 + 60000], label="tied block")


def test_signed_zeros_and_mixed_signs():
    rng = np.random.default_rng(12)
    n, m, eta = 64, 640, 1.0
    M = np.zeros((n, m))
    alpha = np.where(rng.random(n) < 0.5, -0.0, 0.0)
    beta = np.where(rng.random(m) < 0.5, -0.0, 0.0)
    M[:, :100] = rng.standard_normal((n, 100))          # s of both signs
    M[:8, 100:120] = 1e-310                              # subnormal s
    ks = [1, 3200, 3300, n * m // 2, n * m - 3000, n * m]
    check_topk(dev(M), M, alpha, beta, eta, ks, label="zeros")


def test_large_magnitude_and_wide_range():
    rng = np.random.default_rng(13)
    n, m, eta = 257, 900, 0.01
    M = rng.random((n, m)) * 10.0 ** rng.integers(-12, 3, size=(n, m))
    alpha = rng.standard_normal(n) * 50
    beta = rng.standard_normal(m) * 50
    nm = n * m
    check_topk(dev(M), M, alpha, beta, eta, [1, 17, nm // 200, nm // 2, nm - 5], label="wide range")


@pytest.mark.parametrize("name,n,m,sweeps", [
    ("c1", None, None, 20),
    ("syn1_diff", 1600, 1200, 5),
    ("c3", 1500, 2300, 10),
    ("c4", 3000, 700, 5),
    ("c2", 1201, 999, 5),
])
def test_workloads_reduced(name, n, m, sweeps):
    """k of the configuration; then the threshold is fed to the sparsify call: it keeps what info says."""
    p = W.make_problem(name, device="cuda", n=n, m=m)
    M, a, b = p.host()
    alpha, beta = oracle.sinkhorn_sweeps(M, a, b, p.eta, sweeps)
    if p.noise_alpha is not None:
        alpha = alpha + p.noise_alpha; beta = beta + p.noise_beta
    k = p.k_keep()
    ws = torch.full((TopK(p.n, p.m, k).workspace.numel(),), 0xAB, dtype=torch.uint8, device="cuda")  # dirty workspace
    check_topk(p.M, M, alpha, beta, p.eta, [k, max(1, k // 7), k], label=name, topk_ws=ws)
    tk = TopK(p.n, p.m, k)
    tk.threshold(p.M, dev(alpha), dev(beta), p.eta)
    delta, s_k, above, equal = tk.result_host()
    dp = DualPass(p.n, p.m, capacity=above + equal + 4096)
    dp.sparsify_csr(p.M, dev(alpha), dev(beta), p.eta, delta)
    nnz = int(dp.info.cpu()[0])
    # exp is monotone up to its last bit: entries above s_k are kept, entries below it can tie only in T
    assert nnz >= k and nnz - (above + equal) <= 2, (nnz, above, equal, k)


def load_golden(name):
    path = os.path.join(GOLDEN, f"dual_{name}.npz")
    if not os.path.exists(path):
        pytest.skip(f"{path} missing (write it with tests/golden/make_dual_points.py {name})")
    z = np.load(path, allow_pickle=False)
    return z["alpha"], z["beta"], float(z["delta"]), int(z["k"])


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_full_size_configs(name):
    """At the benchmark sizes the threshold is compared with the one the oracle stored for the same
    dual point; the counts are checked by the sparsify call, which counts T_ij >= delta itself."""
    alpha, beta, ref_delta, k = load_golden(name)
    p = W.make_problem(name, device="cuda")
    print(f"[topk] {name} full size n={p.n} m={p.m} k={k}", flush=True)
    ald, bed = dev(alpha), dev(beta)
    tk = TopK(p.n, p.m, k)
    tk.threshold(p.M, ald, bed, p.eta)
    delta, s_k, above, equal = tk.result_host()
    assert abs(delta - ref_delta) <= 1e-12 * ref_delta, (delta, ref_delta)
    assert above < k <= above + equal
    dp = DualPass(p.n, p.m, capacity=above + equal + 4096)
    dp.sparsify_csr(p.M, ald, bed, p.eta, delta)
    nnz = int(dp.info.cpu()[0])
    assert nnz >= k and nnz - (above + equal) <= 2, (nnz, above, equal, k)
    # a second call on the same workspace with another k: the state is rebuilt by every call
    tk2 = TopK(p.n, p.m, k)
    tk2.workspace = tk.workspace
    tk2.k = 1
    tk2.threshold(p.M, ald, bed, p.eta)
    d1, s1, above1, equal1 = tk2.result_host()
    assert above1 == 0 and equal1 >= 1 and s1 >= s_k and d1 >= delta
