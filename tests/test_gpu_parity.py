"""GPU-vs-oracle parity, element by element, through the C ABI (via the ctypes binding)."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2605_08793_amd import binding as B
from paper_2605_08793_amd import workloads as W
from paper_2605_08793_amd.driver import DualPass
from parity_utils import (assert_csr_close, assert_dual_eval_close, assert_half_step_close, assert_sums_close)

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def dev(x, dtype=torch.float64):
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda", dtype=dtype)


def gpu_eval_dict(dp):
    torch.cuda.synchronize()
    return dict(obj=float(dp.obj.cpu()[0]), grad_alpha=dp.grad_alpha.cpu().numpy(),
                grad_beta=dp.grad_beta.cpu().numpy(), row_sum=dp.row_sum.cpu().numpy(),
                col_sum=dp.col_sum.cpu().numpy())


def full_check(Md, M, a, b, alpha, beta, eta, delta, capacity=None, label=""):
    """All entry points on one problem: dual_eval, sparsify_csr, the fused call and both half-steps."""
    print(f"[parity] {label} n={M.shape[0]} m={M.shape[1]} eta={eta} delta={delta!r}", flush=True)
    n, m = M.shape
    ref = oracle.dual_eval(M, a, b, alpha, beta, eta)
    ref_csr = oracle.sparsify_csr(M, alpha, beta, eta, delta)
    nnz = int(ref_csr[0][-1])
    cap = nnz + 64 if capacity is None else capacity
    dp = DualPass(n, m, cap)
    ad, bd, ald, bed = dev(a), dev(b), dev(alpha), dev(beta)
    # separate entry points
    dp.dual_eval(Md, ad, bd, ald, bed, eta)
    got = gpu_eval_dict(dp)
    assert_dual_eval_close(got, ref, a, b, alpha, beta, eta)
    dp.sparsify_csr(Md, ald, bed, eta, delta)
    rp, ci, v, overflow = dp.csr_host()
    assert overflow == 0
    flips = assert_csr_close((rp, ci, v), ref_csr, delta, m)
    # fused entry point: poison outputs first so stale results cannot pass
    for t in (dp.obj, dp.grad_alpha, dp.grad_beta, dp.row_sum, dp.col_sum, dp.val):
        t.fill_(float("nan"))
    dp.row_ptr.fill_(-1); dp.col_idx.fill_(-1); dp.info.fill_(-1)
    dp.dual_eval_sparsify(Md, ad, bd, ald, bed, eta, delta)
    got2 = gpu_eval_dict(dp)
    assert_dual_eval_close(got2, ref, a, b, alpha, beta, eta)
    rp2, ci2, v2, overflow2 = dp.csr_host()
    assert overflow2 == 0
    assert_csr_close((rp2, ci2, v2), ref_csr, delta, m)
    # the fused pass and the separate passes run the same arithmetic on every entry; only the order of the
    # sums can differ in the last bits: column sums are added up per row chunk, a call that expects many
    # entries cuts the rows into more chunks, and the cut decides whether a narrow last panel is run as a strip
    np.testing.assert_allclose(got2["row_sum"], got["row_sum"], rtol=1e-13, atol=0)
    np.testing.assert_allclose(got2["col_sum"], got["col_sum"], rtol=1e-13, atol=0)
    assert abs(got2["obj"] - got["obj"]) <= 1e-13 * max(abs(got["obj"]), eta * got["row_sum"].sum())
    np.testing.assert_array_equal(rp2, rp); np.testing.assert_array_equal(ci2, ci); np.testing.assert_array_equal(v2, v)
    # half-steps
    out_a = torch.full((n,), float("nan"), dtype=torch.float64, device="cuda")
    out_b = torch.full((m,), float("nan"), dtype=torch.float64, device="cuda")
    dp.half_step(Md, ad, ald, bed, eta, 0, out_a)
    dp.half_step(Md, bd, ald, bed, eta, 1, out_b)
    torch.cuda.synchronize()
    assert_half_step_close(out_a.cpu().numpy(), oracle.sinkhorn_half_step(M, a, alpha, beta, eta, 0), eta, "alpha step")
    assert_half_step_close(out_b.cpu().numpy(), oracle.sinkhorn_half_step(M, b, alpha, beta, eta, 1), eta, "beta step")
    return dict(nnz=nnz, flips=flips)


# ------------------------------------------------------------------ small and ragged shapes

SHAPES = [(1, 1), (1, 700), (5, 3), (17, 513), (65, 1025), (130, 64), (300, 1537), (67, 2048), (1030, 130)]


@pytest.mark.parametrize("n,m", SHAPES)
@pytest.mark.parametrize("eta", [0.5, 0.02])
def test_small_shapes(n, m, eta):
    M, a, b, alpha, beta = W.random_small(n, m, seed=100 + n + m, eta=eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    delta = float(np.quantile(T, 0.9)) if n * m > 1 else float(T[0, 0])
    full_check(dev(M), M, a, b, alpha, beta, eta, delta, label="random_small")


@pytest.mark.parametrize("n,m", [(3_000_000, 1), (1, 3_000_000), (500_000, 3), (5, 300_000)])
def test_extreme_aspect_ratios(n, m):
    # one column / one row / a few: many row chunks of a single ragged panel, or thousands of panels of one
    # chunk with a single group of rows
    eta = 0.4
    M, a, b, alpha, beta = W.random_small(n, m, seed=41 + (n % 97), eta=eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    full_check(dev(M), M, a, b, alpha, beta, eta, float(np.quantile(T, 0.99)), label="extreme aspect")


@pytest.mark.parametrize("n,m,dense,as_strip", [
    (700, 512 + 32, False, True),        # the benchmark's case in small: one full panel and 32 more columns
    (2000, 20000, False, True),          # its real width: 39 x 13 tasks and five strip workgroups, up to three chunks each
    (1500, 3 * 512 + 27, False, True),   # odd widths: 8-byte loads
    (333, 1024 + 33, False, False),      # the narrowest last panel that stays a panel of its own
    (260, 512 + 2, False, True),
    (5, 512 + 31, False, True),          # fewer rows than one group
    (1999, 1024 + 16, False, True),      # a last group of fewer than four rows
    (600, 512 + 30, True, True),         # every entry kept: the strip workgroups flush their records in mid-chunk
    (5000, 1024 + 32, True, True),
    (40000, 512 + 8, False, False),      # too many chunks for the places left beside the full panels' tasks
])
def test_narrow_last_panel_as_strip(n, m, dense, as_strip):
    # a last panel of at most 32 columns is shared by a few extra workgroups while the tasks of the full
    # panels fill the chip; everything they leave must be what a workgroup per task would leave
    eta = 0.3
    geometry = B.regot_plan_geometry(n, m, n * m if dense else n * m // 10 + 64)
    print("geometry (g_r, g_c, rounds, tallest chunk, strip workgroups):", geometry, flush=True)
    assert (geometry[4] > 0) == as_strip
    M, a, b, alpha, beta = W.random_small(n, m, seed=300 + n + m, eta=eta)
    T = oracle.plan_dense(M, alpha, beta, eta)
    delta = 0.0 if dense else float(np.quantile(T, 0.93))
    full_check(dev(M), M, a, b, alpha, beta, eta, delta, capacity=n * m if dense else None, label="strip")


@pytest.mark.parametrize("pad,shift", [(3, 0), (2, 1), (1, 1), (4, 2)])
def test_leading_dimension_and_misalignment(pad, shift):
    # ldM > m (odd and even), and a base pointer that is only 8-byte aligned: the 64-bit-load variant
    n, m, eta = 77, 1100, 0.1
    M, a, b, alpha, beta = W.random_small(n, m, seed=5, eta=eta)
    buf = torch.zeros(n * (m + pad) + 8, dtype=torch.float64, device="cuda")
    Md = buf[shift:shift + n * (m + pad)].view(n, m + pad)[:, :m]
    Md.copy_(dev(M))
    assert Md.stride(0) == m + pad
    T = oracle.plan_dense(M, alpha, beta, eta)
    full_check(Md, M, a, b, alpha, beta, eta, float(np.quantile(T, 0.95)), label=f"ld=m+{pad} shift={shift}")


@pytest.mark.parametrize("n,m,pad,shift", [(1, 1, 0, 0), (5, 3, 0, 0), (333, 1057, 0, 0), (700, 544, 0, 0), (77, 1100, 3, 1),
                                           (2000, 2560, 2, 0), (4100, 513, 0, 0)])
def test_read_probe_adds_every_entry_once(n, m, pad, shift):
    # the bandwidth probe walks M with the tiling of the dense calls; its result is the plain sum of the entries
    rng = np.random.default_rng(n + m)
    M = rng.random((n, m)) - 0.3
    buf = torch.full((n * (m + pad) + 8,), float("nan"), dtype=torch.float64, device="cuda")
    Md = buf[shift:shift + n * (m + pad)].view(n, m + pad)[:, :m]
    Md.copy_(dev(M))
    total = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda")
    B.regot_stream_read_probe(Md, total, workspace=B.new_workspace(n, m, -1))
    torch.cuda.synchronize()
    import math
    assert abs(float(total.cpu()[0]) - math.fsum(M.ravel())) <= 1e-12 * np.abs(M).sum()


# --------------------------------------------------------------------- workloads of the paper

@pytest.mark.parametrize("name,n,m,sweeps", [
    ("c1", None, None, 20),            # configuration 1 at full size
    ("syn1_diff", 1600, 1200, 5),      # the paper's smallest synthetic shape
    ("syn2", 1600, 1200, 5),
    ("syn1_diff", 3200, 2400, 3),      # the paper's two larger synthetic shapes (Sec. 5.1)
    ("syn2", 6400, 4800, 2),
    ("c3", 1500, 2300, 10),
    ("c4", 3000, 700, 5),
    ("c2", 1201, 999, 5),
])
def test_workloads_reduced(name, n, m, sweeps):
    p = W.make_problem(name, device="cuda", n=n, m=m)
    M, a, b = p.host()
    alpha, beta = oracle.sinkhorn_sweeps(M, a, b, p.eta, sweeps)
    if p.noise_alpha is not None:
        alpha = alpha + p.noise_alpha; beta = beta + p.noise_beta
    delta = oracle.topk_threshold(M, alpha, beta, p.eta, p.k_keep())
    res = full_check(p.M, M, a, b, alpha, beta, p.eta, delta, label=name)
    assert res["nnz"] >= p.k_keep()


# --------------------------------------------------------------------------------- edge cases

def test_threshold_extremes_and_overflow():
    n, m, eta = 40, 600, 0.3
    M, a, b, alpha, beta = W.random_small(n, m, seed=9, eta=eta)
    Md = dev(M)
    full_check(Md, M, a, b, alpha, beta, eta, 0.0, label="delta=0 (dense CSR)")
    full_check(Md, M, a, b, alpha, beta, eta, float("inf"), label="delta=inf (empty CSR)")
    # capacity too small: flag raised, offsets still exact
    T = oracle.plan_dense(M, alpha, beta, eta)
    delta = float(np.quantile(T, 0.5))
    ref_rp, _, _ = oracle.sparsify_csr(M, alpha, beta, eta, delta)
    dp = DualPass(n, m, capacity=100)
    dp.sparsify_csr(Md, dev(alpha), dev(beta), eta, delta)
    torch.cuda.synchronize()
    assert dp.info.cpu().tolist() == [int(ref_rp[-1]), 1]
    np.testing.assert_array_equal(dp.row_ptr.cpu().numpy(), ref_rp)
    # capacity exactly nnz: fits
    dp = DualPass(n, m, capacity=int(ref_rp[-1]))
    dp.sparsify_csr(Md, dev(alpha), dev(beta), eta, delta)
    rp, ci, v, overflow = dp.csr_host()
    assert overflow == 0
    assert_csr_close((rp, ci, v), oracle.sparsify_csr(M, alpha, beta, eta, delta), delta, m)
    # capacity 0 with an empty pattern
    dp = DualPass(n, m, capacity=0)
    dp.sparsify_csr(Md, dev(alpha), dev(beta), eta, float("inf"))
    torch.cuda.synchronize()
    assert dp.info.cpu().tolist() == [0, 0]


@pytest.mark.parametrize("n,m,capacity", [
    (3000, 1100, 12_000_000),   # four rounds of row chunks, every wave flushes records in mid-pass
    (2500, 1500, 3_800_000),    # two rounds, capacity barely above the number of entries
    (70_000, 40, 10_000_000),   # more than 1024 row blocks: the one-workgroup scan kernel, four rounds
])
def test_dense_pattern_over_several_rounds(n, m, capacity):
    # delta = 0 keeps all n*m entries: the staging buffers overflow many times, and the capacity makes the
    # call cut the rows into several rounds of chunks
    eta = 0.3
    M, a, b, alpha, beta = W.random_small(n, m, seed=77 + n, eta=eta)
    res = full_check(dev(M), M, a, b, alpha, beta, eta, 0.0, capacity=capacity, label="dense pattern, several rounds")
    assert res["nnz"] == n * m


@pytest.mark.parametrize("n,m", [(0, 0), (0, 5), (7, 0)])
def test_empty_problem(n, m):
    eta = 0.2
    rng = np.random.default_rng(1)
    a = rng.uniform(size=n); b = rng.uniform(size=m)
    alpha = rng.standard_normal(n); beta = rng.standard_normal(m)
    Md = torch.zeros((n, m), dtype=torch.float64, device="cuda")
    dp = DualPass(n, m, capacity=4)
    dp.dual_eval_sparsify(Md, dev(a), dev(b), dev(alpha), dev(beta), eta, 0.5)
    got = gpu_eval_dict(dp)
    assert got["obj"] == pytest.approx(float(alpha @ a + beta @ b), rel=1e-14, abs=1e-300)
    np.testing.assert_array_equal(got["grad_alpha"], a)
    np.testing.assert_array_equal(got["grad_beta"], b)
    np.testing.assert_array_equal(dp.row_ptr.cpu().numpy(), np.zeros(n + 1, dtype=np.int64))
    assert dp.info.cpu().tolist() == [0, 0]


def test_underflowing_rows_and_tiny_eta():
    # eta = 0.001 with costs near 1: whole rows of T are exactly 0; sums must be exact zeros,
    # the half-step must stay finite (log-domain), and the pattern of the few surviving entries exact
    n, m, eta = 150, 900, 0.001
    rng = np.random.default_rng(3)
    M = 0.8 + 0.2 * rng.uniform(size=(n, m))
    M[::7, ::13] = rng.uniform(0, 0.01, size=M[::7, ::13].shape)
    a = np.full(n, 1 / n); b = np.full(m, 1 / m)
    alpha = np.zeros(n); beta = np.zeros(m)
    ref = oracle.dual_eval(M, a, b, alpha, beta, eta)
    assert (ref["row_sum"] == 0).sum() > 50
    full_check(dev(M), M, a, b, alpha, beta, eta, 1e-3, label="underflow rows")


def test_large_magnitude_duals():
    # |alpha|, |beta| ~ 50 with eta = 1: T spans ~e^{+-150}; checks the range reduction far from 0
    n, m, eta = 64, 520, 1.0
    M, a, b, _, _ = W.random_small(n, m, seed=12, eta=eta)
    rng = np.random.default_rng(8)
    alpha = 50 * rng.standard_normal(n); beta = 50 * rng.standard_normal(m)
    T = oracle.plan_dense(M, alpha, beta, eta)
    full_check(dev(M), M, a, b, alpha, beta, eta, float(np.quantile(T, 0.99)), label="large duals")


def test_nan_stays_where_it_contributes():
    # inputs are required to be finite; a NaN that slips in must not hang anything or spread: only the sums
    # (and the objective) it contributes to become NaN, everything else is what the oracle gives
    n, m, eta = 700, 1300, 0.05
    M, a, b, alpha, beta = W.random_small(n, m, seed=21, eta=eta)
    M[3, 7] = np.nan
    M[411, 1290] = np.nan
    ref = oracle.dual_eval(M, a, b, alpha, beta, eta)
    assert np.isnan(ref["row_sum"]).sum() == 2 and np.isnan(ref["col_sum"]).sum() == 2
    dp = DualPass(n, m, capacity=n * m)
    dp.dual_eval_sparsify(dev(M), dev(a), dev(b), dev(alpha), dev(beta), eta, 0.5)
    torch.cuda.synchronize()
    assert np.isnan(float(dp.obj.cpu()[0]))
    for name, ref_v, mine in (("row", ref["row_sum"], dp.row_sum), ("col", ref["col_sum"], dp.col_sum)):
        got = mine.cpu().numpy()
        bad = np.isnan(ref_v)
        assert np.array_equal(np.isnan(got), bad), name
        assert_sums_close(got[~bad], ref_v[~bad], name + "_sum away from the NaNs")
    # a NaN never passes the threshold: the pattern is that of the finite entries
    rp, ci, v, ov = dp.csr_host()
    assert ov == 0 and not np.isnan(v).any()
    ref_csr = oracle.sparsify_csr(M, alpha, beta, eta, 0.5)
    assert_csr_close((rp, ci, v), ref_csr, 0.5, m)


@pytest.mark.parametrize("n,m", [(700, 1300), (900, 512 + 20), (64, 200), (2100, 1024 + 31)])
def test_infinite_costs_are_forbidden_assignments(n, m):
    # M_ij = +inf: T_ij = exp(-inf) = 0 exactly (Sec. 3.1), as the oracle's libm gives it: the entry adds nothing to any
    # sum, is no pattern entry for delta > 0 and IS one (with value 0) for delta = 0; half-steps ignore it.  Whole
    # (row, panel) segments, the first rows of a column and a whole chunk of a column are infinite as well.
    eta = 0.05
    M, a, b, alpha, beta = W.random_small(n, m, seed=210 + n, eta=eta)
    rng = np.random.default_rng(n)
    inf = float("inf")
    M[rng.random((n, m)) < 0.01] = inf
    M[3, :min(m - 30, 512)] = inf         # a whole (row, panel) segment (a row of nothing but infinite costs has no update)
    M[7, :] = inf; M[7, m // 2] = 0.3     # a row with a single finite cost
    M[:40, 5] = inf                       # the first groups of rows of a column
    M[:, 9] = inf; M[n - 1, 9] = 0.1      # all of a column but its last row
    M[n // 2:, m - 1] = inf
    last = (m - 1) // 512 * 512           # first column of the last panel (a strip in the second shape)
    if last > 0:
        M[11, last:] = inf                # a row's whole segment in the last panel: an empty partial log-sum-exp
        M[:, m - 2] = inf; M[0, m - 2] = 0.2   # a column of the last panel that is finite in its first row only
    T = oracle.plan_dense(M, alpha, beta, eta)
    assert (T == 0).sum() >= (M == inf).sum() > 0
    delta = float(np.quantile(T[T > 0], 0.9))
    Md = dev(M)
    full_check(Md, M, a, b, alpha, beta, eta, delta, label="inf costs")
    full_check(Md, M, a, b, alpha, beta, eta, 0.0, label="inf costs, dense pattern")
    # the values on a stored pattern that contains such entries
    rp, ci, v = oracle.sparsify_csr(M, alpha, beta, eta, 0.0)
    out = torch.full((len(ci),), float("nan"), dtype=torch.float64, device="cuda")
    B.regot_pattern_values(Md, dev(alpha), dev(beta), eta, dev(rp, torch.int64), dev(ci, torch.int32), None, out, None)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    np.testing.assert_array_equal(got == 0, v == 0)
    np.testing.assert_allclose(got, v, rtol=1e-10, atol=0)


def test_negative_infinite_cost_overflows_like_the_oracle():
    # M_ij = -inf: T_ij = +inf; its row and column sums are +inf, every other sum is untouched
    n, m, eta = 300, 700, 0.1
    M, a, b, alpha, beta = W.random_small(n, m, seed=5, eta=eta)
    M[17, 333] = -float("inf")
    ref = oracle.dual_eval(M, a, b, alpha, beta, eta)
    assert ref["row_sum"][17] == np.inf and ref["col_sum"][333] == np.inf
    dp = DualPass(n, m)
    dp.dual_eval(dev(M), dev(a), dev(b), dev(alpha), dev(beta), eta)
    got = gpu_eval_dict(dp)
    assert got["row_sum"][17] == np.inf and got["col_sum"][333] == np.inf
    keep_r = np.arange(n) != 17; keep_c = np.arange(m) != 333
    assert_sums_close(got["row_sum"][keep_r], ref["row_sum"][keep_r], "row_sum")
    assert_sums_close(got["col_sum"][keep_c], ref["col_sum"][keep_c], "col_sum")


def test_bit_reproducible():
    p = W.make_problem("c1", device="cuda")
    n, m = p.n, p.m
    rng = np.random.default_rng(0)
    alpha = dev(0.01 * rng.standard_normal(n)); beta = dev(0.01 * rng.standard_normal(m))
    outs = []
    for _ in range(3):
        dp = DualPass(n, m, capacity=n * m // 50)
        dp.dual_eval_sparsify(p.M, p.a, p.b, alpha, beta, p.eta, 1e-6)
        torch.cuda.synchronize()
        outs.append([t.cpu().numpy().copy() for t in (dp.obj, dp.grad_alpha, dp.grad_beta, dp.row_ptr, dp.info)]
                    + list(dp.csr_host()[1:3]))
    for other in outs[1:]:
        for x, y in zip(outs[0], other):
            np.testing.assert_array_equal(x, y)


def test_in_place_sweeps_match_oracle_sweeps():
    p = W.make_problem("c1", device="cuda", n=700, m=900)
    M, a, b = p.host()
    dp = DualPass(p.n, p.m)
    alpha, beta = dp.sinkhorn_sweeps(p.M, p.a, p.b, p.eta, 10)
    torch.cuda.synchronize()
    ra, rb = oracle.sinkhorn_sweeps(M, a, b, p.eta, 10)
    # ten chained half-steps: rounding differences compound slightly
    np.testing.assert_allclose(alpha.cpu().numpy(), ra, rtol=0, atol=1e-9 * max(np.abs(ra).max(), p.eta))
    np.testing.assert_allclose(beta.cpu().numpy(), rb, rtol=0, atol=1e-9 * max(np.abs(rb).max(), p.eta))
    # regot_sinkhorn_sweeps is exactly the sequence of half-step calls, and never reads the alpha it is given first
    a2 = torch.full((p.n,), float("nan"), dtype=torch.float64, device="cuda"); b2 = torch.zeros(p.m, dtype=torch.float64, device="cuda")
    for _ in range(10):
        dp.half_step(p.M, p.a, a2, b2, p.eta, 0, a2)
        dp.half_step(p.M, p.b, a2, b2, p.eta, 1, b2)
    a3 = torch.full((p.n,), float("nan"), dtype=torch.float64, device="cuda"); b3 = torch.zeros(p.m, dtype=torch.float64, device="cuda")
    B.regot_sinkhorn_sweeps(p.M, p.a, p.b, a3, b3, p.eta, 10, workspace=dp.workspace)
    B.regot_sinkhorn_sweeps(p.M, p.a, p.b, a3, b3, p.eta, 0, workspace=dp.workspace)     # no sweep: nothing changes
    torch.cuda.synchronize()
    assert torch.equal(a2, a3) and torch.equal(b2, b3) and torch.equal(alpha, a3) and torch.equal(beta, b3)


# ------------------------------------------------------------------ full-size configurations

def load_golden(name):
    path = os.path.join(GOLDEN, f"dual_{name}.npz")
    if not os.path.exists(path):
        pytest.skip(f"{path} missing (write it with tests/golden/make_dual_points.py {name})")
    z = np.load(path, allow_pickle=False)
    return z["alpha"], z["beta"], float(z["delta"]), int(z["k"])


@pytest.mark.parametrize("name", ["c2", "c3", "c4"])
def test_full_size_configs(name):
    """Whole-output parity at the benchmark sizes, same launch path the benchmark times."""
    alpha, beta, delta, k = load_golden(name)
    p = W.make_problem(name, device="cuda")
    M, a, b = p.host()
    res = full_check(p.M, M, a, b, alpha, beta, p.eta, delta, label=f"{name} full size")
    # the stored threshold keeps the configured fraction (up to ties / last-bit differences in M)
    assert abs(res["nnz"] - k) <= max(4, k // 1000)


def test_c5_sampled_rows_and_columns():
    """Configuration 5 (50000^2, 20 GB of M in HBM): the oracle checks sampled rows and columns one by
    one, and properties that hold at any size check the rest.  Chunks are 10000 rows tall here and a
    wave selects ~2500 entries, so this is also the case in which the on-chip buffers of the streaming
    kernel fill up and are flushed before the wave is done."""
    alpha, beta, delta, k = load_golden("c5")
    p = W.make_problem("c5", device="cuda")
    n, m, eta = p.n, p.m, p.eta
    print(f"[parity] c5 sampled n={n} m={m} eta={eta} delta={delta!r}", flush=True)
    a = p.a.cpu().numpy(); b = p.b.cpu().numpy()
    ald, bed = dev(alpha), dev(beta)
    dp = DualPass(n, m, capacity=int(k * 1.05) + 1024)
    dp.dual_eval_sparsify(p.M, p.a, p.b, ald, bed, eta, delta)
    got = gpu_eval_dict(dp)
    rp, ci, v, overflow = dp.csr_host()
    assert overflow == 0
    out_a = torch.empty(n, dtype=torch.float64, device="cuda"); out_b = torch.empty(m, dtype=torch.float64, device="cuda")
    dp.half_step(p.M, p.a, ald, bed, eta, 0, out_a)
    dp.half_step(p.M, p.b, ald, bed, eta, 1, out_b)
    torch.cuda.synchronize()
    out_a = out_a.cpu().numpy(); out_b = out_b.cpu().numpy()
    # the evaluation without the pattern: its waves take 2500 rows each, more than they can hold results of, so it
    # too writes some in mid-stream; every sum against the fused call's (different chunks: equal up to summation order)
    dp2 = DualPass(n, m)
    dp2.dual_eval(p.M, p.a, p.b, ald, bed, eta)
    plain = gpu_eval_dict(dp2)
    np.testing.assert_allclose(plain["row_sum"], got["row_sum"], rtol=1e-13, atol=0)
    np.testing.assert_allclose(plain["col_sum"], got["col_sum"], rtol=1e-13, atol=0)
    assert abs(plain["obj"] - got["obj"]) <= 1e-13 * abs(got["obj"])
    del dp2

    rng = np.random.default_rng(55)
    rows = np.unique(np.concatenate([[0, 1, 3, 9999, 10000, 10001, 19999, 20000, n - 2, n - 1], rng.integers(0, n, 30)]))
    cols = np.unique(np.concatenate([[0, 1, 511, 512, 513, 49663, 49664, m - 2, m - 1], rng.integers(0, m, 30)]))
    # sampled rows: row sums, gradient, CSR rows, alpha update
    Mr = p.M[torch.from_numpy(rows).cuda()].cpu().numpy()
    ref = oracle.dual_eval(Mr, a[rows], b, alpha[rows], beta, eta)
    assert_sums_close(got["row_sum"][rows], ref["row_sum"], "row_sum (sampled rows)")
    assert np.all(np.abs(got["grad_alpha"][rows] - ref["grad_alpha"]) <= 1e-10 * np.maximum(a[rows], ref["row_sum"]))
    r_rp, r_ci, r_v = oracle.sparsify_csr(Mr, alpha[rows], beta, eta, delta)
    for t, i in enumerate(rows):
        g_c_, g_v_ = ci[rp[i]:rp[i + 1]], v[rp[i]:rp[i + 1]]
        o_c_, o_v_ = r_ci[r_rp[t]:r_rp[t + 1]], r_v[r_rp[t]:r_rp[t + 1]]
        if not np.array_equal(g_c_, o_c_):   # only threshold ties may differ
            diff = np.setxor1d(g_c_, o_c_)
            T = oracle.plan_dense(Mr[t:t + 1, diff], alpha[i:i + 1], beta[diff], eta)[0]
            assert np.all(np.abs(T / delta - 1) <= 1e-12), f"row {i}: pattern differs outside the tie band"
        common, gi, oi = np.intersect1d(g_c_, o_c_, return_indices=True)
        np.testing.assert_allclose(g_v_[gi], o_v_[oi], rtol=1e-10, atol=0)
    assert_half_step_close(out_a[rows], oracle.sinkhorn_half_step(Mr, a[rows], alpha[rows], beta, eta, 0), eta, "alpha step")
    # sampled columns: column sums, gradient, beta update
    Mc = p.M[:, torch.from_numpy(cols).cuda()].cpu().numpy()
    refc = oracle.dual_eval(Mc, a, b[cols], alpha, beta[cols], eta)
    assert_sums_close(got["col_sum"][cols], refc["col_sum"], "col_sum (sampled columns)")
    assert np.all(np.abs(got["grad_beta"][cols] - refc["grad_beta"]) <= 1e-10 * np.maximum(b[cols], refc["col_sum"]))
    assert_half_step_close(out_b[cols], oracle.sinkhorn_half_step(Mc, b[cols], alpha, beta[cols], eta, 1), eta, "beta step")
    # properties of the whole output
    S_r, S_c = got["row_sum"].sum(), got["col_sum"].sum()
    assert abs(S_r - S_c) <= 1e-11 * S_r
    L = -eta * S_r + alpha @ a + beta @ b
    assert abs(got["obj"] - L) <= 1e-10 * max(abs(L), eta * S_r, abs(alpha @ a) + abs(beta @ b))
    np.testing.assert_allclose(got["grad_alpha"], a - got["row_sum"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(got["grad_beta"], b - got["col_sum"], rtol=0, atol=1e-15)
    assert rp[0] == 0 and np.all(np.diff(rp) >= 0) and rp[-1] == len(ci) == len(v)
    assert abs(int(rp[-1]) - k) <= max(4, k // 1000)
    d = np.diff(ci.astype(np.int64)); starts = rp[1:-1]; starts = starts[(starts > 0) & (starts < len(ci))]
    ok = d > 0; ok[starts - 1] = True
    assert ok.all() and ci.min() >= 0 and ci.max() < m
    assert v.min() >= delta * (1 - 1e-12)
    # every kept value is the plan entry at its position (spot check through the oracle's dense formula)
    pick = rng.integers(0, len(ci), 2000)
    prow = np.searchsorted(rp, pick, side="right") - 1
    Mpick = p.M[torch.from_numpy(prow).cuda(), torch.from_numpy(ci[pick].astype(np.int64)).cuda()].cpu().numpy()
    Tpick = np.array([oracle.plan_dense(np.array([[Mpick[t]]]), alpha[prow[t]:prow[t] + 1], beta[ci[pick[t]]:ci[pick[t]] + 1], eta)[0, 0]
                      for t in range(len(pick))])
    np.testing.assert_allclose(v[pick], Tpick, rtol=1e-10, atol=0)
    # the pattern is complete: the number of entries >= delta in the sampled rows equals the oracle's (checked
    # above), and the total equals the sum of the per-row counts by construction of row_ptr


def test_c5_entry_counts_of_all_rows():
    """Configuration 5, the integer part of the whole output: the number of kept entries of every one of the 50 000
    rows (row_ptr) and the column indices of every row against the oracle, which gets M back in blocks of rows.  (Values
    are checked on sampled rows in the test above.)  This is the size at which the pass runs three rounds of
    workgroups and flushes records in mid-pass."""
    alpha, beta, delta, k = load_golden("c5")
    p = W.make_problem("c5", device="cuda")
    n, m, eta = p.n, p.m, p.eta
    print(f"[parity] c5 all rows n={n} m={m} delta={delta!r}", flush=True)
    ald, bed = dev(alpha), dev(beta)
    dp = DualPass(n, m, capacity=int(k * 1.05) + 1024)
    dp.dual_eval_sparsify(p.M, p.a, p.b, ald, bed, eta, delta)
    rp, ci, v, overflow = dp.csr_host()
    assert overflow == 0
    block = 2500
    flips = 0
    for r0 in range(0, n, block):
        r1 = min(n, r0 + block)
        Mb = p.M[r0:r1].cpu().numpy()
        o_rp, o_ci, o_v = oracle.sparsify_csr(Mb, alpha[r0:r1], beta, eta, delta)
        g_cnt = np.diff(rp[r0:r1 + 1]); o_cnt = np.diff(o_rp)
        g_ci = ci[rp[r0]:rp[r1]]
        if np.array_equal(g_cnt, o_cnt) and np.array_equal(g_ci, o_ci):
            continue
        # only entries within the tie band of the threshold may differ
        for i in np.nonzero(g_cnt != o_cnt)[0] if not np.array_equal(g_cnt, o_cnt) else range(r1 - r0):
            gc = ci[rp[r0 + i]:rp[r0 + i + 1]]; oc = o_ci[o_rp[i]:o_rp[i + 1]]
            diff = np.setxor1d(gc, oc)
            if len(diff) == 0:
                continue
            T = oracle.plan_dense(Mb[i:i + 1, diff], alpha[r0 + i:r0 + i + 1], beta[diff], eta)[0]
            assert np.all(np.abs(T / delta - 1) <= 1e-12), f"row {r0 + i}: pattern differs outside the tie band"
            flips += len(diff)
        print(f"[parity] c5 rows {r0}..{r1}: checked, {flips} entries in the tie band so far", flush=True)
    assert flips <= 8
    assert int(rp[-1]) == int(dp.info.cpu()[0])


def test_tall_matrix_chunk_height():
    """32 767 x 131 584 (34 GB): two row chunks would be 16 387 and 16 380 rows tall, more than the 14 bits a staged
    entry has for its row inside its chunk; the cut must give more chunks.  The oracle checks the rows around the
    old chunk boundary and the last rows, properties of the whole output check the rest."""
    n, m, eta = 32767, 131584, 0.05
    capacity = 2_400_000                          # one round of workgroups: the fewest, tallest chunks
    g_r, g_c, rounds, tallest, strip = B.regot_plan_geometry(n, m, capacity)
    assert tallest <= 16384 and g_r == 3 and rounds == 1
    gen = torch.Generator(device="cuda"); gen.manual_seed(77)
    Md = torch.rand((n, m), dtype=torch.float64, device="cuda", generator=gen)
    rng = np.random.default_rng(3)
    alpha = 1e-4 * rng.standard_normal(n); beta = 1e-4 * rng.standard_normal(m)
    a = np.full(n, 1.0 / n); b = np.full(m, 1.0 / m)
    delta = float(np.exp(-0.0005 / eta))          # keeps the ~0.05 % smallest costs: about 2.2 * 10^6 entries
    print(f"[parity] tall matrix n={n} m={m} geometry={(g_r, g_c, rounds, tallest, strip)}", flush=True)
    dp = DualPass(n, m, capacity=capacity)
    dp.dual_eval_sparsify(Md, dev(a), dev(b), dev(alpha), dev(beta), eta, delta)
    rp, ci, v, overflow = dp.csr_host()
    assert overflow == 0 and 1_800_000 < rp[-1] < capacity
    rows = np.unique(np.concatenate([np.arange(16370, 16400), np.arange(10915, 10930), np.arange(21840, 21850), np.arange(n - 12, n), [0, 1, 2]]))
    Mr = Md[torch.from_numpy(rows).cuda()].cpu().numpy()
    o_rp, o_ci, o_v = oracle.sparsify_csr(Mr, alpha[rows], beta, eta, delta)
    ref = oracle.dual_eval(Mr, a[rows], b, alpha[rows], beta, eta)
    assert_sums_close(dp.row_sum.cpu().numpy()[rows], ref["row_sum"], "row_sum (sampled rows)")
    for t, i in enumerate(rows):
        np.testing.assert_array_equal(ci[rp[i]:rp[i + 1]], o_ci[o_rp[t]:o_rp[t + 1]], err_msg=f"row {i}")
        np.testing.assert_allclose(v[rp[i]:rp[i + 1]], o_v[o_rp[t]:o_rp[t + 1]], rtol=1e-10, atol=0)
    assert rp[0] == 0 and np.all(np.diff(rp) >= 0) and rp[-1] == len(ci)
    d = np.diff(ci.astype(np.int64)); starts = rp[1:-1]; starts = starts[(starts > 0) & (starts < len(ci))]
    ok = d > 0; ok[starts - 1] = True
    assert ok.all() and ci.min() >= 0 and ci.max() < m and v.min() >= delta
    # every kept value is the plan entry at its position
    pick = rng.integers(0, len(ci), 3000)
    prow = np.searchsorted(rp, pick, side="right") - 1
    Mpick = Md[torch.from_numpy(prow).cuda(), torch.from_numpy(ci[pick].astype(np.int64)).cuda()].cpu().numpy()
    Tpick = np.exp(((alpha[prow] + beta[ci[pick]]) - Mpick) / eta)
    np.testing.assert_allclose(v[pick], Tpick, rtol=1e-9, atol=0)


def test_placement_of_workgroups_is_what_pace_keeping_assumes():
    """Only speed depends on this.  The fused pass lets workgroups b and b + 256 keep each other's pace because they share a
    compute unit, and the scatter kernel gives the pieces of a CSR row to workgroups with equal b mod 8 because those run on
    one die (which die that is changes from launch to launch: the dispatcher's round-robin over the dies does not restart
    at die 0).  The hardware-id registers say whether that is so on this device."""
    for trial in range(3):
        ids = torch.zeros(2 * 512, dtype=torch.int32, device="cuda")
        B.regot_placement_probe(ids)
        torch.cuda.synchronize()
        h = ids.cpu().numpy().astype(np.int64).reshape(512, 2) & 0xFFFFFFFF
        hw, die = h[:, 0], h[:, 1] & 0xF
        cu_key = ((die * 8 + ((hw >> 13) & 7)) * 2 + ((hw >> 12) & 1)) * 16 + ((hw >> 8) & 0xF)
        same_cu = int((cu_key[:256] == cu_key[256:]).sum())
        dies_of_residue = [set(die[np.arange(512) % 8 == r].tolist()) for r in range(8)]
        one_die_per_residue = all(len(d) == 1 for d in dies_of_residue) and len(set.union(*dies_of_residue)) == 8
        print(f"[placement] trial {trial}: compute units in use: {len(np.unique(cu_key))}; b and b + 256 on one compute unit: {same_cu} "
              f"of 256; die of workgroups 0..7: {die[:8].tolist()}; one die per residue of b mod 8: {one_die_per_residue}", flush=True)
        if same_cu != 256 or not one_die_per_residue:
            pytest.skip("the dispatcher places workgroups differently on this device: pace keeping is ineffective here (results unaffected)")
