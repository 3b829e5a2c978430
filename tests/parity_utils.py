"""Comparison helpers for the GPU-vs-oracle parity tests.

Tolerances (fp64, relative 1e-10 as the target states; what "relative" is measured against is fixed here):
  objective     |dL|      <= 1e-10 * max(|L|, eta*S, |alpha.a| + |beta.b|)
  sums          |dr_i|    <= 1e-10 * r_i  (an exact 0 must come back as 0 or below 1e-300)
  gradient      |dg_i|    <= 1e-10 * max(marginal_i, sum_i)   -- not relative to |g_i| itself, which is
                             rounding noise right after a Sinkhorn half-step
  CSR values    relative 1e-10; pattern bit-exact except entries with |T/delta - 1| <= 1e-12
  half-steps    |d alpha_i| <= 1e-10 * max(|alpha_i|, eta)
"""
import numpy as np

RTOL = 1e-10
PATTERN_BAND = 1e-12


def assert_sums_close(got, ref, what):
    got = np.asarray(got); ref = np.asarray(ref)
    assert got.shape == ref.shape, what
    zero = ref == 0.0
    assert np.all(np.abs(got[zero]) < 1e-300), f"{what}: exact zeros not reproduced"
    err = np.abs(got - ref)
    bad = err > RTOL * np.abs(ref)
    assert not bad.any(), f"{what}: max rel err {np.max(err[~zero] / np.abs(ref[~zero])):.3e} at {np.argmax(bad)}"


def assert_dual_eval_close(gpu, ref, a, b, alpha, beta, eta):
    """gpu/ref: dicts with obj, grad_alpha, grad_beta, row_sum, col_sum (numpy)."""
    assert_sums_close(gpu["row_sum"], ref["row_sum"], "row_sum")
    assert_sums_close(gpu["col_sum"], ref["col_sum"], "col_sum")
    ga_tol = RTOL * np.maximum(a, ref["row_sum"])
    gb_tol = RTOL * np.maximum(b, ref["col_sum"])
    assert np.all(np.abs(gpu["grad_alpha"] - ref["grad_alpha"]) <= ga_tol), "grad_alpha"
    assert np.all(np.abs(gpu["grad_beta"] - ref["grad_beta"]) <= gb_tol), "grad_beta"
    S = float(ref["row_sum"].sum()) if len(ref["row_sum"]) else 0.0
    scale = max(abs(ref["obj"]), eta * S, abs(float(alpha @ a)) + abs(float(beta @ b)), 1e-300)
    assert abs(gpu["obj"] - ref["obj"]) <= RTOL * scale, f"obj {gpu['obj']!r} vs {ref['obj']!r}"


def csr_to_pairs(row_ptr, col_idx):
    rows = np.repeat(np.arange(len(row_ptr) - 1, dtype=np.int64), np.diff(row_ptr))
    return rows, col_idx.astype(np.int64)


def assert_csr_close(gpu, ref, delta, m, plan_entry=None):
    """gpu/ref: (row_ptr, col_idx, val).  Pattern must match exactly except for entries within
    PATTERN_BAND (relative) of delta, which may fall on either side; structure is checked in any case."""
    g_rp, g_ci, g_v = gpu
    r_rp, r_ci, r_v = ref
    assert g_rp[0] == 0 and np.all(np.diff(g_rp) >= 0) and g_rp[-1] == len(g_ci) == len(g_v)
    for arr_rp, arr_ci in ((g_rp, g_ci),):
        # strictly ascending columns inside each row: differences are > 0 except at row starts
        d = np.diff(arr_ci.astype(np.int64))
        starts = arr_rp[1:-1]
        starts = starts[(starts > 0) & (starts < len(arr_ci))]
        ok = d > 0
        ok[starts - 1] = True
        assert ok.all(), "columns not strictly ascending inside a row"
        assert len(arr_ci) == 0 or (arr_ci.min() >= 0 and arr_ci.max() < m)
    if np.array_equal(g_rp, r_rp) and np.array_equal(g_ci, r_ci):
        np.testing.assert_allclose(g_v, r_v, rtol=RTOL, atol=0)
        return 0
    g_rows, g_cols = csr_to_pairs(g_rp, g_ci)
    r_rows, r_cols = csr_to_pairs(r_rp, r_ci)
    g_key = g_rows * m + g_cols
    r_key = r_rows * m + r_cols
    only_g = ~np.isin(g_key, r_key)
    only_r = ~np.isin(r_key, g_key)
    # every entry on which the two patterns disagree must sit within the band around delta
    assert np.all(np.abs(g_v[only_g] / delta - 1.0) <= PATTERN_BAND), "GPU keeps an entry the oracle drops, outside the tie band"
    assert np.all(np.abs(r_v[only_r] / delta - 1.0) <= PATTERN_BAND), "GPU drops an entry the oracle keeps, outside the tie band"
    np.testing.assert_allclose(g_v[~only_g], r_v[~only_r], rtol=RTOL, atol=0)
    return int(only_g.sum() + only_r.sum())


def assert_half_step_close(got, ref, eta, what):
    got = np.asarray(got); ref = np.asarray(ref)
    tol = RTOL * np.maximum(np.abs(ref), eta)
    err = np.abs(got - ref)
    assert np.all(err <= tol), f"{what}: max err/tol {np.max(err / tol):.3e}"
