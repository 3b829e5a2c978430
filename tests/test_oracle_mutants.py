"""Do the pins have teeth?  Each case plants ONE plausible mistake (a wrong sign, a dropped term, a
wrong index, an off-by-one) in a private copy of the oracle, on the CPU, and runs the pin suites against
that copy in a child process: the suites must fail.  An untouched copy must pass (the harness itself).
Nothing here touches the GPU or the product library."""
import concurrent.futures
import os
import shutil
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_SUITES = [os.path.join(ROOT, "tests", "test_oracle_pins.py"),
              os.path.join(ROOT, "tests", "test_oracle_hessian_pins.py")]

C = "regot_oracle.c"
PY = "__init__.py"

# (name, file, text to find -- exactly one occurrence --, replacement)
MUTANTS = [
    ("plan entry: beta enters with the wrong sign", C,
     "double s = (alpha_i + beta_j) - M_ij;", "double s = (alpha_i - beta_j) - M_ij;"),
    ("plan entry: multiplied by eta instead of divided", C,
     "double x = s / eta;\n    return exp(x);", "double x = s * eta;\n    return exp(x);"),
    ("dense plan stored transposed", C, "T[i * m + j] = plan_entry", "T[j * n + i] = plan_entry"),
    ("dual_eval: gradient in alpha with the sign of grad f", C,
     "grad_alpha[i] = (double)((long double)a[i] - rowacc[i]);", "grad_alpha[i] = (double)(rowacc[i] - (long double)a[i]);"),
    ("dual_eval: gradient in beta with the sign of grad f", C,
     "grad_beta[j] = (double)((long double)b[j] - c);", "grad_beta[j] = (double)(c - (long double)b[j]);"),
    ("dual_eval: objective without beta^T b", C,
     "*obj = (double)(-(long double)eta * S + dot_a + dot_b);", "*obj = (double)(-(long double)eta * S + dot_a);"),
    ("dual_eval: objective with +eta S", C,
     "*obj = (double)(-(long double)eta * S + dot_a + dot_b);", "*obj = (double)((long double)eta * S + dot_a + dot_b);"),
    ("dual_eval: column sums in reversed order", C, "cacc[j] += (long double)T;", "cacc[m - 1 - j] += (long double)T;"),
    ("dual_eval: leading dimension ignored", C,
     "double T = plan_entry(alpha[i], beta[j], M[i * ldM + j], eta);\n                r += (long double)T;",
     "double T = plan_entry(alpha[i], beta[j], M[i * m + j], eta);\n                r += (long double)T;"),
    ("sparsify: strict comparison with the threshold", C, "if (T >= delta) {", "if (T > delta) {"),
    ("sparsify: one-based column indices", C, "col_idx[p] = (int32_t)j;", "col_idx[p] = (int32_t)(j + 1);"),
    ("sparsify: columns of a row in descending order", C,
     "for (int64_t j = 0; j < m; ++j) {\n            double T = plan_entry(alpha[i], beta[j], M[i * ldM + j], eta);\n            if (T >= delta) {",
     "for (int64_t j = m - 1; j >= 0; --j) {\n            double T = plan_entry(alpha[i], beta[j], M[i * ldM + j], eta);\n            if (T >= delta) {"),
    ("alpha half-step: sign of the log-sum-exp", C,
     "out[i] = eta * log(marginal[i]) - eta * lse;", "out[i] = eta * log(marginal[i]) + eta * lse;"),
    ("alpha half-step: maximum added but not subtracted", C,
     "double x = (beta[j] - M[i * ldM + j]) / eta;\n                sum += (long double)exp(x - mx);",
     "double x = (beta[j] - M[i * ldM + j]) / eta;\n                sum += (long double)exp(x);"),
    ("beta half-step: marginal term dropped", C,
     "out[j] = eta * log(marginal[j]) - eta * lse;", "out[j] = -eta * lse;"),
    ("beta half-step: cost enters with the wrong sign", C,
     "double x = (alpha[i] - M[i * ldM + j]) / eta;\n                        sum[j - lo]",
     "double x = (alpha[i] + M[i * ldM + j]) / eta;\n                        sum[j - lo]"),
    ("top-k: bucket sorted in ascending order", C, "return (x < y) - (x > y);", "return (x > y) - (x < y);"),
    ("top-k: rank counted from the wrong end of the histogram", C,
     "uint32_t bucket = NBUCKET - 1;\n    for (;; --bucket) {\n        if (above + hist[bucket] >= k) break;\n        above += hist[bucket];\n        if (bucket == 0)",
     "uint32_t bucket = 0;\n    for (;; ++bucket) {\n        if (above + hist[bucket] >= k) break;\n        above += hist[bucket];\n        if (bucket == NBUCKET - 1)"),
    ("stored pattern: leading dimension ignored", C,
     "val[p] = plan_entry(alpha[i], beta[j], M[i * ldM + j], eta);", "val[p] = plan_entry(alpha[i], beta[j], M[i * m + j], eta);"),
    ("transposition: position map is the identity", C, "csc_pos[p] = q;", "csc_pos[p] = p;"),
    ("transposition: rows of a column in descending order", C,
     "for (int64_t i = 0; i < n; ++i)            /* rows in ascending order: so are the rows of a column */",
     "for (int64_t i = n - 1; i >= 0; --i)"),
    ("H product: off-diagonal block reads the alpha part of x", C,
     "s += (long double)val[p] * x[n + j];", "s += (long double)val[p] * x[j];"),
    ("H product: tau missing in the alpha rows", C,
     "y[i] = (double)(s / eta + (long double)tau * x[i]);", "y[i] = (double)(s / eta);"),
    ("H product: column-sum diagonal missing", C,
     "long double s = acc[j] + (long double)col_sum[j] * x[n + j];", "long double s = acc[j];"),
    ("H product: transposed block not accumulated", C,
     "acc[j] += (long double)val[p] * x[i];", "acc[j] += 0.0L * x[i];"),
    ("H product: 1/eta missing", C,
     "y[n + j] = (double)(s / eta + (long double)tau * x[n + j]);", "y[n + j] = (double)(s + (long double)tau * x[n + j]);"),
    ("dense H: lower block left empty", C,
     "H[(n + j) * N + i] = val[p] / eta;", "H[(n + j) * N + i] = 0.0;"),
    ("dense H: upper block not divided by eta", C,
     "H[i * N + (n + j)] = val[p] / eta;", "H[i * N + (n + j)] = val[p];"),
    ("dense H: an entry of the pattern in the first column is skipped", C,
     "if (j >= m - 1) continue;\n            H[i * N + (n + j)]", "if (j >= m - 1 || j == 0) continue;\n            H[i * N + (n + j)]"),
    ("H product: an entry of the pattern in the last kept column is skipped", C,
     "if (j >= mb) continue;               /* the dropped column */", "if (j >= mb - 1) continue;"),
    ("lower triangle: values not divided by eta", C,
     "h_row_idx[q] = (int32_t)(n + j);\n                h_val[q] = val[p] / eta;",
     "h_row_idx[q] = (int32_t)(n + j);\n                h_val[q] = val[p];"),
    ("lower triangle: row index without the offset n", C,
     "h_row_idx[q] = (int32_t)(n + j);\n                h_val[q] = val[p] / eta;",
     "h_row_idx[q] = (int32_t)j;\n                h_val[q] = val[p] / eta;"),
    ("lower triangle: tau missing on the beta diagonal", C,
     "h_val[q] = col_sum[j] / eta + tau;", "h_val[q] = col_sum[j] / eta;"),
    ("metrics: entropy term of the primal value with the wrong sign", C,
     "long double Lp = tm + (long double)eta * tlogt - (long double)eta * tsum;",
     "long double Lp = tm - (long double)eta * tlogt - (long double)eta * tsum;"),
    ("metrics: gradient norm includes the fixed last variable", C,
     "if (j < m - 1) g2 += (col[j] - b[j]) * (col[j] - b[j]);", "g2 += (col[j] - b[j]) * (col[j] - b[j]);"),
    ("metrics: marginal error without absolute values", C, "merr += fabsl(r - a[i]);", "merr += (r - a[i]);"),
    ("metrics: <T, M> missing", C, "tm += (long double)T * M[i * ldM + j];", "tm += 0.0L * M[i * ldM + j];"),
]


def load_python_mutants():
    """Mistakes in the Python part of the oracle (the loops over the C functions)."""
    src = open(os.path.join(ROOT, "oracle", PY)).read()
    out = []

    def add(name, old, new):
        if src.count(old) == 1:
            out.append((name, PY, old, new))
        else:                                  # the text moved: fail loudly rather than test nothing
            out.append((name, PY, old, None))
    return out, add


def run_case(case):
    name, fname, old, new = case
    tmp = tempfile.mkdtemp(prefix="oracle_mutant_")
    try:
        dst = os.path.join(tmp, "oracle")
        os.makedirs(dst)
        for f in (C, PY, "build.py"):
            shutil.copy(os.path.join(ROOT, "oracle", f), os.path.join(dst, f))
        if old is not None:
            path = os.path.join(dst, fname)
            text = open(path).read()
            if new is None or text.count(old) != 1:
                return name, "stale", f"the text to replace occurs {text.count(old)} times in {fname}"
            open(path, "w").write(text.replace(old, new))
        env = dict(os.environ, REGOT_TEST_ORACLE_PATH=tmp, OMP_NUM_THREADS="2", PYTHONDONTWRITEBYTECODE="1")
        subprocess.run([sys.executable, os.path.join(dst, "build.py")], check=True, env=env,
                       stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        r = subprocess.run([sys.executable, "-m", "pytest", *PIN_SUITES, "-x", "-q", "-p", "no:cacheprovider"],
                           env=env, cwd=tmp, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
        tail = "\n".join(r.stdout.strip().splitlines()[-3:])
        return name, ("passed" if r.returncode == 0 else "failed"), tail
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def test_untouched_copy_passes():
    name, outcome, tail = run_case(("untouched copy", C, None, None))
    assert outcome == "passed", tail


def test_every_planted_mistake_is_caught():
    py_mutants, add = load_python_mutants()
    add("sweep: beta half-step before alpha half-step",
        "alpha = sinkhorn_half_step(M, a, alpha, beta, eta, 0)\n        beta = sinkhorn_half_step(M, b, alpha, beta, eta, 1)",
        "beta = sinkhorn_half_step(M, b, alpha, beta, eta, 1)\n        alpha = sinkhorn_half_step(M, a, alpha, beta, eta, 0)")
    add("candidate choice: keeps the smaller dual objective", "return (1 if Ls > Lq else 0), Lq, Ls", "return (1 if Ls < Lq else 0), Lq, Ls")
    add("conjugate gradients: preconditioner multiplied instead of divided", "        z = r / diag\n        rz_new", "        z = r * diag\n        rz_new")
    add("conjugate gradients: residual updated with the wrong sign", "        r -= step * Ap", "        r += step * Ap")
    add("conjugate gradients: diagonal without tau", "[:m - 1]]) / eta + tau", "[:m - 1]]) / eta + 0.0 * tau")
    add("reduced system: right-hand side without the eliminated block", "res = g2 - Bt_times(g1 / d1)", "res = g2 - 0.0 * Bt_times(g1 / d1)")
    add("reduced system: Schur complement with the wrong sign", "Sq = d2 * q - Bt_times(B_times(q) / d1)", "Sq = d2 * q + Bt_times(B_times(q) / d1)")
    add("reduced system: first block not divided by its diagonal", "Sq = d2 * q - Bt_times(B_times(q) / d1)", "Sq = d2 * q - Bt_times(B_times(q))")
    add("reduced system: back-substitution drops the coupling", "x1 = (g1 - B_times(x2)) / d1", "x1 = g1 / d1")
    add("reduced system: preconditioner multiplied", "        zed = res / d2\n        rho_new", "        zed = res * d2\n        rho_new")
    add("direction: curvature test inverted", "if not ys > 1e-6 * float(y @ y):", "if ys > 1e-6 * float(y @ y):")
    add("direction: zeta with the wrong sign in the capacitance matrix", "-float(v @ s) + float(v @ w)]])", "float(v @ s) + float(v @ w)]])")
    add("direction: xi term dropped from the capacitance matrix", "K = np.array([[ys + float(y @ q), float(y @ w)],", "K = np.array([[float(y @ q), float(y @ w)],")
    add("direction: not negated", "return -(p - c[0] * q - c[1] * w), True", "return (p - c[0] * q - c[1] * w), True")
    cases = MUTANTS + py_mutants
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(run_case, cases))
    stale = [(n, t) for n, o, t in results if o == "stale"]
    assert not stale, stale
    survivors = [n for n, o, t in results if o == "passed"]
    assert not survivors, f"the pins do not notice: {survivors}"
