"""Host-side checks of libregot.so that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2605_08793_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return B.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "regot.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(regot_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert set(names) == set(B.SYMBOLS)
    for name in names:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    for code in range(0, -10, -1):
        assert B.status_string(code).startswith("REGOT_")
    assert "unknown" in B.status_string(-99)


def test_workspace_bytes(lib):
    small = B.regot_workspace_bytes(1000, 1000, -1)
    with_csr = B.regot_workspace_bytes(1000, 1000, 10000)
    assert 0 < small < with_csr
    assert small % 256 == 0 and with_csr % 256 == 0
    assert B.regot_workspace_bytes(0, 0, 0) > 0
    # the C5 problem (50000^2, 5e6 entries) stays far below the 288 GB of the device
    assert B.regot_workspace_bytes(50000, 50000, 5_500_000) < 2 << 30
    out = ctypes.c_size_t()
    assert lib.regot_workspace_bytes(-1, 5, -1, ctypes.byref(out)) == -2
    assert lib.regot_workspace_bytes(5, 1 << 31, -1, ctypes.byref(out)) == -2
    assert lib.regot_workspace_bytes(5, 5, -2, ctypes.byref(out)) == -7
    assert lib.regot_workspace_bytes(5, 5, -1, None) == -1


# fake, suitably aligned non-NULL addresses: validation must fail before anything dereferences them
P = ctypes.c_void_p(0x10000)
ODD = ctypes.c_void_p(0x10004)
P2 = ctypes.c_void_p(0x18000)
WS = ctypes.c_void_p(0x20000)
BIG = 1 << 40


def dual_eval(lib, n=8, m=8, M=P, ld=8, a=P, b=P, alpha=P, beta=P, eta=0.1, obj=P, ga=P, gb=P, rs=None, cs=None,
              ws=WS, wsb=BIG):
    return lib.regot_dual_eval(n, m, M, ld, a, b, alpha, beta, eta, obj, ga, gb, rs, cs, ws, wsb, None)


def test_dual_eval_argument_errors(lib):
    assert dual_eval(lib, n=-1) == -2
    assert dual_eval(lib, m=1 << 31, ld=1 << 31) == -2
    assert dual_eval(lib, eta=0.0) == -3
    assert dual_eval(lib, eta=-1.0) == -3
    assert dual_eval(lib, eta=float("nan")) == -3
    assert dual_eval(lib, eta=float("inf")) == -3
    assert dual_eval(lib, ld=7) == -4
    assert dual_eval(lib, M=None) == -1
    assert dual_eval(lib, a=None) == -1
    assert dual_eval(lib, beta=None) == -1
    assert dual_eval(lib, obj=None) == -1
    assert dual_eval(lib, gb=None) == -1
    assert dual_eval(lib, M=ODD) == -5
    assert dual_eval(lib, rs=ODD) == -5
    assert dual_eval(lib, ws=None) == -1
    assert dual_eval(lib, ws=ctypes.c_void_p(0x20010)) == -5
    assert dual_eval(lib, wsb=16) == -6


def test_dual_eval_noalloc_argument_errors(lib):
    """The variant with the library's own static workspace: the same checks, all before any HIP call, and a
    clear refusal of problems whose partial sums do not fit REGOT_NOALLOC_MAX_WORKSPACE (32 MiB)."""
    def call(n=8, m=8, M=P, ld=8, a=P, b=P, alpha=P, beta=P, eta=0.1, obj=P, ga=P, gb=P, rs=None, cs=None):
        return lib.regot_dual_eval_noalloc(n, m, M, ld, a, b, alpha, beta, eta, obj, ga, gb, rs, cs, None)
    assert call(n=-1) == -2
    assert call(eta=0.0) == -3
    assert call(ld=7) == -4
    assert call(M=None) == -1
    assert call(a=None) == -1
    assert call(obj=None) == -1
    assert call(cs=ODD) == -5
    assert call(n=50000, m=50000, ld=50000) == -9
    assert "static" in B.status_string(-9)
    # the limit is the documented one: what regot_workspace_bytes reports against 32 MiB
    assert B.regot_workspace_bytes(20000, 20000, -1) <= 32 << 20 < B.regot_workspace_bytes(50000, 50000, -1)
    assert B.regot_workspace_bytes(40000, 10000, -1) <= 32 << 20


def test_placement_probe_argument_errors(lib):
    assert lib.regot_placement_probe(512, None, None) == -1
    assert lib.regot_placement_probe(0, P, None) == -7
    assert lib.regot_placement_probe(1 << 20, P, None) == -7
    assert lib.regot_placement_probe(512, ctypes.c_void_p(0x10002), None) == -5


def test_read_probe_argument_errors(lib):
    def call(n=8, m=8, M=P, ld=8, out=P, ws=WS, wsb=BIG):
        return lib.regot_stream_read_probe(n, m, M, ld, out, ws, wsb, None)
    assert call(n=-1) == -2
    assert call(ld=7) == -4
    assert call(M=None) == -1
    assert call(out=None) == -1
    assert call(out=ODD) == -5
    assert call(ws=None) == -1
    assert call(wsb=16) == -6


def sparsify(lib, n=8, m=8, M=P, ld=8, alpha=P, beta=P, eta=0.1, delta=0.5, rp=P, ci=P, val=P, cap=10, info=P,
             ws=WS, wsb=BIG):
    return lib.regot_sparsify_csr(n, m, M, ld, alpha, beta, eta, delta, rp, ci, val, cap, info, ws, wsb, None)


def test_sparsify_argument_errors(lib):
    assert sparsify(lib, cap=-1) == -7
    assert sparsify(lib, delta=float("nan")) == -7
    assert sparsify(lib, rp=None) == -1
    assert sparsify(lib, info=None) == -1
    assert sparsify(lib, ci=None) == -1
    assert sparsify(lib, val=None) == -1
    assert sparsify(lib, ci=ctypes.c_void_p(0x10002)) == -5
    assert sparsify(lib, eta=0.0) == -3
    assert sparsify(lib, ld=3) == -4
    assert sparsify(lib, wsb=1024) == -6
    # fused entry point shares the checks
    assert lib.regot_dual_eval_sparsify(8, 8, P, 8, P, P, P, P, 0.1, P, P, P, None, None, 0.5, P, P, P, -3, P,
                                        WS, BIG, None) == -7
    assert lib.regot_dual_eval_sparsify(8, 8, P, 8, P, P, P, P, 0.1, None, P, P, None, None, 0.5, P, P, P, 3, P,
                                        WS, BIG, None) == -1


def half_step(lib, n=8, m=8, M=P, ld=8, marg=P, alpha=P, beta=P, eta=0.1, which=0, out=P, ws=WS, wsb=BIG):
    return lib.regot_sinkhorn_half_step(n, m, M, ld, marg, alpha, beta, eta, which, out, ws, wsb, None)


def refresh(lib, n=2000, m=2000, M=P, ld=2000, a=P, b=P, alpha=P, beta=P, eta=0.1, k=500, obj=P, ga=P, gb=P, rs=None,
            cs=None, delta=P, rp=P, ci=P, val=P, cap=1000, info=P, ws=WS, wsb=BIG, tws=WS, twsb=BIG):
    return lib.regot_dual_eval_sparsify_topk(n, m, M, ld, a, b, alpha, beta, eta, k, obj, ga, gb, rs, cs, delta, rp, ci, val,
                                             cap, info, ws, wsb, tws, twsb, None)


def test_refresh_argument_errors(lib):
    assert refresh(lib, k=0) == -7
    assert refresh(lib, k=2000 * 2000 + 1) == -7
    assert refresh(lib, n=0) == -2
    assert refresh(lib, eta=0.0) == -3
    assert refresh(lib, ld=100) == -4
    for name in ("M", "a", "b", "alpha", "beta", "obj", "ga", "gb", "delta", "rp", "ci", "val", "info"):
        assert refresh(lib, **{name: None}) == -1, name
    assert refresh(lib, cap=-1) == -7
    assert refresh(lib, delta=ODD) == -5
    assert refresh(lib, ws=None) == -1
    assert refresh(lib, wsb=1024) == -6
    assert refresh(lib, tws=None) == -1
    assert refresh(lib, twsb=1024) == -6
    out = ctypes.c_int64()
    assert lib.regot_refresh_candidate_capacity(0, 5, 1, ctypes.byref(out)) == -2
    assert lib.regot_refresh_candidate_capacity(5, 5, 26, ctypes.byref(out)) == -7
    assert lib.regot_refresh_candidate_capacity(5, 5, 1, None) == -1
    # candidates: k and a fraction of a percent of the matrix more, never more than the matrix
    c3 = B.regot_refresh_candidate_capacity(20000, 20000, 2_000_000)
    assert 2_000_000 < c3 < 4_000_000
    assert B.regot_refresh_candidate_capacity(100, 100, 5000) == 100 * 100


def test_half_step_argument_errors(lib):
    assert half_step(lib, which=2) == -7
    assert half_step(lib, which=-1) == -7
    assert half_step(lib, n=0) == -2          # the update is undefined on an empty problem
    assert half_step(lib, m=0, ld=0) == -2
    assert half_step(lib, marg=None) == -1
    assert half_step(lib, which=0, beta=None) == -1
    assert half_step(lib, which=1, alpha=None) == -1
    assert half_step(lib, out=None) == -1
    assert half_step(lib, eta=-0.5) == -3
    assert half_step(lib, wsb=0) == -6
    assert half_step(lib, out=ODD) == -5


def topk(lib, n=8, m=8, M=P, ld=8, alpha=P, beta=P, eta=0.1, k=5, delta=P, s_k=None, info=P, ws=WS, wsb=BIG):
    return lib.regot_topk_threshold(n, m, M, ld, alpha, beta, eta, k, delta, s_k, info, ws, wsb, None)


def test_topk_argument_errors(lib):
    assert topk(lib, k=0) == -7
    assert topk(lib, k=65) == -7              # k > n*m
    assert topk(lib, k=-3) == -7
    assert topk(lib, n=0) == -2               # no k-th largest entry of an empty matrix
    assert topk(lib, m=0, ld=0) == -2
    assert topk(lib, eta=0.0) == -3
    assert topk(lib, ld=7) == -4
    assert topk(lib, M=None) == -1
    assert topk(lib, alpha=None) == -1
    assert topk(lib, beta=None) == -1
    assert topk(lib, delta=None) == -1
    assert topk(lib, info=None) == -1
    assert topk(lib, s_k=ODD) == -5
    assert topk(lib, ws=None) == -1
    assert topk(lib, wsb=4096) == -6


def test_topk_workspace_bytes(lib):
    out = ctypes.c_size_t()
    assert lib.regot_topk_workspace_bytes(5, 5, 0, ctypes.byref(out)) == -7
    assert lib.regot_topk_workspace_bytes(5, 5, 26, ctypes.byref(out)) == -7
    assert lib.regot_topk_workspace_bytes(0, 5, 1, ctypes.byref(out)) == -2
    assert lib.regot_topk_workspace_bytes(5, 5, 1, None) == -1
    tiny = B.regot_topk_workspace_bytes(5, 5, 3)
    assert 0 < tiny < 2 << 20 and tiny % 256 == 0
    # the pool grows with k but stays below 1/16 of the matrix (+ the fixed part)
    c3_small = B.regot_topk_workspace_bytes(20000, 20000, 1000)
    c3 = B.regot_topk_workspace_bytes(20000, 20000, 2_000_000)
    c3_all = B.regot_topk_workspace_bytes(20000, 20000, 400_000_000)
    assert c3_small < c3 <= c3_all <= 20000 * 20000 * 8 // 16 + (2 << 20)
    assert B.regot_topk_workspace_bytes(50000, 50000, 2_500_000_000) <= (1 << 31) + (2 << 20)


def pattern_values(lib, n=8, m=8, M=P, ld=8, alpha=P, beta=P, eta=0.1, rp=P, ci=P, pos=None, cap=10, val=P, valc=None):
    return lib.regot_pattern_values(n, m, M, ld, alpha, beta, eta, rp, ci, pos, cap, val, valc, None)


def test_pattern_values_argument_errors(lib):
    assert pattern_values(lib, cap=-1) == -7
    assert pattern_values(lib, rp=None) == -1
    assert pattern_values(lib, ci=None) == -1
    assert pattern_values(lib, val=None) == -1
    assert pattern_values(lib, valc=P) == -1          # column-order values need csc_pos
    assert pattern_values(lib, ci=ctypes.c_void_p(0x10002)) == -5
    assert pattern_values(lib, eta=0.0) == -3
    assert pattern_values(lib, ld=3) == -4
    assert pattern_values(lib, n=0) == 0              # nothing to do, nothing enqueued
    assert pattern_values(lib, cap=0, ci=None, val=None) == 0


def test_pattern_transpose_argument_errors(lib):
    out = ctypes.c_size_t()
    assert lib.regot_pattern_transpose_workspace_bytes(5, 5, -1, ctypes.byref(out)) == -7
    assert lib.regot_pattern_transpose_workspace_bytes(5, 5, 1 << 31, ctypes.byref(out)) == -7
    assert lib.regot_pattern_transpose_workspace_bytes(-1, 5, 3, ctypes.byref(out)) == -2
    assert lib.regot_pattern_transpose_workspace_bytes(5, 5, 3, None) == -1
    small = B.regot_pattern_transpose_workspace_bytes(100, 100, 0)
    big = B.regot_pattern_transpose_workspace_bytes(20000, 20000, 2_000_000)
    assert 0 < small < big < 64 << 20 and big % 256 == 0
    f = lib.regot_pattern_transpose
    assert f(8, 8, 5, None, P, P, P, P, WS, BIG, None) == -1
    assert f(8, 8, 5, P, None, P, P, P, WS, BIG, None) == -1
    assert f(8, 8, 5, P, P, P, P, ODD, WS, BIG, None) == -5
    assert f(8, 8, 5, P, P, P, P, P, None, BIG, None) == -1
    assert f(8, 8, 5, P, P, P, P, P, WS, 64, None) == -6
    assert f(8, 8, -2, P, P, P, P, P, WS, BIG, None) == -7


def matvec(lib, n=8, m=8, eta=0.1, tau=0.0, rp=P, ci=P, val=P, cp=P, ri=P, valc=P, cap=10, r=P, c=P, x=P, y=P):
    return lib.regot_hessian_matvec(n, m, eta, tau, rp, ci, val, cp, ri, valc, cap, r, c, x, y, None)


def test_hessian_argument_errors(lib):
    assert matvec(lib, n=0) == -2
    assert matvec(lib, m=0) == -2
    assert matvec(lib, eta=-1.0) == -3
    assert matvec(lib, tau=float("nan")) == -7
    assert matvec(lib, cap=-4) == -7
    for name in ("rp", "ci", "val", "cp", "ri", "valc", "r", "c", "x", "y"):
        assert matvec(lib, **{name: None}) == -1, name
    assert matvec(lib, y=ODD) == -5
    out = ctypes.c_size_t()
    assert lib.regot_hessian_workspace_bytes(0, 5, ctypes.byref(out)) == -2
    assert lib.regot_hessian_workspace_bytes(5, 5, None) == -1
    assert 0 < B.regot_hessian_workspace_bytes(50000, 50000) < 1 << 20

    def lower(n=8, m=8, eta=0.1, tau=0.0, rp=P, ci=P, val=P, cap=10, r=P, c=P, hcp=P, hri=P, hv=P, hcap=30, info=P,
              vo=0, ws=WS, wsb=BIG):
        return lib.regot_hessian_lower_csc(n, m, eta, tau, rp, ci, val, cap, r, c, hcp, hri, hv, hcap, info, vo, ws, wsb,
                                           None)
    assert lower(n=0) == -2
    assert lower(eta=0.0) == -3
    assert lower(vo=2) == -7
    assert lower(hcap=-1) == -7
    assert lower(hcp=None) == -1
    assert lower(info=None) == -1
    assert lower(hv=None) == -1
    assert lower(hri=ctypes.c_void_p(0x10002)) == -5
    assert lower(ws=None) == -1
    assert lower(wsb=8) == -6


def test_metrics_and_choice_argument_errors(lib):
    def metrics(n=8, m=8, a=P, b=P, alpha=P, beta=P, eta=0.1, r=P, c=P, out=P, ws=WS, wsb=BIG):
        return lib.regot_dual_metrics(n, m, a, b, alpha, beta, eta, r, c, out, ws, wsb, None)
    assert metrics(n=-1) == -2
    assert metrics(eta=0.0) == -3
    for name in ("a", "b", "alpha", "beta", "r", "c", "out"):
        assert metrics(**{name: None}) == -1, name
    assert metrics(out=ODD) == -5
    assert metrics(ws=None) == -1
    assert metrics(wsb=64) == -6

    def choose(n=8, m=8, oq=P, os_=P, aq=P, bq=P, as_=P, bs=P, ao=P, bo=P, ch=P):
        return lib.regot_choose_candidate(n, m, oq, os_, aq, bq, as_, bs, ao, bo, ch, None)
    assert choose(m=-3) == -2
    for name in ("oq", "os_", "aq", "bq", "as_", "bs", "ao", "bo", "ch"):
        assert choose(**{name: None}) == -1, name
    assert choose(ch=ODD) == -5


def test_pcg_and_direction_argument_errors(lib):
    def pcg(n=8, m=8, eta=0.1, tau=0.0, rp=P, ci=P, val=P, cp=P, ri=P, valc=P, cap=10, r=P, c=P, rhs=P, x=P, rtol=1e-8,
            its=5, restart=1, info=P, ws=WS, wsb=BIG):
        return lib.regot_pcg_solve(n, m, eta, tau, rp, ci, val, cp, ri, valc, cap, r, c, rhs, x, rtol, its, restart, info,
                                   ws, wsb, None)
    assert pcg(n=0) == -2
    assert pcg(eta=0.0) == -3
    assert pcg(rtol=-1.0) == -7
    assert pcg(rtol=float("nan")) == -7
    assert pcg(its=-1) == -7
    assert pcg(restart=3) == -7
    for name in ("rp", "ci", "val", "cp", "ri", "valc", "r", "c", "rhs", "x", "info"):
        assert pcg(**{name: None}) == -1, name
    assert pcg(x=ODD) == -5
    assert pcg(ws=None) == -1
    assert pcg(wsb=128) == -6
    out = ctypes.c_size_t()
    assert lib.regot_pcg_workspace_bytes(0, 3, ctypes.byref(out)) == -2
    assert lib.regot_pcg_workspace_bytes(3, 3, None) == -1
    assert B.regot_pcg_workspace_bytes(20000, 20000) < 4 << 20       # ten vectors of 40000 doubles and some KB

    def reduced(n=8, m=8, eta=0.1, tau=0.0, rp=P, ci=P, val=P, cp=P, ri=P, valc=P, cap=10, r=P, c=P, rhs=P, x=P, rtol=1e-8,
                its=5, restart=1, info=P, ws=WS, wsb=BIG):
        return lib.regot_pcg_solve_reduced(n, m, eta, tau, rp, ci, val, cp, ri, valc, cap, r, c, rhs, x, rtol, its, restart,
                                           info, ws, wsb, None)
    assert reduced(m=0) == -2
    assert reduced(eta=float("inf")) == -3
    assert reduced(rtol=-1.0) == -7
    assert reduced(its=-1) == -7
    assert reduced(restart=2) == -7
    assert reduced(cap=-1) == -7
    for name in ("rp", "ci", "val", "cp", "ri", "valc", "r", "c", "rhs", "x", "info"):
        assert reduced(**{name: None}) == -1, name
    assert reduced(rhs=ODD) == -5
    assert reduced(ws=None) == -1
    assert reduced(wsb=128) == -6

    def pcg2(n=8, m=8, eta=0.1, tau=0.0, rp=P, ci=P, val=P, cp=P, ri=P, valc=P, cap=10, r=P, c=P, rhs_a=P, rhs_b=P, x_a=P,
             x_b=P2, rtol=1e-8, its=5, restart=1, info=P, ws=WS, wsb=BIG):
        return lib.regot_pcg_solve2(n, m, eta, tau, rp, ci, val, cp, ri, valc, cap, r, c, rhs_a, rhs_b, x_a, x_b, rtol,
                                    its, restart, info, ws, wsb, None)
    assert pcg2(m=0) == -2
    assert pcg2(eta=-1.0) == -3
    assert pcg2(its=100001) == -7
    for name in ("rp", "cp", "r", "c", "rhs_a", "rhs_b", "x_a", "x_b", "info"):
        assert pcg2(**{name: None}) == -1, name
    assert pcg2(x_b=P) == -7                          # the two solutions need two arrays
    assert pcg2(rhs_b=ODD) == -5
    assert pcg2(wsb=128) == -6

    def reduced2(n=8, m=8, eta=0.1, tau=0.0, rp=P, ci=P, val=P, cp=P, ri=P, valc=P, cap=10, r=P, c=P, rhs_a=P, rhs_b=P,
                 x_a=P, x_b=P2, rtol=1e-8, its=5, restart=1, info=P, ws=WS, wsb=BIG):
        return lib.regot_pcg_solve2_reduced(n, m, eta, tau, rp, ci, val, cp, ri, valc, cap, r, c, rhs_a, rhs_b, x_a, x_b,
                                            rtol, its, restart, info, ws, wsb, None)
    assert reduced2(n=0) == -2
    assert reduced2(eta=0.0) == -3
    assert reduced2(its=100001) == -7
    for name in ("rp", "cp", "r", "c", "rhs_a", "rhs_b", "x_a", "x_b", "info"):
        assert reduced2(**{name: None}) == -1, name
    assert reduced2(x_b=P) == -7
    assert reduced2(x_a=ODD) == -5
    assert reduced2(wsb=128) == -6

    def direction(n=8, m=8, p=P, q=P, s=P, y=P, v=P, d=P, info=P, ws=WS, wsb=BIG):
        return lib.regot_splr_direction(n, m, p, q, s, y, v, d, info, ws, wsb, None)
    assert direction(ws=None) == -1
    assert direction(wsb=64) == -6
    assert direction(m=0) == -2
    assert direction(p=None) == -1
    assert direction(d=None) == -1
    assert direction(info=None) == -1
    assert direction(q=None) == -1                    # the previous-step vectors come all or none
    assert direction(v=ODD) == -5


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(TypeError):
        B._ws(torch.zeros(256, dtype=torch.uint8))     # a host pointer as workspace would fault in the kernels
    M = torch.zeros(4, 4, dtype=torch.float64)
    v = torch.zeros(4, dtype=torch.float64)
    with pytest.raises(TypeError):
        B.regot_dual_eval(M, v, v, v, v, 0.1, torch.zeros(1, dtype=torch.float64), v, v, workspace=torch.zeros(256))


def test_binding_refuses_views_that_are_not_dense_rows():
    """A row stride below m (an expanded row, an overlapping view) would be read as n dense rows."""
    import torch
    row = torch.zeros(8, dtype=torch.float64)
    with pytest.raises(TypeError):
        B._matrix_layout(row.expand(5, 8))                      # stride (0, 1)
    with pytest.raises(TypeError):
        B._matrix_layout(torch.zeros(40, dtype=torch.float64).as_strided((5, 8), (4, 1)))   # overlapping rows
    with pytest.raises(TypeError):
        B._matrix_layout(torch.zeros(8, 5, dtype=torch.float64).t())                        # column-major
    big = torch.zeros(6, 12, dtype=torch.float64)
    assert B._matrix_layout(big) == (6, 12, 12)
    assert B._matrix_layout(big[1:5, 2:10]) == (4, 8, 12)       # a strided block of a larger matrix
    assert B._matrix_layout(big[2:3, 1:4]) == (1, 3, 3)
    assert B._matrix_layout(torch.zeros(0, 7, dtype=torch.float64))[:2] == (0, 7)


def test_chunk_height_fits_the_record_format(lib):
    """A staged CSR entry keeps its row relative to its chunk in 14 bits: no chunk may be taller than 16384
    rows, in particular not for n just below or above multiples of 16384 rows per chunk."""
    cases = [(212991, 20000, 10**6), (32767, 132096, 10**6), (229375, 20000, 10**6), (16384 * 13 - 1, 20000, 0),
             (16384 * 13, 20000, 0), (16384 * 13 + 1, 20000, 0), (2**31 - 1, 1, 0), (2**31 - 1, 600, 10**8)]
    for base in (16380, 16384):
        for g in (1, 2, 3, 12, 13, 25, 51, 512):
            for d in range(-5, 6):
                cases.append((base * g + d, 20000, 10**6))
                cases.append((base * g + d, 512 * 300, 10**9))
    for n, m, cap in cases:
        if n < 1:
            continue
        for capacity in (-1, cap):
            g_r, g_c, rounds, tallest, strip = B.regot_plan_geometry(n, m, capacity)
            assert g_c == (m + 511) // 512 and g_r >= 1 and 1 <= rounds <= 4
            assert tallest <= 16384, (n, m, capacity, g_r, tallest)
            assert tallest >= (n + g_r - 1) // g_r
            assert 0 <= strip <= g_r and (strip == 0 or (g_r * (g_c - 1) + strip <= 512 * rounds and m - 512 * (g_c - 1) <= 32))
    # the benchmark shape: 39 full panels x 13 chunks and the 32-column strip on the five places left
    assert B.regot_plan_geometry(20000, 20000, 2_201_024) == (13, 40, 1, 1540, 5)
    assert B.regot_plan_geometry(40000, 10000, 4_400_000)[4] == 0          # a wide last panel stays a panel
    out = (ctypes.c_int64 * 5)()
    assert lib.regot_plan_geometry(-1, 5, -1, out) == -2
    assert lib.regot_plan_geometry(5, 5, -2, out) == -7
    assert lib.regot_plan_geometry(5, 5, -1, None) == -1
    assert B.regot_plan_geometry(0, 0, -1)[0] == 0


def test_product_never_imports_the_oracle():
    """The oracle is test infrastructure: nothing under the package may import, load or run it."""
    pkg = os.path.join(ROOT, "paper_2605_08793_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if not f.endswith((".py", ".hip", ".hpp", ".h")):
                continue
            text = open(os.path.join(dirpath, f)).read()
            assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), f
            assert "liboracle" not in text and "regot_oracle" not in text, f
    text = open(os.path.join(ROOT, "oracle", "__init__.py")).read() + open(os.path.join(ROOT, "oracle", "regot_oracle.c")).read()
    assert "paper_2605_08793_amd" not in text and "libregot" not in text


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asking for more must end with a message, not with a number."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)
    assert "{" not in r.stdout


def test_sinkhorn_sweeps_argument_errors(lib):
    def sweeps(n=8, m=8, M=P, ld=8, a=P, b=P, alpha=P, beta=P, eta=0.1, k=3, ws=WS, wsb=BIG):
        return lib.regot_sinkhorn_sweeps(n, m, M, ld, a, b, alpha, beta, eta, k, ws, wsb, None)
    assert sweeps(k=-1) == -7
    assert sweeps(alpha=None) == -1
    assert sweeps(beta=None) == -1
    assert sweeps(a=None) == -1
    assert sweeps(M=None) == -1
    assert sweeps(ld=4) == -4
    assert sweeps(eta=0.0) == -3
    assert sweeps(n=-1) == -2
    assert sweeps(ws=None) == -1
    assert sweeps(wsb=64) == -6
    assert sweeps(k=0) == 0                           # nothing to enqueue
    assert sweeps(k=0, b=None) == -1 and sweeps(k=0, ld=2) == -4


def test_header_is_plain_c_and_links_from_c(tmp_path):
    """include/regot.h compiles as C99 and as C++ without warnings, and a C program linked against the library can make
    the host-side calls (no GPU work is enqueued)."""
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    inc = os.path.join(root, "include")
    src = tmp_path / "use_regot.c"
    src.write_text(
        '#include <stdio.h>\n#include "regot.h"\n'
        'int main(void) {\n'
        '    size_t bytes = 0; int64_t g[5];\n'
        '    if (regot_workspace_bytes(1000, 2000, 50000, &bytes) != REGOT_OK || bytes == 0) return 1;\n'
        '    if (regot_plan_geometry(20000, 20000, 2200000, g) != REGOT_OK || g[1] != 40 || g[2] != 1) return 2;\n'
        '    if (regot_workspace_bytes(-1, 5, -1, &bytes) != REGOT_ERR_DIM) return 3;\n'
        '    printf("%s\\n", regot_status_string(REGOT_ERR_LD));\n'
        '    return 0;\n}\n')
    gcc, gxx = shutil.which("gcc"), shutil.which("g++")
    if gcc is None:
        pytest.skip("no C compiler")
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    if gxx is not None:
        subprocess.run([gxx, "-std=c++11", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)],
                       check=True)
    exe = tmp_path / "use_regot"
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-l:" + os.path.basename(B.LIB_PATH),
                    "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, stdout=subprocess.PIPE, text=True).stdout
    assert "REGOT_ERR_LD" in out
