"""ctypes binding of libregot.so: argument marshalling only.

Each function has the name of the C entry point it calls (see include/regot.h).
PyTorch is used for device memory and for the current stream; every step of the
computation runs in the HIP kernels.  There is no fallback: if the library is not
built, the first call raises.
"""
import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libregot.so")

SYMBOLS = (
    "regot_status_string",
    "regot_workspace_bytes",
    "regot_plan_geometry",
    "regot_dual_eval",
    "regot_dual_eval_noalloc",
    "regot_sparsify_csr",
    "regot_dual_eval_sparsify",
    "regot_sinkhorn_half_step",
    "regot_sinkhorn_sweeps",
    "regot_topk_workspace_bytes",
    "regot_topk_threshold",
    "regot_pattern_values",
    "regot_pattern_transpose_workspace_bytes",
    "regot_pattern_transpose",
    "regot_hessian_matvec",
    "regot_hessian_workspace_bytes",
    "regot_hessian_lower_csc",
    "regot_dual_metrics",
    "regot_choose_candidate",
    "regot_pcg_workspace_bytes",
    "regot_refresh_candidate_capacity",
    "regot_dual_eval_sparsify_topk",
    "regot_pcg_solve",
    "regot_pcg_solve2",
    "regot_pcg_solve_reduced",
    "regot_pcg_solve2_reduced",
    "regot_splr_direction",
    "regot_profile_stage1",
    "regot_stream_read_probe",
    "regot_placement_probe",
)

_lib = None


class RegotError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def load():
    """Open libregot.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2605_08793_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    i64, dbl, p, sz = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_size_t
    lib.regot_status_string.argtypes = [ctypes.c_int]
    lib.regot_status_string.restype = ctypes.c_char_p
    lib.regot_workspace_bytes.argtypes = [i64, i64, i64, ctypes.POINTER(sz)]
    lib.regot_plan_geometry.argtypes = [i64, i64, i64, ctypes.POINTER(i64)]
    lib.regot_dual_eval.argtypes = [i64, i64, p, i64, p, p, p, p, dbl, p, p, p, p, p, p, sz, p]
    lib.regot_dual_eval_noalloc.argtypes = [i64, i64, p, i64, p, p, p, p, dbl, p, p, p, p, p, p]
    lib.regot_sparsify_csr.argtypes = [i64, i64, p, i64, p, p, dbl, dbl, p, p, p, i64, p, p, sz, p]
    lib.regot_dual_eval_sparsify.argtypes = [i64, i64, p, i64, p, p, p, p, dbl, p, p, p, p, p,
                                             dbl, p, p, p, i64, p, p, sz, p]
    lib.regot_sinkhorn_half_step.argtypes = [i64, i64, p, i64, p, p, p, dbl, ctypes.c_int, p, p, sz, p]
    lib.regot_sinkhorn_sweeps.argtypes = [i64, i64, p, i64, p, p, p, p, dbl, ctypes.c_int, p, sz, p]
    lib.regot_topk_workspace_bytes.argtypes = [i64, i64, i64, ctypes.POINTER(sz)]
    lib.regot_topk_threshold.argtypes = [i64, i64, p, i64, p, p, dbl, i64, p, p, p, p, sz, p]
    lib.regot_pattern_values.argtypes = [i64, i64, p, i64, p, p, dbl, p, p, p, i64, p, p, p]
    lib.regot_pattern_transpose_workspace_bytes.argtypes = [i64, i64, i64, ctypes.POINTER(sz)]
    lib.regot_pattern_transpose.argtypes = [i64, i64, i64, p, p, p, p, p, p, sz, p]
    lib.regot_hessian_matvec.argtypes = [i64, i64, dbl, dbl, p, p, p, p, p, p, i64, p, p, p, p, p]
    lib.regot_hessian_workspace_bytes.argtypes = [i64, i64, ctypes.POINTER(sz)]
    lib.regot_hessian_lower_csc.argtypes = [i64, i64, dbl, dbl, p, p, p, i64, p, p, p, p, p, i64, p, ctypes.c_int,
                                            p, sz, p]
    lib.regot_dual_metrics.argtypes = [i64, i64, p, p, p, p, dbl, p, p, p, p, sz, p]
    lib.regot_choose_candidate.argtypes = [i64, i64, p, p, p, p, p, p, p, p, p, p]
    lib.regot_refresh_candidate_capacity.argtypes = [i64, i64, i64, ctypes.POINTER(i64)]
    lib.regot_dual_eval_sparsify_topk.argtypes = [i64, i64, p, i64, p, p, p, p, dbl, i64, p, p, p, p, p, p, p, p, p, i64, p,
                                                  p, sz, p, sz, p]
    lib.regot_pcg_workspace_bytes.argtypes = [i64, i64, ctypes.POINTER(sz)]
    lib.regot_pcg_solve.argtypes = [i64, i64, dbl, dbl, p, p, p, p, p, p, i64, p, p, p, p, dbl, ctypes.c_int, ctypes.c_int,
                                    p, p, sz, p]
    lib.regot_pcg_solve_reduced.argtypes = lib.regot_pcg_solve.argtypes
    lib.regot_pcg_solve2.argtypes = [i64, i64, dbl, dbl, p, p, p, p, p, p, i64, p, p, p, p, p, p, dbl, ctypes.c_int,
                                     ctypes.c_int, p, p, sz, p]
    lib.regot_pcg_solve2_reduced.argtypes = lib.regot_pcg_solve2.argtypes
    lib.regot_splr_direction.argtypes = [i64, i64, p, p, p, p, p, p, p, p, sz, p]
    lib.regot_profile_stage1.argtypes = [p, p]
    lib.regot_stream_read_probe.argtypes = [i64, i64, p, i64, p, p, sz, p]
    lib.regot_placement_probe.argtypes = [ctypes.c_int, p, p]
    for name in SYMBOLS[1:]:
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().regot_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise RegotError(status, where)


def _p(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _ws(workspace: torch.Tensor):
    """(pointer, bytes) of a workspace; it has to live on the device, a host pointer would fault in the kernels."""
    if not isinstance(workspace, torch.Tensor) or not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous CUDA tensor")
    return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _matrix(M: torch.Tensor):
    if not isinstance(M, torch.Tensor) or not M.is_cuda:
        raise TypeError("M must be a 2-D float64 CUDA tensor")
    return _matrix_layout(M)


def _matrix_layout(M: torch.Tensor):
    """(n, m, ldM) of a row-major float64 matrix, after checking that n rows of m elements at that
    leading dimension lie inside its storage (the kernels read exactly those)."""
    if M.dtype != torch.float64 or M.dim() != 2:
        raise TypeError("M must be a 2-D float64 CUDA tensor")
    n, m = M.shape
    if n > 0 and m > 0 and M.stride(1) != 1:
        raise TypeError("M must be row-major (unit stride along columns)")
    if n > 1 and m > 0 and M.stride(0) < m:
        # an expanded or overlapping view: the kernels would read n dense rows from a storage that
        # need not hold them
        raise TypeError(f"M must have a row stride of at least m = {m} elements (got {M.stride(0)})")
    ld = M.stride(0) if (n > 1 and m > 0) else max(m, 1)
    if n > 0 and m > 0:
        have = M.untyped_storage().nbytes() // M.element_size()
        if M.storage_offset() + (n - 1) * ld + m > have:
            raise TypeError("M reaches beyond its storage")
    return n, m, ld


def _vector(v: Optional[torch.Tensor], length: int, name: str, dtype=torch.float64, optional=False):
    if v is None:
        if optional:
            return None
        raise TypeError(f"{name} is required")
    if v.dtype != dtype or not v.is_cuda or v.dim() != 1 or v.numel() != length or (length > 1 and v.stride(0) != 1):
        raise TypeError(f"{name} must be a contiguous 1-D {dtype} CUDA tensor of length {length}")
    return v


def regot_workspace_bytes(n: int, m: int, csr_capacity: int = -1) -> int:
    out = ctypes.c_size_t(0)
    _check(load().regot_workspace_bytes(int(n), int(m), int(csr_capacity), ctypes.byref(out)),
           "regot_workspace_bytes")
    return int(out.value)


def regot_plan_geometry(n: int, m: int, csr_capacity: int = -1):
    """(g_r, g_c, rounds, rows of the tallest chunk, strip workgroups) of the dense calls' decomposition."""
    out = (ctypes.c_int64 * 5)()
    _check(load().regot_plan_geometry(int(n), int(m), int(csr_capacity), out), "regot_plan_geometry")
    return tuple(int(x) for x in out)


def new_workspace(n: int, m: int, csr_capacity: int = -1, device="cuda") -> torch.Tensor:
    """A device buffer of the size regot_workspace_bytes() asks for (torch allocations are 256-byte aligned)."""
    return torch.empty(max(regot_workspace_bytes(n, m, csr_capacity), 256), dtype=torch.uint8, device=device)


def regot_dual_eval(M, a, b, alpha, beta, eta, obj, grad_alpha, grad_beta, row_sum=None, col_sum=None, *,
                    workspace, stream=None) -> None:
    n, m, ld = _matrix(M)
    _check(load().regot_dual_eval(
        n, m, _p(M), ld, _p(_vector(a, n, "a")), _p(_vector(b, m, "b")),
        _p(_vector(alpha, n, "alpha")), _p(_vector(beta, m, "beta")), float(eta),
        _p(_vector(obj, 1, "obj")), _p(_vector(grad_alpha, n, "grad_alpha")), _p(_vector(grad_beta, m, "grad_beta")),
        _p(_vector(row_sum, n, "row_sum", optional=True)), _p(_vector(col_sum, m, "col_sum", optional=True)),
        *_ws(workspace), _stream(stream)), "regot_dual_eval")


def regot_dual_eval_noalloc(M, a, b, alpha, beta, eta, obj, grad_alpha, grad_beta, row_sum=None, col_sum=None, *,
                            stream=None) -> None:
    n, m, ld = _matrix(M)
    _check(load().regot_dual_eval_noalloc(
        n, m, _p(M), ld, _p(_vector(a, n, "a")), _p(_vector(b, m, "b")),
        _p(_vector(alpha, n, "alpha")), _p(_vector(beta, m, "beta")), float(eta),
        _p(_vector(obj, 1, "obj")), _p(_vector(grad_alpha, n, "grad_alpha")), _p(_vector(grad_beta, m, "grad_beta")),
        _p(_vector(row_sum, n, "row_sum", optional=True)), _p(_vector(col_sum, m, "col_sum", optional=True)),
        _stream(stream)), "regot_dual_eval_noalloc")


def regot_sparsify_csr(M, alpha, beta, eta, delta, row_ptr, col_idx, val, info, *, workspace, stream=None) -> None:
    n, m, ld = _matrix(M)
    capacity = int(col_idx.numel())
    _vector(val, capacity, "val")
    _vector(col_idx, capacity, "col_idx", torch.int32)
    _check(load().regot_sparsify_csr(
        n, m, _p(M), ld, _p(_vector(alpha, n, "alpha")), _p(_vector(beta, m, "beta")), float(eta), float(delta),
        _p(_vector(row_ptr, n + 1, "row_ptr", torch.int64)), _p(col_idx), _p(val), capacity,
        _p(_vector(info, 2, "info", torch.int64)),
        *_ws(workspace), _stream(stream)), "regot_sparsify_csr")


def regot_dual_eval_sparsify(M, a, b, alpha, beta, eta, obj, grad_alpha, grad_beta, row_sum, col_sum,
                             delta, row_ptr, col_idx, val, info, *, workspace, stream=None) -> None:
    n, m, ld = _matrix(M)
    capacity = int(col_idx.numel())
    _vector(val, capacity, "val")
    _vector(col_idx, capacity, "col_idx", torch.int32)
    _check(load().regot_dual_eval_sparsify(
        n, m, _p(M), ld, _p(_vector(a, n, "a")), _p(_vector(b, m, "b")),
        _p(_vector(alpha, n, "alpha")), _p(_vector(beta, m, "beta")), float(eta),
        _p(_vector(obj, 1, "obj")), _p(_vector(grad_alpha, n, "grad_alpha")), _p(_vector(grad_beta, m, "grad_beta")),
        _p(_vector(row_sum, n, "row_sum", optional=True)), _p(_vector(col_sum, m, "col_sum", optional=True)),
        float(delta), _p(_vector(row_ptr, n + 1, "row_ptr", torch.int64)), _p(col_idx), _p(val), capacity,
        _p(_vector(info, 2, "info", torch.int64)),
        *_ws(workspace), _stream(stream)), "regot_dual_eval_sparsify")


def regot_refresh_candidate_capacity(n: int, m: int, k: int) -> int:
    out = ctypes.c_int64(0)
    _check(load().regot_refresh_candidate_capacity(int(n), int(m), int(k), ctypes.byref(out)),
           "regot_refresh_candidate_capacity")
    return int(out.value)


def regot_dual_eval_sparsify_topk(M, a, b, alpha, beta, eta, k, obj, grad_alpha, grad_beta, row_sum, col_sum, delta,
                                  row_ptr, col_idx, val, info, *, workspace, topk_workspace, stream=None) -> None:
    n, m, ld = _matrix(M)
    capacity = int(col_idx.numel())
    _vector(val, capacity, "val")
    _vector(col_idx, capacity, "col_idx", torch.int32)
    _check(load().regot_dual_eval_sparsify_topk(
        n, m, _p(M), ld, _p(_vector(a, n, "a")), _p(_vector(b, m, "b")),
        _p(_vector(alpha, n, "alpha")), _p(_vector(beta, m, "beta")), float(eta), int(k),
        _p(_vector(obj, 1, "obj")), _p(_vector(grad_alpha, n, "grad_alpha")), _p(_vector(grad_beta, m, "grad_beta")),
        _p(_vector(row_sum, n, "row_sum", optional=True)), _p(_vector(col_sum, m, "col_sum", optional=True)),
        _p(_vector(delta, 1, "delta")), _p(_vector(row_ptr, n + 1, "row_ptr", torch.int64)), _p(col_idx), _p(val),
        capacity, _p(_vector(info, 2, "info", torch.int64)), *_ws(workspace), *_ws(topk_workspace), _stream(stream)),
        "regot_dual_eval_sparsify_topk")


def regot_sinkhorn_half_step(M, marginal, alpha, beta, eta, which, out, *, workspace, stream=None) -> None:
    n, m, ld = _matrix(M)
    length = n if which == 0 else m
    _check(load().regot_sinkhorn_half_step(
        n, m, _p(M), ld, _p(_vector(marginal, length, "marginal")),
        _p(_vector(alpha, n, "alpha", optional=(which == 0))), _p(_vector(beta, m, "beta", optional=(which == 1))),
        float(eta), int(which), _p(_vector(out, length, "out")),
        *_ws(workspace), _stream(stream)), "regot_sinkhorn_half_step")


def regot_sinkhorn_sweeps(M, a, b, alpha, beta, eta, sweeps, *, workspace, stream=None) -> None:
    n, m, ld = _matrix(M)
    _check(load().regot_sinkhorn_sweeps(
        n, m, _p(M), ld, _p(_vector(a, n, "a")), _p(_vector(b, m, "b")), _p(_vector(alpha, n, "alpha")),
        _p(_vector(beta, m, "beta")), float(eta), int(sweeps), *_ws(workspace), _stream(stream)), "regot_sinkhorn_sweeps")


def regot_topk_workspace_bytes(n: int, m: int, k: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().regot_topk_workspace_bytes(int(n), int(m), int(k), ctypes.byref(out)),
           "regot_topk_workspace_bytes")
    return int(out.value)


def new_topk_workspace(n: int, m: int, k: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(regot_topk_workspace_bytes(n, m, k), 256), dtype=torch.uint8, device=device)


def regot_topk_threshold(M, alpha, beta, eta, k, delta, s_k, info, *, workspace, stream=None) -> None:
    n, m, ld = _matrix(M)
    _check(load().regot_topk_threshold(
        n, m, _p(M), ld, _p(_vector(alpha, n, "alpha")), _p(_vector(beta, m, "beta")), float(eta), int(k),
        _p(_vector(delta, 1, "delta")), _p(_vector(s_k, 1, "s_k", optional=True)),
        _p(_vector(info, 2, "info", torch.int64)),
        *_ws(workspace), _stream(stream)), "regot_topk_threshold")


def _entries(t, name, dtype, capacity, optional=False):
    """An entry array of a pattern: 1-D, contiguous, at least `capacity` long."""
    if t is None:
        if optional:
            return None
        raise TypeError(f"{name} is required")
    if t.dtype != dtype or not t.is_cuda or t.dim() != 1 or t.numel() < capacity or (t.numel() > 1 and t.stride(0) != 1):
        raise TypeError(f"{name} must be a contiguous 1-D {dtype} CUDA tensor with at least {capacity} entries")
    return t


def regot_pattern_values(M, alpha, beta, eta, row_ptr, col_idx, csc_pos, val, val_csc, *, stream=None) -> None:
    n, m, ld = _matrix(M)
    capacity = int(col_idx.numel())
    _check(load().regot_pattern_values(
        n, m, _p(M), ld, _p(_vector(alpha, n, "alpha")), _p(_vector(beta, m, "beta")), float(eta),
        _p(_vector(row_ptr, n + 1, "row_ptr", torch.int64)), _p(_entries(col_idx, "col_idx", torch.int32, capacity)),
        _p(_entries(csc_pos, "csc_pos", torch.int64, capacity, optional=True)), capacity,
        _p(_entries(val, "val", torch.float64, capacity)),
        _p(_entries(val_csc, "val_csc", torch.float64, capacity, optional=True)), _stream(stream)),
        "regot_pattern_values")


def regot_pattern_transpose_workspace_bytes(n: int, m: int, nnz: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().regot_pattern_transpose_workspace_bytes(int(n), int(m), int(nnz), ctypes.byref(out)),
           "regot_pattern_transpose_workspace_bytes")
    return int(out.value)


def regot_pattern_transpose(n, m, nnz, row_ptr, col_idx, col_ptr, row_idx, csc_pos, *, workspace, stream=None) -> None:
    nnz = int(nnz)
    _check(load().regot_pattern_transpose(
        int(n), int(m), nnz, _p(_vector(row_ptr, n + 1, "row_ptr", torch.int64)),
        _p(_entries(col_idx, "col_idx", torch.int32, nnz)), _p(_vector(col_ptr, m + 1, "col_ptr", torch.int64)),
        _p(_entries(row_idx, "row_idx", torch.int32, nnz)), _p(_entries(csc_pos, "csc_pos", torch.int64, nnz)),
        *_ws(workspace), _stream(stream)), "regot_pattern_transpose")


def regot_hessian_matvec(n, m, eta, tau, row_ptr, col_idx, val, col_ptr, row_idx, val_csc, row_sum, col_sum, x, y, *,
                         stream=None) -> None:
    capacity = int(col_idx.numel())
    _check(load().regot_hessian_matvec(
        int(n), int(m), float(eta), float(tau), _p(_vector(row_ptr, n + 1, "row_ptr", torch.int64)),
        _p(_entries(col_idx, "col_idx", torch.int32, capacity)), _p(_entries(val, "val", torch.float64, capacity)),
        _p(_vector(col_ptr, m + 1, "col_ptr", torch.int64)), _p(_entries(row_idx, "row_idx", torch.int32, capacity)),
        _p(_entries(val_csc, "val_csc", torch.float64, capacity)), capacity,
        _p(_vector(row_sum, n, "row_sum")), _p(_vector(col_sum, m, "col_sum")),
        _p(_vector(x, n + m - 1, "x")), _p(_vector(y, n + m - 1, "y")), _stream(stream)), "regot_hessian_matvec")


def regot_hessian_workspace_bytes(n: int, m: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().regot_hessian_workspace_bytes(int(n), int(m), ctypes.byref(out)), "regot_hessian_workspace_bytes")
    return int(out.value)


def regot_hessian_lower_csc(n, m, eta, tau, row_ptr, col_idx, val, row_sum, col_sum, h_col_ptr, h_row_idx, h_val, info,
                            values_only=False, *, workspace, stream=None) -> None:
    capacity = int(col_idx.numel())
    h_capacity = int(h_row_idx.numel())
    _check(load().regot_hessian_lower_csc(
        int(n), int(m), float(eta), float(tau), _p(_vector(row_ptr, n + 1, "row_ptr", torch.int64)),
        _p(_entries(col_idx, "col_idx", torch.int32, capacity)), _p(_entries(val, "val", torch.float64, capacity)),
        capacity, _p(_vector(row_sum, n, "row_sum")), _p(_vector(col_sum, m, "col_sum")),
        _p(_vector(h_col_ptr, n + m, "h_col_ptr", torch.int64)),
        _p(_entries(h_row_idx, "h_row_idx", torch.int32, h_capacity)),
        _p(_entries(h_val, "h_val", torch.float64, h_capacity)), h_capacity,
        _p(_vector(info, 2, "info", torch.int64)), 1 if values_only else 0,
        *_ws(workspace), _stream(stream)), "regot_hessian_lower_csc")


def regot_dual_metrics(a, b, alpha, beta, eta, row_sum, col_sum, metrics, *, workspace, stream=None) -> None:
    n, m = int(a.numel()), int(b.numel())
    _check(load().regot_dual_metrics(
        n, m, _p(_vector(a, n, "a")), _p(_vector(b, m, "b")), _p(_vector(alpha, n, "alpha")),
        _p(_vector(beta, m, "beta")), float(eta), _p(_vector(row_sum, n, "row_sum")), _p(_vector(col_sum, m, "col_sum")),
        _p(_vector(metrics, 4, "metrics")), *_ws(workspace),
        _stream(stream)), "regot_dual_metrics")


def regot_choose_candidate(obj_q, obj_s, alpha_q, beta_q, alpha_s, beta_s, alpha_out, beta_out, choice, *,
                           stream=None) -> None:
    n, m = int(alpha_q.numel()), int(beta_q.numel())
    _check(load().regot_choose_candidate(
        n, m, _p(_vector(obj_q, 1, "obj_q")), _p(_vector(obj_s, 1, "obj_s")),
        _p(_vector(alpha_q, n, "alpha_q")), _p(_vector(beta_q, m, "beta_q")),
        _p(_vector(alpha_s, n, "alpha_s")), _p(_vector(beta_s, m, "beta_s")),
        _p(_vector(alpha_out, n, "alpha_out")), _p(_vector(beta_out, m, "beta_out")),
        _p(_vector(choice, 1, "choice", torch.int64)), _stream(stream)), "regot_choose_candidate")


def regot_pcg_workspace_bytes(n: int, m: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().regot_pcg_workspace_bytes(int(n), int(m), ctypes.byref(out)), "regot_pcg_workspace_bytes")
    return int(out.value)


def regot_pcg_solve(n, m, eta, tau, row_ptr, col_idx, val, col_ptr, row_idx, val_csc, row_sum, col_sum, rhs, x, rtol,
                    iterations, restart, info, *, workspace, stream=None) -> None:
    capacity = int(col_idx.numel())
    N = n + m - 1
    _check(load().regot_pcg_solve(
        int(n), int(m), float(eta), float(tau), _p(_vector(row_ptr, n + 1, "row_ptr", torch.int64)),
        _p(_entries(col_idx, "col_idx", torch.int32, capacity)), _p(_entries(val, "val", torch.float64, capacity)),
        _p(_vector(col_ptr, m + 1, "col_ptr", torch.int64)), _p(_entries(row_idx, "row_idx", torch.int32, capacity)),
        _p(_entries(val_csc, "val_csc", torch.float64, capacity)), capacity,
        _p(_vector(row_sum, n, "row_sum")), _p(_vector(col_sum, m, "col_sum")),
        _p(_vector(rhs, N, "rhs")), _p(_vector(x, N, "x")), float(rtol), int(iterations), 1 if restart else 0,
        _p(_vector(info, 4, "info")), *_ws(workspace), _stream(stream)),
        "regot_pcg_solve")


def regot_pcg_solve_reduced(n, m, eta, tau, row_ptr, col_idx, val, col_ptr, row_idx, val_csc, row_sum, col_sum, rhs, x,
                            rtol, iterations, restart, info, *, workspace, stream=None) -> None:
    capacity = int(col_idx.numel())
    N = n + m - 1
    _check(load().regot_pcg_solve_reduced(
        int(n), int(m), float(eta), float(tau), _p(_vector(row_ptr, n + 1, "row_ptr", torch.int64)),
        _p(_entries(col_idx, "col_idx", torch.int32, capacity)), _p(_entries(val, "val", torch.float64, capacity)),
        _p(_vector(col_ptr, m + 1, "col_ptr", torch.int64)), _p(_entries(row_idx, "row_idx", torch.int32, capacity)),
        _p(_entries(val_csc, "val_csc", torch.float64, capacity)), capacity,
        _p(_vector(row_sum, n, "row_sum")), _p(_vector(col_sum, m, "col_sum")),
        _p(_vector(rhs, N, "rhs")), _p(_vector(x, N, "x")), float(rtol), int(iterations), 1 if restart else 0,
        _p(_vector(info, 4, "info")), *_ws(workspace), _stream(stream)),
        "regot_pcg_solve_reduced")


def regot_pcg_solve2(n, m, eta, tau, row_ptr, col_idx, val, col_ptr, row_idx, val_csc, row_sum, col_sum, rhs_a, rhs_b,
                     x_a, x_b, rtol, iterations, restart, info, *, workspace, stream=None) -> None:
    capacity = int(col_idx.numel())
    N = n + m - 1
    _check(load().regot_pcg_solve2(
        int(n), int(m), float(eta), float(tau), _p(_vector(row_ptr, n + 1, "row_ptr", torch.int64)),
        _p(_entries(col_idx, "col_idx", torch.int32, capacity)), _p(_entries(val, "val", torch.float64, capacity)),
        _p(_vector(col_ptr, m + 1, "col_ptr", torch.int64)), _p(_entries(row_idx, "row_idx", torch.int32, capacity)),
        _p(_entries(val_csc, "val_csc", torch.float64, capacity)), capacity,
        _p(_vector(row_sum, n, "row_sum")), _p(_vector(col_sum, m, "col_sum")),
        _p(_vector(rhs_a, N, "rhs_a")), _p(_vector(rhs_b, N, "rhs_b")), _p(_vector(x_a, N, "x_a")),
        _p(_vector(x_b, N, "x_b")), float(rtol), int(iterations), 1 if restart else 0,
        _p(_vector(info, 8, "info")), *_ws(workspace), _stream(stream)),
        "regot_pcg_solve2")


def regot_pcg_solve2_reduced(n, m, eta, tau, row_ptr, col_idx, val, col_ptr, row_idx, val_csc, row_sum, col_sum, rhs_a,
                             rhs_b, x_a, x_b, rtol, iterations, restart, info, *, workspace, stream=None) -> None:
    capacity = int(col_idx.numel())
    N = n + m - 1
    _check(load().regot_pcg_solve2_reduced(
        int(n), int(m), float(eta), float(tau), _p(_vector(row_ptr, n + 1, "row_ptr", torch.int64)),
        _p(_entries(col_idx, "col_idx", torch.int32, capacity)), _p(_entries(val, "val", torch.float64, capacity)),
        _p(_vector(col_ptr, m + 1, "col_ptr", torch.int64)), _p(_entries(row_idx, "row_idx", torch.int32, capacity)),
        _p(_entries(val_csc, "val_csc", torch.float64, capacity)), capacity,
        _p(_vector(row_sum, n, "row_sum")), _p(_vector(col_sum, m, "col_sum")),
        _p(_vector(rhs_a, N, "rhs_a")), _p(_vector(rhs_b, N, "rhs_b")), _p(_vector(x_a, N, "x_a")),
        _p(_vector(x_b, N, "x_b")), float(rtol), int(iterations), 1 if restart else 0,
        _p(_vector(info, 8, "info")), *_ws(workspace), _stream(stream)),
        "regot_pcg_solve2_reduced")


def regot_splr_direction(n, m, p, q, s_prev, y_prev, v, d, info, *, workspace, stream=None) -> None:
    N = n + m - 1
    _check(load().regot_splr_direction(
        int(n), int(m), _p(_vector(p, N, "p")), _p(_vector(q, N, "q", optional=True)),
        _p(_vector(s_prev, N, "s_prev", optional=True)), _p(_vector(y_prev, N, "y_prev", optional=True)),
        _p(_vector(v, N, "v", optional=True)), _p(_vector(d, N, "d")), _p(_vector(info, 2, "info")),
        *_ws(workspace), _stream(stream)), "regot_splr_direction")


def regot_profile_stage1(start_event, stop_event) -> None:
    """start_event / stop_event: raw hipEvent_t handles (ints) or None; see include/regot.h."""
    _check(load().regot_profile_stage1(ctypes.c_void_p(start_event) if start_event else None,
                                       ctypes.c_void_p(stop_event) if stop_event else None),
           "regot_profile_stage1")


def regot_stream_read_probe(M, total, *, workspace, stream=None) -> None:
    """total[0] = sum of all entries of M, by a pass with the tiling of the dense calls (a bandwidth probe)."""
    n, m, ld = _matrix(M)
    _check(load().regot_stream_read_probe(n, m, _p(M), ld, _p(_vector(total, 1, "total")), *_ws(workspace), _stream(stream)),
           "regot_stream_read_probe")


def regot_placement_probe(ids, *, stream=None) -> None:
    """ids: int32 CUDA tensor [2 * grid]: hardware-id and die-id registers of every workgroup of a grid launched like the fused pass."""
    if ids.dtype != torch.int32 or not ids.is_cuda or ids.dim() != 1 or ids.numel() % 2 or not ids.is_contiguous():
        raise TypeError("ids must be a contiguous 1-D int32 CUDA tensor of even length")
    _check(load().regot_placement_probe(ids.numel() // 2, _p(ids), _stream(stream)), "regot_placement_probe")
