"""Host-side driver: owns the buffers of one problem size and issues library calls.

It runs fixed numbers of Sinkhorn sweeps (alpha half-step, then beta half-step, as a
candidate generator does in Sec. 4.3) and objective / gradient / pattern evaluations
(Algorithm 1, lines 1-2).  No arithmetic happens here: every method is a sequence of
calls into libregot.so on the current stream.
"""
import torch

from . import binding as B


class DualPass:
    """Buffers and calls for an n x m problem; `capacity` = CSR entries to reserve (-1: no sparsify)."""

    def __init__(self, n: int, m: int, capacity: int = -1, device="cuda"):
        self.n, self.m, self.capacity = int(n), int(m), int(capacity)
        dev = torch.device(device)
        f64 = dict(dtype=torch.float64, device=dev)
        self.workspace = B.new_workspace(n, m, capacity, dev)
        self.obj = torch.zeros(1, **f64)
        self.grad_alpha = torch.zeros(n, **f64)
        self.grad_beta = torch.zeros(m, **f64)
        self.row_sum = torch.zeros(n, **f64)
        self.col_sum = torch.zeros(m, **f64)
        if capacity >= 0:
            self.row_ptr = torch.zeros(n + 1, dtype=torch.int64, device=dev)
            self.col_idx = torch.zeros(capacity, dtype=torch.int32, device=dev)
            self.val = torch.zeros(capacity, **f64)
            self.info = torch.zeros(2, dtype=torch.int64, device=dev)

    def dual_eval(self, M, a, b, alpha, beta, eta):
        B.regot_dual_eval(M, a, b, alpha, beta, eta, self.obj, self.grad_alpha, self.grad_beta,
                          self.row_sum, self.col_sum, workspace=self.workspace)

    def sparsify_csr(self, M, alpha, beta, eta, delta):
        B.regot_sparsify_csr(M, alpha, beta, eta, delta, self.row_ptr, self.col_idx, self.val, self.info,
                             workspace=self.workspace)

    def dual_eval_sparsify(self, M, a, b, alpha, beta, eta, delta):
        B.regot_dual_eval_sparsify(M, a, b, alpha, beta, eta, self.obj, self.grad_alpha, self.grad_beta,
                                   self.row_sum, self.col_sum, delta, self.row_ptr, self.col_idx, self.val,
                                   self.info, workspace=self.workspace)

    def metrics(self, a, b, alpha, beta, eta):
        """Primal value, duality gap, marginal error and gradient norm at the point of the last evaluation
        (its row / column sums); result on the device in .metric_out."""
        if not hasattr(self, "metric_out"):
            self.metric_out = torch.zeros(4, dtype=torch.float64, device=self.row_sum.device)
        B.regot_dual_metrics(a, b, alpha, beta, eta, self.row_sum, self.col_sum, self.metric_out,
                             workspace=self.workspace)
        return self.metric_out

    def half_step(self, M, marginal, alpha, beta, eta, which, out):
        B.regot_sinkhorn_half_step(M, marginal, alpha, beta, eta, which, out, workspace=self.workspace)

    def sinkhorn_sweeps(self, M, a, b, eta, sweeps, alpha=None, beta=None):
        """`sweeps` x (alpha half-step, beta half-step), in place; starts from zero unless duals are given."""
        f64 = dict(dtype=torch.float64, device=M.device)
        alpha = torch.zeros(self.n, **f64) if alpha is None else alpha
        beta = torch.zeros(self.m, **f64) if beta is None else beta
        B.regot_sinkhorn_sweeps(M, a, b, alpha, beta, eta, int(sweeps), workspace=self.workspace)
        return alpha, beta

    def csr_host(self):
        """(row_ptr, col_idx, val, overflow) copied to numpy; synchronises."""
        info = self.info.cpu()
        nnz, overflow = int(info[0]), int(info[1])
        k = min(nnz, self.capacity)
        return (self.row_ptr.cpu().numpy(), self.col_idx[:k].cpu().numpy(), self.val[:k].cpu().numpy(), overflow)


class PatternRefresh(DualPass):
    """The fused evaluation that finds the top-k threshold itself: one read of M instead of the two of
    `TopK.threshold` followed by `DualPass.dual_eval_sparsify` (Sec. 3.1 top-k rule + Sec. 4.4).

    Buffers as in DualPass (`capacity` entries for the CSR, by default k plus room for ties); .delta holds
    the threshold, .info[1] bit 1 says that the caller has to make the two calls instead."""

    def __init__(self, n: int, m: int, k: int, capacity: int = -1, device="cuda"):
        capacity = int(k) + 4096 if capacity < 0 else int(capacity)
        super().__init__(n, m, capacity, device)
        self.k = int(k)
        dev = torch.device(device)
        self.workspace = B.new_workspace(n, m, B.regot_refresh_candidate_capacity(n, m, k), dev)
        self.topk_workspace = B.new_topk_workspace(n, m, k, dev)
        self.delta = torch.zeros(1, dtype=torch.float64, device=dev)

    def refresh(self, M, a, b, alpha, beta, eta):
        B.regot_dual_eval_sparsify_topk(M, a, b, alpha, beta, eta, self.k, self.obj, self.grad_alpha, self.grad_beta,
                                        self.row_sum, self.col_sum, self.delta, self.row_ptr, self.col_idx, self.val,
                                        self.info, workspace=self.workspace, topk_workspace=self.topk_workspace)


class TopK:
    """Buffers and the call for the top-k threshold of an n x m problem (Sec. 3.1)."""

    def __init__(self, n: int, m: int, k: int, device="cuda"):
        self.n, self.m, self.k = int(n), int(m), int(k)
        dev = torch.device(device)
        self.workspace = B.new_topk_workspace(n, m, k, dev)
        self.delta = torch.zeros(1, dtype=torch.float64, device=dev)
        self.s_k = torch.zeros(1, dtype=torch.float64, device=dev)
        self.info = torch.zeros(2, dtype=torch.int64, device=dev)

    def threshold(self, M, alpha, beta, eta):
        """Enqueue the search; results stay on the device in .delta, .s_k, .info."""
        B.regot_topk_threshold(M, alpha, beta, eta, self.k, self.delta, self.s_k, self.info,
                               workspace=self.workspace)

    def result_host(self):
        """(delta, s_k, above, equal) as Python numbers; synchronises."""
        info = self.info.cpu()
        return float(self.delta.cpu()[0]), float(self.s_k.cpu()[0]), int(info[0]), int(info[1])


class SparseTerm:
    """The sparse term H_Omega of the quasi-Newton matrix on a stored pattern (Sec. 3.1, eq. (7)).

    Built once per pattern from the CSR structure a sparsify call left on the device (the symbolic
    step: the pattern by columns); `refresh` then recomputes the values at the current dual point
    (Sec. 4.2), `matvec` applies H_Omega + tau I and `lower_csc` writes its lower triangle by columns.
    """

    def __init__(self, n: int, m: int, row_ptr, col_idx, nnz: int):
        self.n, self.m, self.nnz = int(n), int(m), int(nnz)
        dev = row_ptr.device
        e = max(self.nnz, 1)
        # the stored pattern is a copy: the buffers of the sparsify call are free to take the next pattern
        self.row_ptr = row_ptr.clone()
        self.col_idx = col_idx[:e].clone() if col_idx.numel() >= e else torch.zeros(e, dtype=torch.int32, device=dev)
        self.col_ptr = torch.zeros(m + 1, dtype=torch.int64, device=dev)
        self.row_idx = torch.zeros(e, dtype=torch.int32, device=dev)
        self.csc_pos = torch.zeros(e, dtype=torch.int64, device=dev)
        self.val = torch.zeros(e, dtype=torch.float64, device=dev)
        self.val_csc = torch.zeros(e, dtype=torch.float64, device=dev)
        ws = torch.empty(max(B.regot_pattern_transpose_workspace_bytes(n, m, self.nnz), 256), dtype=torch.uint8, device=dev)
        B.regot_pattern_transpose(n, m, self.nnz, self.row_ptr, self.col_idx, self.col_ptr, self.row_idx, self.csc_pos,
                                  workspace=ws)
        self.h_capacity = n + m - 1 + self.nnz
        self.h_col_ptr = torch.zeros(n + m, dtype=torch.int64, device=dev)
        self.h_row_idx = torch.zeros(self.h_capacity, dtype=torch.int32, device=dev)
        self.h_val = torch.zeros(self.h_capacity, dtype=torch.float64, device=dev)
        self.h_info = torch.zeros(2, dtype=torch.int64, device=dev)
        self.h_workspace = torch.empty(max(B.regot_hessian_workspace_bytes(n, m), 256), dtype=torch.uint8, device=dev)
        self._structure_done = False

    def refresh(self, M, alpha, beta, eta):
        B.regot_pattern_values(M, alpha, beta, eta, self.row_ptr, self.col_idx, self.csc_pos, self.val, self.val_csc)

    def matvec(self, eta, tau, row_sum, col_sum, x, y):
        B.regot_hessian_matvec(self.n, self.m, eta, tau, self.row_ptr, self.col_idx, self.val, self.col_ptr,
                               self.row_idx, self.val_csc, row_sum, col_sum, x, y)

    def lower_csc(self, eta, tau, row_sum, col_sum):
        """Structure and values on the first call, values alone afterwards."""
        B.regot_hessian_lower_csc(self.n, self.m, eta, tau, self.row_ptr, self.col_idx, self.val, row_sum, col_sum,
                                  self.h_col_ptr, self.h_row_idx, self.h_val, self.h_info,
                                  values_only=self._structure_done, workspace=self.h_workspace)
        self._structure_done = True


class CandidateGenerator:
    """Candidate iterates on a side stream (Sec. 4.3).

    `launch` starts, on a stream of its own, a few Sinkhorn sweeps from a copy of the current duals and an
    evaluation of the result, and returns at once: the host goes on with its serial work (the symbolic
    analysis in the paper) and the main stream with the quasi-Newton step.  `select` then evaluates the
    quasi-Newton candidate on the main stream, waits (on the device) for the side stream, and keeps the
    candidate with the larger dual objective.  Nothing here waits on the host.  The side stream has its
    own buffers and workspace, and the default priority.
    """

    def __init__(self, n: int, m: int, device="cuda"):
        dev = torch.device(device)
        self.n, self.m = int(n), int(m)
        self.stream = torch.cuda.Stream(device=dev)
        self.side = DualPass(n, m, device=dev)
        self.alpha_s = torch.zeros(n, dtype=torch.float64, device=dev)
        self.beta_s = torch.zeros(m, dtype=torch.float64, device=dev)
        self.choice = torch.zeros(1, dtype=torch.int64, device=dev)
        self.ready = torch.cuda.Event()
        self.done = torch.cuda.Event()

    def launch(self, M, a, b, alpha, beta, eta, sweeps: int):
        main = torch.cuda.current_stream()
        self.ready.record(main)                 # the duals as they are now on the main stream
        with torch.cuda.stream(self.stream):
            self.stream.wait_event(self.ready)
            self.alpha_s.copy_(alpha)
            self.beta_s.copy_(beta)
            self.side.sinkhorn_sweeps(M, a, b, eta, sweeps, self.alpha_s, self.beta_s)
            self.side.dual_eval(M, a, b, self.alpha_s, self.beta_s, eta)
            self.done.record(self.stream)

    def select(self, main_pass: "DualPass", M, a, b, eta, alpha_q, beta_q, alpha_out, beta_out):
        """Enqueue on the current stream: L at the quasi-Newton candidate (in main_pass), then the choice."""
        main_pass.dual_eval(M, a, b, alpha_q, beta_q, eta)
        torch.cuda.current_stream().wait_event(self.done)
        B.regot_choose_candidate(main_pass.obj, self.side.obj, alpha_q, beta_q, self.alpha_s, self.beta_s,
                                 alpha_out, beta_out, self.choice)
        return self.choice


class DirectionSolver:
    """The quasi-Newton direction d = -B^{-1} g (Algorithm 1, lines 3-7) by conjugate gradients on the sparse term.

    The iterations are enqueued in portions; between portions the host reads one flag to see whether the
    solve has converged (the only host synchronisation, and only in this driver: the library calls are
    asynchronous)."""

    def __init__(self, term: SparseTerm):
        self.term = term
        n, m = term.n, term.m
        dev = term.row_ptr.device
        N = n + m - 1
        f64 = dict(dtype=torch.float64, device=dev)
        self.workspace = torch.empty(max(B.regot_pcg_workspace_bytes(n, m), 256), dtype=torch.uint8, device=dev)
        self.p = torch.zeros(N, **f64)
        self.q = torch.zeros(N, **f64)
        self.v = torch.zeros(N, **f64)
        self.d = torch.zeros(N, **f64)
        self.solve_info = torch.zeros(4, **f64)
        self.solve2_info = torch.zeros(8, **f64)
        self.info = torch.zeros(2, **f64)

    def solve(self, eta, tau, row_sum, col_sum, rhs, x, rtol=1e-8, max_iter=1000, portion=24, reduced=False):
        """x = (H_Omega + tau I)^{-1} rhs; returns (iterations, converged, relative residual).
        reduced: iterate on the Schur complement of the first block (regot_pcg_solve_reduced)."""
        t = self.term
        call = B.regot_pcg_solve_reduced if reduced else B.regot_pcg_solve
        done, restart = 0, True
        while True:
            its = min(portion, max_iter - done)
            call(t.n, t.m, eta, tau, t.row_ptr, t.col_idx, t.val, t.col_ptr, t.row_idx, t.val_csc,
                 row_sum, col_sum, rhs, x, rtol, its, restart, self.solve_info, workspace=self.workspace)
            restart = False
            done += its
            info = self.solve_info.cpu()
            if info[1] != 0 or done >= max_iter:
                rel = float(info[2] / info[3]) if info[3] > 0 else 0.0
                return int(info[0]), bool(info[1] != 0), rel

    def solve2(self, eta, tau, row_sum, col_sum, rhs_a, rhs_b, x_a, x_b, rtol=1e-8, max_iter=1000, portion=24,
               reduced=False):
        """Two systems with the same matrix in one iteration (the pattern is read once for both); each stops
        on its own.  Returns ((iterations, converged, relative residual) of a, the same of b)."""
        t = self.term
        call = B.regot_pcg_solve2_reduced if reduced else B.regot_pcg_solve2
        done, restart = 0, True
        while True:
            its = min(portion, max_iter - done)
            call(t.n, t.m, eta, tau, t.row_ptr, t.col_idx, t.val, t.col_ptr, t.row_idx, t.val_csc,
                 row_sum, col_sum, rhs_a, rhs_b, x_a, x_b, rtol, its, restart, self.solve2_info,
                 workspace=self.workspace)
            restart = False
            done += its
            info = self.solve2_info.cpu()
            if (info[1] != 0 and info[5] != 0) or done >= max_iter:
                out = []
                for k in (0, 4):
                    rel = float(info[k + 2] / info[k + 3]) if info[k + 3] > 0 else 0.0
                    out.append((int(info[k]), bool(info[k + 1] != 0), rel))
                return tuple(out)

    def direction(self, eta, tau, row_sum, col_sum, g, s_prev=None, y_prev=None, rtol=1e-8, max_iter=1000, reduced=True):
        """Result in .d; .info = (rank-two term used, (y^-)^T s^-).  Returns the iteration counts of the solves.
        reduced: the solves iterate on the Schur complement of the first block (half the iterations)."""
        t = self.term
        if s_prev is None or y_prev is None:
            it_p = self.solve(eta, tau, row_sum, col_sum, g, self.p, rtol, max_iter, portion=16 if reduced else 24,
                              reduced=reduced)
            B.regot_splr_direction(t.n, t.m, self.p, None, None, None, None, self.d, self.info, workspace=self.workspace)
            return it_p, None
        t.matvec(eta, tau, row_sum, col_sum, s_prev, self.v)
        it_p, it_q = self.solve2(eta, tau, row_sum, col_sum, g, y_prev, self.p, self.q, rtol, max_iter,
                                 portion=16 if reduced else 24, reduced=reduced)
        B.regot_splr_direction(t.n, t.m, self.p, self.q, s_prev, y_prev, self.v, self.d, self.info,
                               workspace=self.workspace)
        return it_p, it_q
