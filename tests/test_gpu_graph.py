"""The library only enqueues kernels on the caller's stream (no allocation, no host synchronisation,
no memset nodes), so a sequence of calls can be captured into a HIP graph and replayed.  Every replay
is checked against the eager result, with eager work and synchronisations in between."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_08793_amd import workloads as W
from paper_2605_08793_amd.driver import DualPass, TopK

pytestmark = pytest.mark.gpu


def test_captured_step_replays_like_eager():
    p = W.make_problem("c2", device="cuda", n=1201, m=999)
    M, a, b = p.host()
    eta = p.eta
    alpha0, beta0 = oracle.sinkhorn_sweeps(M, a, b, eta, 2)
    k = p.k_keep()
    delta = oracle.topk_threshold(M, alpha0, beta0, eta, k) * (1 - 1e-7)
    alpha = torch.from_numpy(alpha0).cuda(); beta = torch.from_numpy(beta0).cuda()
    dp = DualPass(p.n, p.m, capacity=3 * k)
    tk = TopK(p.n, p.m, k)
    new_alpha = torch.empty_like(alpha); new_beta = torch.empty_like(beta)

    def step():
        tk.threshold(p.M, alpha, beta, eta)
        dp.dual_eval_sparsify(p.M, p.a, p.b, alpha, beta, eta, delta)
        dp.half_step(p.M, p.a, alpha, beta, eta, 0, new_alpha)
        dp.half_step(p.M, p.b, new_alpha, beta, eta, 1, new_beta)

    def snapshot():
        torch.cuda.synchronize()
        nnz = int(dp.info.cpu()[0])
        return dict(obj=dp.obj.clone(), ga=dp.grad_alpha.clone(), gb=dp.grad_beta.clone(), rp=dp.row_ptr.clone(),
                    ci=dp.col_idx[:nnz].clone(), val=dp.val[:nnz].clone(), na=new_alpha.clone(), nb=new_beta.clone(),
                    delta=tk.delta.clone(), info=tk.info.clone())

    step()                                      # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    rng = np.random.default_rng(0)
    for replay in range(4):
        # move the dual point (the graph reads the same buffers), compute eagerly, then replay
        alpha.copy_(torch.from_numpy(alpha0 + 0.05 * eta * replay * rng.standard_normal(p.n)).cuda())
        beta.copy_(torch.from_numpy(beta0 + 0.05 * eta * replay * rng.standard_normal(p.m)).cuda())
        step()
        eager = snapshot()
        for t in (dp.obj, dp.grad_alpha, dp.grad_beta, dp.val, new_alpha, new_beta, tk.delta):
            t.fill_(float("nan"))
        dp.row_ptr.fill_(-1); dp.col_idx.fill_(-1); tk.info.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        replayed = snapshot()
        for key in eager:
            assert torch.equal(eager[key], replayed[key]), (replay, key)
    ref = oracle.dual_eval(M, a, b, alpha.cpu().numpy(), beta.cpu().numpy(), eta)
    assert abs(float(dp.obj.cpu()[0]) - ref["obj"]) <= 1e-10 * max(abs(ref["obj"]), eta)
