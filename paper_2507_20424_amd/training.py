"""The loop of Alg. 1 ("Data Parallel Training") over M replicas resident on one GPU.

Orchestration only: which library call happens at which iteration.  Every update of the
parameters is done by the HIP kernels behind `paper_2507_20424_amd.dppf`; gradients come from
the caller (a callback that fills the gradient tensors in place).
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

from . import dppf


class DppfLoop:
    """M workers, each a list of T tensors (parameters x, momentum v, gradients g).

    Every iteration the caller's `grad_fn(t)` must leave worker m's gradient of tensor j in
    ``g[m][j]``.  Iterations whose count is a multiple of `tau` end with a consensus round
    (Alg. 1: the branch ``t mod tau = 0``), done as ONE fused call (last local step + pull-push
    update, Sec. 5 Eq. 5); the others are plain local steps.  `schedule` is one of "fixed",
    "decreasing", "increasing" (appendix, "How to Schedule The Pushing Force?") and needs
    `total_iterations`."""

    def __init__(self, x: Sequence[Sequence], v: Sequence[Sequence], g: Sequence[Sequence], *, tau: int, pull: float,
                 push: float, lr: float, momentum: float = 0.9, weight_decay: float = 0.0,
                 schedule: str = "fixed", total_iterations: Optional[int] = None):
        import torch
        if tau < 1:
            raise ValueError("tau must be >= 1")
        if schedule != "fixed" and not total_iterations:
            raise ValueError("a push schedule needs total_iterations")
        self.M, self.T = len(x), len(x[0])
        self.x, self.v, self.g = x, v, g
        self.plan = dppf.Plan(self.M, [int(t.numel()) for t in x[0]])
        self.xt, self.vt, self.gt = dppf.PointerTable(x), dppf.PointerTable(v), dppf.PointerTable(g)
        self.tau, self.pull, self.push = int(tau), float(pull), float(push)
        self.lr, self.momentum, self.weight_decay = float(lr), float(momentum), float(weight_decay)
        self.schedule, self.total = schedule, total_iterations
        self.t = 0
        dev = x[0][0].device
        self.r = torch.zeros(self.M, device=dev)          # distances measured by the latest round
        self.c = torch.zeros(self.M, device=dev)          # coefficients alpha - lambda/r of that round
        self.stats = torch.zeros(2 * self.M + 1, device=dev)
        self.push_used = self.push

    def step(self, grad_fn: Callable[[int], None], lr: Optional[float] = None) -> bool:
        """One iteration of Alg. 1 for all workers.  Returns True if it ended with a round."""
        grad_fn(self.t)
        eta = self.lr if lr is None else float(lr)
        self.t += 1
        if self.t % self.tau != 0:
            self.plan.local_sgd_step(self.xt, self.vt, self.gt, eta, self.momentum, self.weight_decay)
            return False
        self.push_used = dppf.push_schedule(self.schedule, self.push, self.t, self.total or 1)
        self.plan.round(self.xt, self.vt, self.gt, eta, self.momentum, self.weight_decay, self.pull, self.push_used,
                        r_out=self.r, c_out=self.c)
        return True

    def round_statistics(self):
        """(relaxed MV, pull strengths alpha*r_m, push strength) of the latest round, as the
        appendix's ablation logs them.  Synchronises."""
        dppf.round_statistics(self.r, self.M, self.pull, self.push_used, self.stats)
        out = self.stats.cpu().numpy()
        return float(out[0]), out[1:self.M + 1].copy(), float(out[self.M + 1])

    def average(self, out: List) -> None:
        """x_A, the value Alg. 1 returns, into the T tensors of `out`."""
        self.plan.replica_mean(self.xt, out)

    def close(self) -> None:
        self.plan.close()
