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
        self.stats = torch.zeros(2 * self.M + 3, device=dev)
        self.avg_norm = torch.zeros(1, device=dev)
        self.push_used = self.push
        self._params = None                                # set by from_modules

    @classmethod
    def from_modules(cls, modules: Sequence, **kwargs) -> "DppfLoop":
        """M replicas of one torch.nn.Module on the same GPU (identical parameter lists).  The
        parameters are updated in place; gradients are read from ``p.grad`` after the caller's
        backward passes, wherever autograd put them (the gradient pointer table is rebuilt every
        iteration); momentum buffers are created here."""
        import torch
        params = [[p for p in mod.parameters() if p.requires_grad] for mod in modules]
        shapes = [tuple(p.shape) for p in params[0]]
        for row in params:
            if [tuple(p.shape) for p in row] != shapes:
                raise ValueError("the replicas must have identical parameter lists")
            for p in row:
                if not p.is_contiguous() or p.dtype != torch.float32:
                    raise ValueError("parameters must be contiguous float32 tensors")
        x = [[p.data for p in row] for row in params]
        v = [[torch.zeros_like(p.data) for p in row] for row in params]
        g = [[torch.zeros_like(p.data) for p in row] for row in params]     # placeholders until backward ran
        loop = cls(x, v, g, **kwargs)
        loop._params = params
        return loop

    def _gradients_from_autograd(self) -> None:
        rows = []
        for row in self._params:
            for p in row:
                if p.grad is None or not p.grad.is_contiguous():
                    raise ValueError("every parameter needs a contiguous .grad before step()")
            rows.append([p.grad for p in row])
        self.g = rows
        self.gt = dppf.PointerTable(rows)

    def step(self, grad_fn: Callable[[int], None], lr: Optional[float] = None) -> bool:
        """One iteration of Alg. 1 for all workers.  Returns True if it ended with a round."""
        grad_fn(self.t)
        if self._params is not None:
            self._gradients_from_autograd()
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
        """(relaxed MV, pull strengths alpha*r_m, push strength, ||x_A||) of the latest round, as the
        appendix's ablations log them.  Synchronises."""
        self.plan.average_norm(self.avg_norm)
        dppf.round_statistics(self.r, self.M, self.pull, self.push_used, self.stats, avg_norm=self.avg_norm)
        out = self.stats.cpu().numpy()
        return float(out[0]), out[1:self.M + 1].copy(), float(out[self.M + 1]), float(out[2 * self.M + 1])

    def average(self, out: List) -> None:
        """x_A, the value Alg. 1 returns, into the T tensors of `out`."""
        self.plan.replica_mean(self.xt, out)

    def close(self) -> None:
        self.plan.close()
