"""Outer loop of marginal-likelihood optimisation (paper Section 2.1 hierarchy, Section 4 and
Appendix B settings): Adam on softplus-constrained hyperparameters, each step one batched
linear solve (conjugate gradients or alternating projections, warm-started or cold) followed by
the stochastic gradient.

Host-side glue only: theta lives in a handful of fp64 scalars, every n-sized array stays on the
device and every n-sized operation is a libgpws call.
"""
from __future__ import annotations

import time
from dataclasses import dataclass, field

import numpy as np
import torch

from . import binding as gp

KIND_CODE = {"se": gp.GP_SE_ARD, "matern32": gp.GP_MATERN32_ARD}


def softplus(raw):
    return np.logaddexp(0.0, raw)


def softplus_inverse(theta):
    theta = np.asarray(theta, dtype=np.float64)
    return theta + np.log(-np.expm1(-theta))


class AdamState:
    """Bias-corrected Adam ascent on raw = softplus^{-1}(theta) (Section 4, Appendix B); host scalars only."""

    def __init__(self, theta0, lr=0.1, b1=0.9, b2=0.999, eps=1e-8):
        self.raw = softplus_inverse(theta0)
        self.m = np.zeros_like(self.raw)
        self.v = np.zeros_like(self.raw)
        self.k = 0
        self.lr, self.b1, self.b2, self.eps = lr, b1, b2, eps

    @property
    def theta(self):
        return softplus(self.raw)

    def ascend(self, grad_theta):
        """One step given dL/dtheta at the current theta (chain rule through the softplus applied here)."""
        theta = self.theta
        graw = np.asarray(grad_theta, dtype=np.float64) * (-np.expm1(-theta))
        self.k += 1
        self.m = self.b1 * self.m + (1 - self.b1) * graw
        self.v = self.b2 * self.v + (1 - self.b2) * graw * graw
        mhat = self.m / (1 - self.b1 ** self.k)
        vhat = self.v / (1 - self.b2 ** self.k)
        self.raw = self.raw + self.lr * mhat / (np.sqrt(vhat) + self.eps)
        return self.theta


@dataclass
class StepRecord:
    theta: np.ndarray
    iters: int
    kmv_count: int
    rc: int
    solve_ms: float
    grad_ms: float
    step_ms: float
    max_relres: float
    grad: np.ndarray = field(repr=False, default=None)
    relres: np.ndarray = field(repr=False, default=None)    # final relative residual of every column


class MllOptimizer:
    """Adam ascent on L(theta) with the linear solves done by gp_cg_solve (solver="cg"),
    gp_ap_solve (solver="ap", blocks of `block` indices; iters then counts block updates) or
    gp_sgd_solve (solver="sgd", mini-batches of `batch` distinct rows drawn once, seeded, and reused
    by every solve; iters counts steps, at most max_iters and at most 4096).

    warm=True keeps the probes Z fixed and passes the previous step's V as x0 (Section 3);
    warm=False starts every solve from zero and, if resample is given, redraws the probes
    each step (the conventional procedure the paper compares against).
    """

    def __init__(self, X, y, Z, kind, ell0, a0, sigma0, tol, warm=True, lr=0.1, max_iters=1000,
                 resample=None, device="cuda:0", solver="cg", block=2000, batch=1000,
                 sgd_lr=50.0, sgd_momentum=0.9, seed=1234):
        self.dev = torch.device(device)
        self.X = torch.as_tensor(np.ascontiguousarray(X, dtype=np.float32)).to(self.dev)
        self.n, self.d = self.X.shape
        B = np.concatenate([np.asarray(y, dtype=np.float32)[:, None], np.asarray(Z, dtype=np.float32)], axis=1)
        self.B = torch.as_tensor(np.ascontiguousarray(B)).to(self.dev)
        self.t = self.B.shape[1]
        self.V = torch.zeros_like(self.B)
        self.warm = warm
        self.resample = resample
        self.tol = tol
        self.max_iters = max_iters
        self.adam = AdamState(np.concatenate([np.asarray(ell0, dtype=np.float64), [a0, sigma0]]), lr=lr)
        self.have_solution = False
        self.stream = torch.cuda.current_stream(self.dev)
        self.ctx = gp.gp_create(KIND_CODE[kind], self.n, self.d, self.X, self.stream.cuda_stream)
        if solver not in ("cg", "ap", "sgd"):
            raise ValueError(f"unknown solver {solver!r}")
        self.solver = solver
        self.block = int(block)
        self.batch = min(int(batch), self.n)
        self.sgd_lr, self.sgd_momentum = float(sgd_lr), float(sgd_momentum)
        if solver == "sgd":
            # the library draws no random numbers: the mini-batch index sequences are made here
            self.max_iters = min(self.max_iters, 4096)
            gen = torch.Generator(device=self.dev)
            gen.manual_seed(seed)
            self.batches = torch.stack([torch.randperm(self.n, generator=gen, device=self.dev)[: self.batch]
                                        for _ in range(self.max_iters)]).to(torch.int32).contiguous()
        need = (gp.gp_workspace_bytes(self.ctx, self.t) if solver == "cg"
                else gp.gp_ap_workspace_bytes(self.ctx, self.t, self.block) if solver == "ap"
                else gp.gp_sgd_workspace_bytes(self.ctx, self.t, self.batch))
        if need == 0:
            raise ValueError("workspace size query failed (t or block out of range)")
        self.work = torch.empty(need, dtype=torch.uint8, device=self.dev)
        self.history = []

    @property
    def theta(self):
        return self.adam.theta

    @property
    def k(self):
        return self.adam.k

    def close(self):
        if self.ctx is not None:
            gp.gp_destroy(self.ctx)
            self.ctx = None

    def step(self):
        t0 = time.perf_counter()
        theta = self.theta
        ell, a, sigma = theta[: self.d], theta[self.d], theta[self.d + 1]
        gp.gp_set_theta(self.ctx, ell, a, sigma)
        if not self.warm and self.resample is not None:
            self.B[:, 1:] = self.resample(self.k)
        x0 = self.V if (self.warm and self.have_solution) else None
        t1 = time.perf_counter()
        if self.solver == "cg":
            rc, iters, kmv, relres = gp.gp_cg_solve(self.ctx, self.B, self.t, x0, self.V, self.t, self.t, self.tol,
                                                    self.max_iters, self.work, self.work.numel())
        elif self.solver == "ap":
            rc, iters, kmv, relres, _ = gp.gp_ap_solve(self.ctx, self.B, self.t, x0, self.V, self.t, self.t, self.tol,
                                                       self.block, self.max_iters, self.work, self.work.numel())
        else:
            rc, iters, kmv, relres = gp.gp_sgd_solve(self.ctx, self.B, self.t, x0, self.V, self.t, self.t, self.tol,
                                                     self.batches, self.batch, self.max_iters, self.sgd_lr,
                                                     self.sgd_momentum, self.work, self.work.numel())
        t2 = time.perf_counter()
        g = gp.gp_mll_grad(self.ctx, self.V, self.t, self.B, self.t, self.t, self.d)
        t3 = time.perf_counter()
        self.have_solution = True
        self.adam.ascend(g)
        t4 = time.perf_counter()
        rec = StepRecord(theta, iters, kmv, rc, (t2 - t1) * 1e3, (t3 - t2) * 1e3, (t4 - t0) * 1e3,
                         float(relres.max()), g, np.array(relres, dtype=np.float64))
        self.history.append(rec)
        return rec
