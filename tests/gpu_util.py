"""Helpers for the GPU parity tests: device buffers via torch, calls via the C ABI binding."""
import numpy as np
import torch

KIND_CODE = {"se": 0, "matern32": 1}


class Dev:
    """One libgpws context plus the device copies of a workload's arrays."""

    def __init__(self, X, kind, ell, a, sigma):
        from paper_2405_18328_amd import binding as gp
        self.gp = gp
        self.dev = torch.device("cuda:0")
        self.X = torch.from_numpy(np.ascontiguousarray(X, dtype=np.float32)).to(self.dev)
        self.n, self.d = self.X.shape
        self.ctx = gp.gp_create(KIND_CODE[kind], self.n, self.d, self.X, torch.cuda.current_stream().cuda_stream)
        self.set_theta(ell, a, sigma)
        self._work = None
        self._apwork = None

    def set_theta(self, ell, a, sigma):
        self.gp.gp_set_theta(self.ctx, ell, a, sigma)

    def to(self, arr):
        return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).to(self.dev)

    def kmv(self, V, add_noise, ldv=None, ldo=None):
        n, t = V.shape
        ldv = ldv or t
        ldo = ldo or t
        Vd = torch.full((n, ldv), float("nan"), device=self.dev)
        Vd[:, :t] = self.to(V)
        out = torch.full((n, ldo), -777.0, device=self.dev)
        self.gp.gp_kmv(self.ctx, Vd, ldv, t, out, ldo, add_noise)
        torch.cuda.synchronize()
        o = out.cpu().numpy().astype(np.float64)
        if ldo > t:
            assert (o[:, t:] == -777.0).all(), "padding columns of the output were written"
        return o[:, :t]

    def predict(self, Xstar, V, ldo=None):
        m, t = Xstar.shape[0], V.shape[1]
        ldo = ldo or t
        Xd = torch.from_numpy(np.ascontiguousarray(Xstar, dtype=np.float32)).to(self.dev)
        Vd = self.to(V)
        out = torch.full((m, ldo), -777.0, device=self.dev)
        self.gp.gp_predict(self.ctx, Xd, m, Vd, t, t, out, ldo)
        torch.cuda.synchronize()
        o = out.cpu().numpy().astype(np.float64)
        if ldo > t:
            assert (o[:, t:] == -777.0).all(), "padding columns of the output were written"
        return o[:, :t]

    def work(self, t):
        need = self.gp.gp_workspace_bytes(self.ctx, t)
        if self._work is None or self._work.numel() < need:
            self._work = torch.empty(need, dtype=torch.uint8, device=self.dev)
        return self._work

    def solve(self, B, tol, max_iters=2000, X0=None, Vd=None):
        """Returns (rc, iters, kmv_count, relres, V device tensor)."""
        n, t = B.shape
        Bd = B if isinstance(B, torch.Tensor) else self.to(B)
        if Vd is None:
            Vd = torch.zeros((n, t), device=self.dev)
        w = self.work(t)
        rc, iters, kmv, relres = self.gp.gp_cg_solve(self.ctx, Bd, t, X0, Vd, t, t, tol, max_iters, w, w.numel())
        return rc, iters, kmv, relres, Vd

    def ap_solve(self, B, tol, block, max_iters=100000, X0=None, Vd=None, picks=False):
        """Returns (rc, iters, kmv_count, relres, picks, V device tensor)."""
        n, t = B.shape
        Bd = B if isinstance(B, torch.Tensor) else self.to(B)
        if Vd is None:
            Vd = torch.zeros((n, t), device=self.dev)
        need = self.gp.gp_ap_workspace_bytes(self.ctx, t, block)
        if self._apwork is None or self._apwork.numel() < need:
            self._apwork = None
            self._apwork = torch.empty(need, dtype=torch.uint8, device=self.dev)
        w = self._apwork
        rc, iters, kmv, relres, pk = self.gp.gp_ap_solve(self.ctx, Bd, t, X0, Vd, t, t, tol, block, max_iters, w,
                                                         w.numel(), want_picks=picks)
        return rc, iters, kmv, relres, pk, Vd

    def sgd_solve(self, B, tol, batches, lr, momentum=0.9, max_iters=None, X0=None, Vd=None):
        """batches: int array [steps, batch].  Returns (rc, iters, kmv_count, relres_est, V device tensor)."""
        n, t = B.shape
        Bd = B if isinstance(B, torch.Tensor) else self.to(B)
        if Vd is None:
            Vd = torch.zeros((n, t), device=self.dev)
        bt = torch.from_numpy(np.ascontiguousarray(batches, dtype=np.int32)).to(self.dev)
        steps, batch = bt.shape
        if max_iters is None:
            max_iters = steps
        assert max_iters <= steps
        need = self.gp.gp_sgd_workspace_bytes(self.ctx, t, batch)
        w = torch.empty(need, dtype=torch.uint8, device=self.dev)
        rc, iters, kmv, relres = self.gp.gp_sgd_solve(self.ctx, Bd, t, X0, Vd, t, t, tol, bt, batch, max_iters, lr,
                                                      momentum, w, w.numel())
        return rc, iters, kmv, relres, Vd

    def grad(self, Vd, Bd):
        t = Bd.shape[1]
        return self.gp.gp_mll_grad(self.ctx, Vd, t, Bd, t, t, self.d)

    def close(self):
        if self.ctx is not None:
            self.gp.gp_destroy(self.ctx)
            self.ctx = None


def relerr(got, ref):
    return float(np.linalg.norm(np.asarray(got, dtype=np.float64) - ref) / np.linalg.norm(ref))
