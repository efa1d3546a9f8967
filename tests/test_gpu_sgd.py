"""GPU parity of the stochastic-gradient solver (gp_sgd_solve) against the fp64 CPU oracle, with the
same mini-batch index sequences on both sides (the library draws no random numbers).

Tolerances:
  iterate after k steps   normwise relative error <= 1e-4 per column for k <= 50 (each step adds one
                          fp32 rounding of the batch rows' products, relative 1e-6, amplified by the
                          momentum recurrence 1 / (1 - rho) = 10; observed ~1e-6);
  estimated residuals     relative 1e-3 (they are fp32 values summed in fp64);
  converged solve         the estimated residual must pass tol; the number of steps equals the oracle's
                          up to 3 % (a column whose estimate crosses tol within rounding of the
                          threshold may stop a few steps apart); the true fp64 residual is reported by
                          the paper to lie below the estimate, and is asserted <= 2 tol.
"""
import numpy as np
import pytest
import torch

from oracle import gp_oracle as orc
from paper_2405_18328_amd.inputs import make
from tests.gpu_util import Dev

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    yield


def _batches(n, b, steps, seed):
    rng = np.random.default_rng(seed)
    return np.stack([rng.permutation(n)[:b] for _ in range(steps)]).astype(np.int32)


def _colrel(got, ref):
    num = np.linalg.norm(got.astype(np.float64) - ref, axis=0)
    return num / np.maximum(np.linalg.norm(ref, axis=0), 1e-300)


@pytest.mark.parametrize("name,kw,b", [
    ("config1", dict(n=700, s=4), 100),      # SE d=8, batch not a multiple of 32
    ("config2", dict(n=1100, s=66), 256),    # Matern d=26, t = 67: three column passes of the tile kernel
    ("config3", dict(n=900, s=2), 900),      # the whole data set as one batch: deterministic heavy ball
])
def test_sgd_steps_match_oracle(name, kw, b):
    w = make(name, **kw)
    a, sigma = 1.1, 0.5
    H = orc.coefficient_matrix(w.X, w.ell, a, sigma, w.kind)
    B = np.asarray(w.B, dtype=np.float64)
    lr = 0.08 * b / (a * a + sigma * sigma) if b < w.n else 0.5 * w.n / np.linalg.eigvalsh(H)[-1]
    bt = _batches(w.n, b, 50, 3)
    rng = np.random.default_rng(4)
    X0 = (0.3 * rng.standard_normal(B.shape)).astype(np.float32)
    dv = Dev(w.X, w.kind, w.ell, a, sigma)
    try:
        for x0 in (None, X0):
            for k in (1, 2, 7, 50):
                Uo, ito, rro = orc.sgd_batched(H, B, list(bt), X0=x0, tol=1e-12, lr=lr, momentum=0.9, max_iters=k)
                rc, it, kmv, rr, Vd = dv.sgd_solve(w.B, 1e-12, bt, lr, max_iters=k, X0=None if x0 is None else dv.to(x0))
                assert rc == 1 and it == k == ito and kmv == (0 if x0 is None else 1)
                got = Vd.cpu().numpy()
                assert np.isfinite(got).all()
                assert (_colrel(got, Uo) <= 1e-4).all(), (k, _colrel(got, Uo).max())
                np.testing.assert_allclose(rr, rro, rtol=1e-3)
    finally:
        dv.close()


def test_sgd_converged_solve_tolerances_freeze_and_warm_start():
    w = make("config1", n=1500, s=6)
    a, sigma = 1.0, 0.6
    b = 200
    H = orc.coefficient_matrix(w.X, w.ell, a, sigma, w.kind)
    B = np.asarray(w.B, dtype=np.float64).copy()
    B[:, -1] = 0.0
    t = B.shape[1]
    tol = np.array([0.01] + [0.1] * (t - 1))          # Appendix B
    lr = 0.08 * b / (a * a + sigma * sigma)
    bt = _batches(w.n, b, 3000, 9)
    Uo, ito, rro = orc.sgd_batched(H, B, list(bt), tol=tol, lr=lr, momentum=0.9)
    assert ito < 3000
    dv = Dev(w.X, w.kind, w.ell, a, sigma)
    try:
        rc, it, kmv, rr, Vd = dv.sgd_solve(B.astype(np.float32), tol, bt, lr)
        got = Vd.cpu().numpy().astype(np.float64)
        assert rc == 0 and kmv == 0
        assert (rr[:-1] < tol[:-1]).all() and rr[-1] == 0.0 and (got[:, -1] == 0.0).all()
        assert abs(it - ito) <= max(2, 0.03 * ito), (it, ito)
        true_rel = np.linalg.norm(H @ got[:, :-1] - B[:, :-1], axis=0) / np.linalg.norm(B[:, :-1], axis=0)
        print(f"[sgd] steps {it} (oracle {ito}), estimated {rr[:-1].max():.4f}, true {true_rel.max():.4f}", flush=True)
        assert (true_rel <= 2.0 * tol[:-1]).all()
        # probe columns stopped early: they are further from the solution than the y column
        sol = np.linalg.solve(H, B[:, :-1])
        err = np.linalg.norm(got[:, :-1] - sol, axis=0) / np.linalg.norm(sol, axis=0)
        assert err[0] < err[1:].min()
        # warm start at nearby hyperparameters (Section 3): fewer steps than from zero, one full product
        ell2 = np.asarray(w.ell) * 1.03
        H2 = orc.coefficient_matrix(w.X, ell2, a, sigma, w.kind)
        dv.set_theta(ell2, a, sigma)
        _, cold_o, _ = orc.sgd_batched(H2, B, list(bt), tol=tol, lr=lr, momentum=0.9)
        _, warm_o, _ = orc.sgd_batched(H2, B, list(bt), X0=Uo, tol=tol, lr=lr, momentum=0.9)
        rc1, cold, _, _, _ = dv.sgd_solve(B.astype(np.float32), tol, bt, lr)
        rc2, warm, kmvw, _, _ = dv.sgd_solve(B.astype(np.float32), tol, bt, lr, X0=Vd.clone())
        assert rc1 == 0 and rc2 == 0 and kmvw == 1
        assert warm < cold and warm_o < cold_o
        assert abs(cold - cold_o) <= max(2, 0.03 * cold_o) and abs(warm - warm_o) <= max(3, 0.1 * warm_o), (cold, cold_o, warm, warm_o)
        # x0 = the solution: no steps, returned unchanged (in place)
        Vs = dv.to(np.linalg.solve(H2, B))
        keep = Vs.clone()
        rc, it0, _, rr0, Vout = dv.sgd_solve(B.astype(np.float32), tol, bt, lr, X0=Vs, Vd=Vs)
        assert rc == 0 and it0 == 0 and (Vout == keep).all()
    finally:
        dv.close()


@pytest.mark.parametrize("path", ["fp32", "f16x2", "f16x3"])
def test_sgd_every_product_path(monkeypatch, path):
    monkeypatch.setenv("GPWS_PATH", path)
    w = make("config5", n=1000, s=4)
    a, sigma = 0.9, 0.4
    b = 160
    H = orc.coefficient_matrix(w.X, w.ell, a, sigma, w.kind)
    B = np.asarray(w.B, dtype=np.float64)
    lr = 0.08 * b / (a * a + sigma * sigma)
    bt = _batches(w.n, b, 30, 5)
    dv = Dev(w.X, w.kind, w.ell, a, sigma)
    try:
        Uo, _, rro = orc.sgd_batched(H, B, list(bt), tol=1e-12, lr=lr, momentum=0.9)
        rc, it, _, rr, Vd = dv.sgd_solve(w.B, 1e-12, bt, lr)
        assert rc == 1 and it == 30
        assert (_colrel(Vd.cpu().numpy(), Uo) <= 1e-4).all()
        np.testing.assert_allclose(rr, rro, rtol=1e-3)
    finally:
        dv.close()


def test_sgd_paper_batch_size_and_extreme_shapes():
    """Mini-batches of 1000 (Appendix B) on n = 5000 with 65 columns; then batch = 1, n = 1."""
    w = make("config2", n=5000, s=64)
    a, sigma = 1.0, 0.5
    ell = np.asarray(w.ell_truth, dtype=np.float64)
    H = orc.coefficient_matrix(w.X, ell, a, sigma, w.kind)
    B = np.asarray(w.B, dtype=np.float64)
    bt = _batches(w.n, 1000, 12, 6)
    dv = Dev(w.X, w.kind, ell, a, sigma)
    try:
        Uo, _, rro = orc.sgd_batched(H, B, list(bt), tol=1e-12, lr=50.0, momentum=0.9)
        rc, it, _, rr, Vd = dv.sgd_solve(w.B, 1e-12, bt, 50.0)
        assert rc == 1 and it == 12
        assert (_colrel(Vd.cpu().numpy(), Uo) <= 1e-4).all()
        np.testing.assert_allclose(rr, rro, rtol=1e-3)
        one = _batches(w.n, 1, 20, 7)
        Uo, _, _ = orc.sgd_batched(H, B, list(one), tol=1e-12, lr=0.5, momentum=0.9)
        rc, it, _, _, Vd = dv.sgd_solve(w.B, 1e-12, one, 0.5)
        assert rc == 1 and it == 20 and (_colrel(Vd.cpu().numpy(), Uo) <= 1e-4).all()
        # no steps allowed: the start is returned
        rc, it, _, rr, Vd = dv.sgd_solve(w.B, 1e-3, bt, 50.0, max_iters=0)
        assert rc == 1 and it == 0 and (Vd.cpu().numpy() == 0).all() and np.allclose(rr, 1.0)
    finally:
        dv.close()
    X = np.array([[0.3, -0.2]], dtype=np.float32)
    dv = Dev(X, "se", np.array([1.0, 2.0]), 1.5, 0.5)
    try:
        bt1 = np.zeros((200, 1), dtype=np.int32)
        rc, it, _, rr, Vd = dv.sgd_solve(np.array([[2.0]], dtype=np.float32), 1e-4, bt1, 0.1, momentum=0.5)
        assert rc == 0 and it < 200
        assert abs(float(Vd.cpu().numpy()[0, 0]) - 2.0 / (1.5 ** 2 + 0.25)) < 1e-3
    finally:
        dv.close()


def test_sgd_argument_errors_and_divergence_report():
    w = make("config1", n=300, s=2)
    dv = Dev(w.X, w.kind, w.ell, 1.0, 0.5)
    gp = dv.gp
    try:
        Bd = dv.to(w.B)
        Vd = torch.zeros_like(Bd)
        t = Bd.shape[1]
        bt = torch.from_numpy(_batches(w.n, 50, 40, 1)).to(dv.dev)
        assert gp.gp_sgd_workspace_bytes(dv.ctx, t, 0) == 0 and gp.gp_sgd_workspace_bytes(dv.ctx, t, 301) == 0
        need = gp.gp_sgd_workspace_bytes(dv.ctx, t, 50)
        wk = torch.empty(need + 256, dtype=torch.uint8, device=dv.dev)

        def call(**kw):
            a = dict(tol=0.01, batches=bt, batch=50, max_iters=40, lr=5.0, momentum=0.9, work=wk, bytes=wk.numel())
            a.update(kw)
            return gp.gp_sgd_solve(dv.ctx, Bd, t, None, Vd, t, t, a["tol"], a["batches"], a["batch"], a["max_iters"],
                                   a["lr"], a["momentum"], a["work"], a["bytes"])

        for kw, code in [(dict(batch=0), -1), (dict(batch=301), -1), (dict(lr=0.0), -1), (dict(lr=float("nan")), -1),
                         (dict(momentum=1.0), -1), (dict(momentum=-0.1), -1), (dict(max_iters=-1), -1),
                         (dict(tol=-1.0), -1), (dict(batches=None), -1), (dict(bytes=need - 1), -3),
                         (dict(work=wk[16:], bytes=need), -3)]:
            with pytest.raises(gp.GpError) as e:
                call(**kw)
            assert e.value.code == code, kw
        # an index outside [0, n) is reported, not dereferenced
        bad = bt.clone()
        bad[3, 7] = w.n
        with pytest.raises(gp.GpError) as e:
            call(batches=bad)
        assert e.value.code == -1
        # a learning rate far too large: the residual estimate overflows and the call says so
        with pytest.raises(gp.GpError) as e:
            call(lr=1e6, max_iters=40, tol=1e-12)
        assert e.value.code == -4
        # the context still works afterwards
        rc, it, _, rr = call(tol=0.2, lr=10.0)
        assert rc in (0, 1) and np.isfinite(rr).all()
    finally:
        dv.close()


def test_sgd_many_columns_and_padded_leading_dimensions():
    """t = 300 (more than one pass of 256 columns in the streaming kernels) with leading dimensions larger
    than t for B, x0 and V; the padding columns of V must not be written."""
    w = make("config3", n=420, s=4)
    a, sigma = 1.0, 0.5
    t, b = 300, 96
    rng = np.random.default_rng(3)
    B = rng.standard_normal((w.n, t)).astype(np.float32)
    X0 = (0.2 * rng.standard_normal((w.n, t))).astype(np.float32)
    H = orc.coefficient_matrix(w.X, w.ell, a, sigma, w.kind)
    bt = _batches(w.n, b, 12, 2)
    lr = 0.08 * b / (a * a + sigma * sigma)
    dv = Dev(w.X, w.kind, w.ell, a, sigma)
    gp = dv.gp
    try:
        ldb, ldv = t + 5, t + 9
        Bd = torch.full((w.n, ldb), 7.0, device=dv.dev)
        Bd[:, :t] = dv.to(B)
        Vd = torch.full((w.n, ldv), -777.0, device=dv.dev)
        Vd[:, :t] = dv.to(X0)
        btd = torch.from_numpy(bt).to(dv.dev)
        need = gp.gp_sgd_workspace_bytes(dv.ctx, t, b)
        wk = torch.empty(need, dtype=torch.uint8, device=dv.dev)
        Uo, _, rro = orc.sgd_batched(H, B.astype(np.float64), list(bt), X0=X0.astype(np.float64), tol=1e-12, lr=lr,
                                     momentum=0.9)
        rc, it, kmv, rr = gp.gp_sgd_solve(dv.ctx, Bd, ldb, Vd, Vd, ldv, t, 1e-12, btd, b, 12, lr, 0.9, wk, wk.numel())
        assert rc == 1 and it == 12 and kmv == 1
        got = Vd.cpu().numpy()
        assert (got[:, t:] == -777.0).all()
        assert (_colrel(got[:, :t], Uo) <= 1e-4).all()
        np.testing.assert_allclose(rr, rro, rtol=1e-3)
    finally:
        dv.close()


def test_sgd_random_small_shapes():
    """Twelve seeded combinations of n, d, t, batch size and kernel (odd sizes, t = 1, batch = n): ten
    steps against the oracle with the same mini-batches."""
    rng = np.random.default_rng(2025)
    for case in range(12):
        n = int(rng.integers(33, 700))
        d = int(rng.integers(1, 20))
        t = int(rng.integers(1, 40))
        b = int(rng.integers(1, n + 1)) if case else n
        kind = "se" if case % 2 else "matern32"
        X = rng.standard_normal((n, d)).astype(np.float32)
        ell = rng.uniform(0.8, 2.5, size=d) * np.sqrt(d)
        a, sigma = float(rng.uniform(0.5, 1.5)), float(rng.uniform(0.3, 1.0))
        B = rng.standard_normal((n, t)).astype(np.float32)
        print(f"[sgd-shape] case {case}: n={n} d={d} t={t} batch={b} {kind}", flush=True)
        H = orc.coefficient_matrix(X, ell, a, sigma, kind)
        lr = 0.5 * b / np.linalg.eigvalsh(H)[-1] / 10.0        # stable for any batch: the largest eigenvalue bounds every block's
        bt = _batches(n, b, 10, case)
        dv = Dev(X, kind, ell, a, sigma)
        try:
            Uo, ito, rro = orc.sgd_batched(H, B.astype(np.float64), list(bt), tol=1e-12, lr=lr, momentum=0.9)
            rc, it, _, rr, Vd = dv.sgd_solve(B, 1e-12, bt, lr)
            assert rc == 1 and it == ito == 10
            assert (_colrel(Vd.cpu().numpy(), Uo) <= 1e-4).all(), case
            np.testing.assert_allclose(rr, rro, rtol=1e-3)
        finally:
            dv.close()
