"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle
on the same seeded inputs.  Run with -m gpu on an MI355X.

Tolerances (floating point):
  K V            normwise relative error <= 1e-5 (the stated bar); observed ~2e-7.
  CG solutions   the recursive residual must meet tol; the true residual recomputed in fp64
                 may exceed tol by the fp32 attainable-accuracy term C eps32 kappa(H), stated per test;
                 forward error vs the Cholesky solution <= kappa * residual.
  MLL gradient   normwise relative error <= 1e-3 with identical probes (the stated bar).
"""
import numpy as np
import pytest
import torch

from oracle import gp_oracle as orc
from paper_2405_18328_amd.inputs import make
from tests.gpu_util import Dev, relerr

pytestmark = pytest.mark.gpu

KMV_TOL = 1e-5
GRAD_TOL = 1e-3


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    yield


def _dev(w, **theta):
    return Dev(w.X, w.kind, theta.get("ell", w.ell), theta.get("a", w.a), theta.get("sigma", w.sigma))


# ------------------------------------------------------------------ K V
KMV_CASES = [
    ("config1", dict(), None),                        # n=2048, d=8, t=17: the whole small config
    ("config1", dict(n=1000, s=4), None),             # ragged n (not a multiple of 32), t=5
    ("config1", dict(n=31, s=2), None),               # smaller than one tile
    ("config2", dict(n=3000), None),                  # d=26 Matern, t=65, ragged, start theta
    ("config2", dict(n=2048), "truth"),               # same at the data-generating lengthscales
    ("config3", dict(n=4500), None),                  # d=3 SE
    ("config4", dict(n=1500), None),                  # d=90 Matern, ell = sqrt(d)
    ("config4", dict(n=1024, ell_value=1.0), None),   # literal ell = 1: K is numerically the identity
    ("config5", dict(n=4000), None),                  # d=11 SE with duplicated rows
]


@pytest.mark.parametrize("name,kw,theta", KMV_CASES)
@pytest.mark.parametrize("add_noise", [0, 1])
def test_kmv_matches_dense_oracle(name, kw, theta, add_noise):
    w = make(name, **kw)
    ell = w.ell_truth if theta == "truth" else w.ell
    dv = Dev(w.X, w.kind, ell, 1.3, 0.6)
    try:
        got = dv.kmv(w.B, add_noise)
        ref = orc.kmv_dense(w.X, ell, 1.3, w.kind, w.B, sigma=0.6 if add_noise else None)
        assert np.isfinite(got).all()
        assert relerr(got, ref) <= KMV_TOL
        # element by element, scaled by the size of the terms that were summed
        scale = np.abs(ref).max()
        assert np.abs(got - ref).max() <= 50 * KMV_TOL * scale
    finally:
        dv.close()


@pytest.mark.parametrize("t", [1, 2, 17, 32, 33, 64, 65, 66, 97, 130])
def test_kmv_column_counts_and_leading_dimensions(t):
    w = make("config5", n=700, s=max(t - 1, 1))
    rng = np.random.default_rng(t)
    V = rng.standard_normal((w.n, t)).astype(np.float32)
    dv = _dev(w)
    try:
        ref = orc.kmv_dense(w.X, w.ell, w.a, w.kind, V, sigma=w.sigma)
        got = dv.kmv(V, 1, ldv=t + 3, ldo=t + 5)
        assert relerr(got, ref) <= KMV_TOL
    finally:
        dv.close()


PATH_CASES = [("config1", dict(n=1500)), ("config2", dict(n=2100)), ("config4", dict(n=1100)), ("config5", dict(n=2500))]


@pytest.mark.parametrize("path", ["fp32", "f16x2", "f16x3"])
@pytest.mark.parametrize("name,kw", PATH_CASES)
def test_kmv_every_product_path(monkeypatch, path, name, kw):
    """The library picks the product path (fp32 MFMA, split-fp16 with 2 or 3 distance pieces) from
    the largest scaled squared norm; GPWS_PATH pins it so that each path meets the same bar."""
    monkeypatch.setenv("GPWS_PATH", path)
    w = make(name, **kw)
    dv = Dev(w.X, w.kind, w.ell, 0.9, 0.3)
    try:
        for V in (w.B, w.B * np.float32(1e-12), w.B * np.logspace(-8, 8, w.s + 1, dtype=np.float32)):
            got = dv.kmv(V, 1)
            ref = orc.kmv_dense(w.X, w.ell, 0.9, w.kind, V, sigma=0.3)
            assert relerr(got, ref) <= KMV_TOL
            # per column as well: the power-of-two column scaling must not favour large columns
            cerr = np.linalg.norm(got - ref, axis=0) / np.linalg.norm(ref, axis=0)
            assert cerr.max() <= KMV_TOL, cerr
    finally:
        dv.close()


@pytest.mark.parametrize("kind,path", [("se", None), ("matern32", None), ("matern32", "f16x3"), ("se", "f16x3")])
def test_kmv_and_gradient_at_the_largest_dimension(monkeypatch, kind, path):
    """d = 126 (the documented maximum): the SE operand set no longer fits the widest fp16 bucket and
    the product must fall back to fp32 (also when another path is asked for); Matern-3/2 still fits,
    with two pieces by default and with three (the largest kernels of the library) when pinned."""
    if path:
        monkeypatch.setenv("GPWS_PATH", path)
    rng = np.random.default_rng(126)
    n, d, t = 700, 126, 5
    X = rng.standard_normal((n, d)).astype(np.float32)
    ell = np.full(d, np.sqrt(d)) * rng.uniform(0.8, 1.25, d)
    V = rng.standard_normal((n, t)).astype(np.float32)
    B = rng.standard_normal((n, t)).astype(np.float32)
    dv = Dev(X, kind, ell, 1.2, 0.3)
    try:
        assert dv.gp.gp_product_path(dv.ctx) == (0 if kind == "se" else (2 if path else 1))
        assert relerr(dv.kmv(V, 1), orc.kmv_dense(X, ell, 1.2, kind, V, sigma=0.3)) <= KMV_TOL
        g = dv.grad(dv.to(V), dv.to(B))
        assert relerr(g, orc.mll_grad_hutchinson(X, ell, 1.2, 0.3, kind, B, V=V)) <= GRAD_TOL
        Xs = rng.standard_normal((40, d)).astype(np.float32)
        assert relerr(dv.predict(Xs, V), orc.cross_kmv(Xs, X, ell, 1.2, kind, V)) <= KMV_TOL
    finally:
        dv.close()


def test_kmv_path_selection_by_norm():
    """Small lengthscales blow up |x/ell|^2: the automatic choice must still meet the bar
    (three fp16 pieces, then the fp32 MFMA path beyond fp16's range)."""
    w = make("config3", n=2000)
    for scale, in ((1.0,), (0.08,), (0.004,)):
        ell = w.ell * scale
        dv = Dev(w.X, w.kind, ell, 1.0, 0.1)
        try:
            got = dv.kmv(w.B, 1)
            ref = orc.kmv_dense(w.X, ell, 1.0, w.kind, w.B, sigma=0.1)
            assert relerr(got, ref) <= KMV_TOL, scale
        finally:
            dv.close()


def test_kmv_large_n_sampled_rows_and_properties():
    """n large enough for an unsplit launch with two sub-tiles per wave; the oracle computes exact
    rows for a seeded sample, plus properties that hold at any size."""
    w = make("config5", n=70001)
    dv = _dev(w)
    try:
        got = dv.kmv(w.B, 1)
        rows = np.random.default_rng(3).choice(w.n, size=96, replace=False)
        rows[:3] = [0, w.n - 1, 32767]
        ref = orc.kmv_rows(w.X, w.ell, w.a, w.kind, w.B, rows, sigma=w.sigma)
        assert relerr(got[rows], ref) <= KMV_TOL
        # duplicated input rows give equal output rows for K V (without the noise term)
        gk = dv.kmv(w.B, 0)
        Xv = w.X.view([("", w.X.dtype)] * w.d).ravel()
        _, first, inv = np.unique(Xv, return_index=True, return_inverse=True)
        dup = np.nonzero(first[inv] != np.arange(w.n))[0][:200]
        assert dup.size > 50
        src = first[inv][dup]
        assert np.abs(gk[dup] - gk[src]).max() <= 1e-5 * np.abs(gk).max()
        # symmetry of K: u^T (K v) = v^T (K u)
        u, v = gk[:, 1], gk[:, 2]
        b1, b2 = w.B[:, 1].astype(np.float64), w.B[:, 2].astype(np.float64)
        assert abs(b2 @ u - b1 @ v) <= 1e-5 * (np.linalg.norm(b2) * np.linalg.norm(u))
    finally:
        dv.close()


def test_kmv_infinite_lengthscale_closed_form():
    """ell -> inf: K V = a^2 1 (1^T V), valid at any n."""
    w = make("config3", n=20000)
    dv = Dev(w.X, w.kind, np.full(w.d, 1e6), 1.5, 0.0)
    try:
        got = dv.kmv(w.B, 0)
        ref = 2.25 * np.ones((w.n, 1)) * w.B.astype(np.float64).sum(axis=0)
        assert np.abs(got - ref).max() <= 1e-5 * np.abs(w.B).sum(axis=0).max() * 2.25
    finally:
        dv.close()


def test_kmv_is_deterministic():
    w = make("config2", n=2500)
    dv = _dev(w)
    try:
        a = dv.kmv(w.B, 1)
        b = dv.kmv(w.B, 1)
        assert np.array_equal(a, b)
    finally:
        dv.close()


# ------------------------------------------------------------------ CG
def test_cg_config1_against_cholesky():
    """The whole small config: one batched solve to relative residual 1e-6, compared with the
    CPU Cholesky solve.  fp32 attainable accuracy: true residual <= tol + 40 eps32 kappa(H)."""
    w = make("config1")
    dv = _dev(w)
    try:
        rc, iters, kmv, relres, Vd = dv.solve(w.B, w.tol)
        assert rc == 0 and kmv == iters
        assert (relres < w.tol).all()
        H = orc.coefficient_matrix(w.X, w.ell, w.a, w.sigma, w.kind)
        V = Vd.cpu().numpy().astype(np.float64)
        Bn = np.linalg.norm(w.B, axis=0)
        true_rel = np.linalg.norm(H @ V - w.B, axis=0) / Bn
        ev = np.linalg.eigvalsh(H)
        kappa = ev[-1] / ev[0]
        eps32 = 2.0 ** -24
        bound = w.tol + 40 * eps32 * kappa
        assert true_rel.max() <= bound, (true_rel.max(), bound)
        Vstar = orc.chol_solve(H, w.B)
        assert relerr(V, Vstar) <= kappa * bound
        # iteration count against the oracle's fp64 CG with the same rule; at tol = 1e-6 the fp32
        # recurrence sits near its attainable accuracy and rounding delays convergence, so the
        # fp32 count may exceed the fp64 one by up to 20 %
        _, it64, _ = orc.cg_batched(orc.dense_matvec(H), w.B, tol=w.tol, max_iters=2000)
        assert it64 - 2 <= iters <= 1.2 * it64 + 2, (iters, it64)
    finally:
        dv.close()


@pytest.mark.parametrize("name,kw", [("config2", dict(n=2500)), ("config5", dict(n=1800)), ("config3", dict(n=1500))])
def test_cg_stopping_rule_and_solution(name, kw):
    w = make(name, **kw)
    dv = _dev(w)
    try:
        t = w.s + 1
        tol = np.full(t, 0.1, dtype=np.float32)      # Appendix B: 0.01 for y, 0.1 for the probes
        tol[0] = 0.01
        rc, iters, kmv, relres, Vd = dv.solve(w.B, tol)
        assert rc == 0 and (relres < tol).all()
        H = orc.coefficient_matrix(w.X, w.ell, w.a, w.sigma, w.kind)
        V = Vd.cpu().numpy().astype(np.float64)
        true_rel = np.linalg.norm(H @ V - w.B, axis=0) / np.linalg.norm(w.B, axis=0)
        assert (true_rel < tol * 1.02).all()
        # Iteration counts.  In exact arithmetic the count is fixed by H and B; in floating point
        # rounding in the product delays convergence on ill-conditioned H (kappa ~ 1e5 here), so the
        # fp32 path legitimately needs more products than the fp64 oracle.  Two checks: never fewer
        # than fp64 (minus slack), and within 15 % of the oracle's own CG when its product is
        # rounded to fp32 -- i.e. the count is what fp32 products imply, not an implementation defect.
        _, it64, _ = orc.cg_batched(orc.dense_matvec(H), w.B, tol=tol, max_iters=5000)
        H32 = H.astype(np.float32)
        mv32 = lambda P: (H32 @ P.astype(np.float32)).astype(np.float64)
        _, it32, _ = orc.cg_batched(mv32, w.B, tol=tol, max_iters=5000)
        assert iters >= it64 - 2, (iters, it64)
        assert abs(iters - it32) <= max(2, 0.15 * it32), (iters, it32, it64)
    finally:
        dv.close()


def test_cg_warm_start_semantics():
    w = make("config2", n=2000)
    dv = _dev(w)
    try:
        tol = 1e-3
        rc, it_cold, kmv_cold, _, Vd = dv.solve(w.B, tol)
        assert rc == 0 and it_cold > 3 and kmv_cold == it_cold
        # same theta, x0 = previous solution: nothing to do, one product for the initial residual
        rc, it0, kmv0, relres0, Vd2 = dv.solve(w.B, tol * 1.5, X0=Vd, Vd=Vd.clone())
        assert rc == 0 and it0 == 0 and kmv0 == 1 and (relres0 < tol * 1.5).all()
        assert torch.equal(Vd2, Vd)
        # a small step in theta: warm start (in place, dX0 == dV) needs fewer iterations than cold
        ell2 = w.ell * 1.03
        dv.set_theta(ell2, w.a * 1.02, w.sigma * 0.98)
        rc, it_cold2, _, _, Vc = dv.solve(w.B, tol)
        Vw = Vd.clone()
        rc, it_warm, kmv_warm, _, Vw = dv.solve(w.B, tol, X0=Vw, Vd=Vw)
        assert rc == 0 and it_warm < it_cold2 and kmv_warm == it_warm + 1
        H2 = orc.coefficient_matrix(w.X, ell2, w.a * 1.02, w.sigma * 0.98, w.kind)
        for Vx in (Vc, Vw):
            V = Vx.cpu().numpy().astype(np.float64)
            tr = np.linalg.norm(H2 @ V - w.B, axis=0) / np.linalg.norm(w.B, axis=0)
            assert (tr < tol * 1.05).all()
        # oracle CG from the same x0 takes about as many iterations
        _, it64, _ = orc.cg_batched(orc.dense_matvec(H2), w.B, X0=Vd.cpu().numpy(), tol=tol, max_iters=5000)
        assert abs(it_warm - it64) <= max(2, 0.15 * it64), (it_warm, it64)
    finally:
        dv.close()


def test_cg_edge_cases():
    w = make("config1", n=600, s=5)
    dv = _dev(w)
    try:
        B = w.B.copy()
        B[:, 3] = 0.0                                   # a zero right-hand side
        X0 = np.random.default_rng(0).standard_normal(B.shape).astype(np.float32)
        rc, iters, kmv, relres, Vd = dv.solve(B, 1e-4, X0=dv.to(X0))
        V = Vd.cpu().numpy()
        assert rc == 0 and (V[:, 3] == 0).all() and relres[3] == 0
        H = orc.coefficient_matrix(w.X, w.ell, w.a, w.sigma, w.kind)
        live = [0, 1, 2, 4, 5]
        tr = np.linalg.norm(H @ V[:, live] - B[:, live], axis=0) / np.linalg.norm(B[:, live], axis=0)
        assert (tr < 1.1e-4).all()
        # iteration cap: usable iterate, flagged
        rc, iters, kmv, relres, _ = dv.solve(B, 1e-6, max_iters=3)
        assert rc == dv.gp.GP_NOT_CONVERGED and iters == 3 and (relres[live] > 1e-6).all()
        rc, iters, kmv, relres, Vz = dv.solve(B, 1e-6, max_iters=0)
        assert rc == dv.gp.GP_NOT_CONVERGED and iters == 0 and (Vz == 0).all()
        # a single right-hand side
        rc, iters, _, relres, V1 = dv.solve(B[:, :1], 1e-5)
        assert rc == 0 and relerr(V1.cpu().numpy(), orc.chol_solve(H, B[:, :1])) < 1e-3
        # deterministic: two identical solves give identical bits
        _, _, _, _, Va = dv.solve(w.B, 1e-5)
        _, _, _, _, Vb = dv.solve(w.B, 1e-5)
        assert torch.equal(Va, Vb)
    finally:
        dv.close()


@pytest.mark.parametrize("n,d,t", [(1, 1, 1), (2, 1, 3), (33, 2, 1), (257, 1, 1024), (300, 3, 200)])
@pytest.mark.parametrize("kind", ["se", "matern32"])
def test_extreme_shapes_all_entry_points(n, d, t, kind):
    """Smallest problems, a single input dimension, the largest number of right-hand sides, and
    leading dimensions larger than t, through every method entry point."""
    rng = np.random.default_rng(1000 * n + t)
    X = rng.standard_normal((n, d)).astype(np.float32)
    ell = rng.uniform(0.7, 1.5, d)
    a, sigma = 1.1, 0.7
    B = rng.standard_normal((n, t)).astype(np.float32)
    V = rng.standard_normal((n, t)).astype(np.float32)
    dv = Dev(X, kind, ell, a, sigma)
    gp = dv.gp
    try:
        H = orc.coefficient_matrix(X, ell, a, sigma, kind)
        assert relerr(dv.kmv(V, 1, ldv=t + 1, ldo=t + 2), H @ V.astype(np.float64)) <= KMV_TOL
        # solve with padded leading dimensions, solution written in place of the initial guess
        ldb, ldv = t + 3, t + 2
        Bd = torch.full((n, ldb), float("nan"), device=dv.dev)
        Bd[:, :t] = dv.to(B)
        Vd = torch.full((n, ldv), 7.0, device=dv.dev)
        Vd[:, :t] = 0.0
        work = dv.work(t)
        rc, iters, kmv, relres = gp.gp_cg_solve(dv.ctx, Bd, ldb, Vd, Vd, ldv, t, 1e-5, 500, work, work.numel())
        assert rc == 0 and iters <= n + 2
        got = Vd.cpu().numpy()
        assert (got[:, t:] == 7.0).all(), "padding columns of dV were written"
        ref = orc.chol_solve(H, B)
        assert relerr(got[:, :t], ref) <= 1e-3
        g = gp.gp_mll_grad(dv.ctx, Vd, ldv, Bd, ldb, t, d)
        gref = orc.mll_grad_hutchinson(X, ell, a, sigma, kind, B, V=got[:, :t])
        assert np.isfinite(g).all() and relerr(g, gref) <= GRAD_TOL
        Xs = rng.standard_normal((5, d)).astype(np.float32)
        assert relerr(dv.predict(Xs, V), orc.cross_kmv(Xs, X, ell, a, kind, V)) <= KMV_TOL
    finally:
        dv.close()


def test_cg_sherman_morrison_at_scale():
    """ell -> inf makes H = sigma^2 I + a^2 11^T, whose inverse has a closed form at any n."""
    w = make("config3", n=150000, s=3)
    a, sigma = 0.8, 0.5
    dv = Dev(w.X, w.kind, np.full(w.d, 1e6), a, sigma)
    try:
        rc, iters, _, relres, Vd = dv.solve(w.B, 1e-5, max_iters=20)
        B = w.B.astype(np.float64)
        closed = (B - a * a * np.ones((w.n, 1)) * B.sum(axis=0) / (sigma ** 2 + w.n * a * a)) / sigma ** 2
        assert rc == 0 and iters <= 8      # two distinct eigenvalues: 2 steps exactly, a few more in fp32
        assert relerr(Vd.cpu().numpy(), closed) < 1e-4
    finally:
        dv.close()


# ------------------------------------------------------------------ gradient
GRAD_CASES = [
    ("config1", dict()),                     # SE, d=8, t=17
    ("config2", dict(n=1500)),               # Matern, d=26, t=65
    ("config5", dict(n=1400)),               # SE, d=11, duplicated rows
    ("config3", dict(n=1300, s=7)),          # SE, d=3, t=8
    ("config4", dict(n=700, s=20)),          # Matern, d=90: several column passes
    ("config2", dict(n=900, s=99)),          # t=100: two right-hand-side blocks
    ("config1", dict(n=500, s=0)),           # no probes: quadratic term only
]


@pytest.mark.parametrize("name,kw", GRAD_CASES)
def test_gradient_matches_oracle_at_same_V(name, kw):
    """The tile pass against the oracle's estimator evaluated at the same V (isolates it from
    solver error), for an arbitrary V, and the two vector identities."""
    w = make(name, **kw)
    a, sigma = 1.2, 0.45
    ell = w.ell * np.linspace(0.8, 1.3, w.d)
    dv = Dev(w.X, w.kind, ell, a, sigma)
    try:
        rng = np.random.default_rng(11)
        V = (rng.standard_normal(w.B.shape) * 0.3).astype(np.float32)
        Vd, Bd = dv.to(V), dv.to(w.B)
        g = dv.grad(Vd, Bd)
        ref = orc.mll_grad_hutchinson(w.X, ell, a, sigma, w.kind, w.B, V=V)
        assert g.shape == (w.d + 2,) and np.isfinite(g).all()
        assert relerr(g, ref) <= GRAD_TOL, (g, ref)
        assert relerr(g[: w.d], ref[: w.d]) <= GRAD_TOL
        s = w.s
        V64, B64 = V.astype(np.float64), w.B.astype(np.float64)
        gs = sigma * (V64[:, 0] @ V64[:, 0] - (np.sum(V64[:, 1:] * B64[:, 1:]) / s if s else 0.0))
        assert g[-1] == pytest.approx(gs, rel=1e-6)
        # dL/da through the library's own product K C
        C = np.concatenate([V[:, :1], w.B[:, 1:]], axis=1)
        KC = dv.kmv(C, 0)
        ga = (2 / a) * (0.5 * V64[:, 0] @ KC[:, 0] - (np.sum(V64[:, 1:] * KC[:, 1:]) / (2 * s) if s else 0.0))
        assert g[-2] == pytest.approx(ga, rel=1e-4, abs=1e-4 * np.abs(g).max())
    finally:
        dv.close()


@pytest.mark.parametrize("path", ["fp32", "f16x2", "f16x3"])
@pytest.mark.parametrize("name,kw", [("config2", dict(n=1100)), ("config5", dict(n=1300, s=40)), ("config3", dict(n=900, s=5))])
def test_gradient_every_product_path(monkeypatch, path, name, kw):
    """Same bar on each arithmetic path of the tile pass, with badly scaled columns of V: the fp16
    paths rescale the right-hand-side columns by powers of two and must not lose the small ones."""
    monkeypatch.setenv("GPWS_PATH", path)
    w = make(name, **kw)
    dv = Dev(w.X, w.kind, w.ell, 0.8, 0.2)
    try:
        rng = np.random.default_rng(23)
        V0 = rng.standard_normal(w.B.shape).astype(np.float32)
        for colscale in (np.ones(w.s + 1), np.logspace(-6, 6, w.s + 1), np.full(w.s + 1, 1e-9)):
            V = (V0 * colscale).astype(np.float32)
            g = dv.grad(dv.to(V), dv.to(w.B))
            ref = orc.mll_grad_hutchinson(w.X, w.ell, 0.8, 0.2, w.kind, w.B, V=V)
            assert np.isfinite(g).all()
            assert relerr(g, ref) <= GRAD_TOL, (path, g, ref)
    finally:
        dv.close()


@pytest.mark.parametrize("name,kw", [("config1", dict()), ("config2", dict(n=2000))])
def test_gradient_end_to_end_after_solve(name, kw):
    """Solve tightly on the GPU, then compare the gradient with the oracle's Cholesky-based
    estimator using identical probes: the 1e-3 bar of the whole path."""
    w = make(name, **kw)
    dv = _dev(w)
    try:
        rc, iters, _, _, Vd = dv.solve(w.B, 2e-6)
        assert rc == 0
        g = dv.grad(Vd, dv.to(w.B))
        ref = orc.mll_grad_hutchinson(w.X, w.ell, w.a, w.sigma, w.kind, w.B)
        assert relerr(g, ref) <= GRAD_TOL, (g, ref)
    finally:
        dv.close()


# ------------------------------------------------------------------ prediction (cross-covariance product)
PREDICT_CASES = [
    ("config1", dict(n=1500), 333, 1),       # t = 1: the posterior mean, ragged m
    ("config2", dict(n=2100), 700, 65),      # Matern d = 26, all columns of a batch
    ("config5", dict(n=9000), 8500, 3),      # m large enough for two sub-tiles per wave
    ("config3", dict(n=1200), 1, 2),         # a single test point
    ("config4", dict(n=1000), 40, 5),        # d = 90
]


@pytest.mark.parametrize("name,kw,m,t", PREDICT_CASES)
def test_predict_matches_dense_oracle(name, kw, m, t):
    """OUT = k(X*, X) V against the dense oracle, X* drawn around the training inputs."""
    w = make(name, **kw)
    rng = np.random.default_rng(m + t)
    Xs = (w.X[rng.integers(0, w.n, size=m)] + 0.3 * rng.standard_normal((m, w.d)) * w.X.std(axis=0)).astype(np.float32)
    if m > 4:
        Xs[:3] = w.X[:3]                       # test points that coincide with training points
    V = rng.standard_normal((w.n, t)).astype(np.float32)
    dv = Dev(w.X, w.kind, w.ell, 1.1, 0.2)
    try:
        got = dv.predict(Xs, V, ldo=t + 2)
        ref = orc.cross_kmv(Xs, w.X, w.ell, 1.1, w.kind, V)
        assert got.shape == (m, t) and np.isfinite(got).all()
        assert relerr(got, ref) <= KMV_TOL
        assert np.abs(got - ref).max() <= 50 * KMV_TOL * np.abs(ref).max()
        # X* = X reproduces the square product without the noise term
        if w.n <= 2100:
            sq = dv.kmv(V, 0)
            assert relerr(dv.predict(w.X, V), sq) <= KMV_TOL   # coincident points: only the square product sets r^2 = 0 exactly
    finally:
        dv.close()


@pytest.mark.parametrize("path", ["fp32", "f16x2", "f16x3"])
def test_predict_every_product_path_and_far_points(monkeypatch, path):
    """Test points far from the data raise the scaled norm: the product must move to the arithmetic
    that covers it (three fp16 pieces, then fp32) whatever the training inputs alone would select."""
    monkeypatch.setenv("GPWS_PATH", path)
    w = make("config3", n=1800)
    rng = np.random.default_rng(9)
    V = rng.standard_normal((w.n, 4)).astype(np.float32)
    dv = Dev(w.X, w.kind, w.ell * 2.0, 1.0, 0.1)
    try:
        for spread in (1.0, 12.0):
            Xs = (spread * rng.standard_normal((257, w.d))).astype(np.float32)
            got = dv.predict(Xs, V)
            ref = orc.cross_kmv(Xs, w.X, w.ell * 2.0, 1.0, w.kind, V)
            assert np.abs(got - ref).max() <= KMV_TOL * max(np.abs(ref).max(), 1e-3 * np.abs(V).sum(axis=0).max())
    finally:
        dv.close()
    monkeypatch.delenv("GPWS_PATH")
    dv = Dev(w.X, w.kind, w.ell * 0.05, 1.0, 0.1)   # automatic choice, scaled norms beyond fp16's range for far points
    try:
        Xs = np.concatenate([w.X[:50], 40.0 * rng.standard_normal((50, w.d))]).astype(np.float32)
        got = dv.predict(Xs, V)
        ref = orc.cross_kmv(Xs, w.X, w.ell * 0.05, 1.0, w.kind, V)
        # Here |x/ell|^2 reaches ~1e6 and the fp32 fallback forms r^2 by cancellation of terms that
        # large: its absolute error is eps32 (|xs_i|^2 + |xs_j|^2), which for the coincident pairs of
        # the first 50 rows (r^2 = 0, K = 1) is a 1e-4-class error of the row; K is almost the
        # identity in this regime.  The far rows must come out as (numerically) zero.
        assert np.abs(got[:50] - ref[:50]).max() <= 1e-3 * np.abs(ref).max()
        assert np.abs(got[50:] - ref[50:]).max() <= KMV_TOL * np.abs(ref).max()
    finally:
        dv.close()


def test_posterior_mean_end_to_end():
    """Solve H v_y = y on the GPU, predict at held-out points, compare with the oracle's Cholesky mean."""
    w = make("config1", n=1200)
    rng = np.random.default_rng(4)
    Xs = rng.standard_normal((300, w.d)).astype(np.float32)
    dv = _dev(w)
    try:
        rc, _, _, _, Vd = dv.solve(w.B[:, :1], 1e-6)
        assert rc == 0
        mu = dv.predict(Xs, Vd.cpu().numpy())
        vy = orc.chol_solve(orc.coefficient_matrix(w.X, w.ell, w.a, w.sigma, w.kind), w.B[:, :1])
        ref = orc.cross_kmv(Xs, w.X, w.ell, w.a, w.kind, vy)
        assert np.abs(mu - ref).max() <= 1e-4 * np.abs(ref).max()
    finally:
        dv.close()


# ------------------------------------------------------------------ error paths (host-side checks)
def test_argument_errors_return_codes():
    w = make("config1", n=200, s=3)
    dv = _dev(w)
    gp = dv.gp
    try:
        t = 4
        Bd = dv.to(w.B)
        out = torch.empty_like(Bd)
        with pytest.raises(gp.GpError) as e:
            gp.gp_kmv(dv.ctx, Bd, 3, t, out, t, 0)            # ld < t
        assert e.value.code == gp.GP_ERR_ARG and "leading dimension" in str(e.value)
        with pytest.raises(gp.GpError) as e:
            gp.gp_kmv(dv.ctx, Bd, t, t, Bd, t, 0)             # aliasing
        assert e.value.code == gp.GP_ERR_ARG
        with pytest.raises(gp.GpError) as e:
            gp.gp_kmv(dv.ctx, Bd, t, 0, out, t, 0)
        assert e.value.code == gp.GP_ERR_ARG
        with pytest.raises(gp.GpError) as e:
            gp.gp_set_theta(dv.ctx, np.array([1.0] * (w.d - 1) + [-1.0]), 1.0, 1.0)
        assert e.value.code == gp.GP_ERR_ARG
        small = torch.empty(1024, dtype=torch.uint8, device=dv.dev)
        with pytest.raises(gp.GpError) as e:
            gp.gp_cg_solve(dv.ctx, Bd, t, None, out, t, t, 1e-3, 10, small, small.numel())
        assert e.value.code == gp.GP_ERR_WORKSPACE
        with pytest.raises(gp.GpError) as e:
            gp.gp_cg_solve(dv.ctx, Bd, t, None, out, t, t, 0.0, 10, dv.work(t), dv.work(t).numel())
        assert e.value.code == gp.GP_ERR_ARG
        with pytest.raises(gp.GpError) as e:
            gp.gp_predict(dv.ctx, dv.X, 0, Bd, t, t, out, t)  # no test points
        assert e.value.code == gp.GP_ERR_ARG
        with pytest.raises(gp.GpError) as e:
            gp.gp_predict(dv.ctx, None, 5, Bd, t, t, out, t)
        assert e.value.code == gp.GP_ERR_ARG
        with pytest.raises(gp.GpError) as e:
            gp.gp_predict(dv.ctx, dv.X, 5, Bd, t, t, out, t - 1)
        assert e.value.code == gp.GP_ERR_ARG
        # a context without theta refuses to compute
        ctx2 = gp.gp_create(0, w.n, w.d, dv.X, None)
        with pytest.raises(gp.GpError):
            gp.gp_kmv(ctx2, Bd, t, t, out, t, 0)
        gp.gp_destroy(ctx2)
        # the context is still usable after the errors
        assert relerr(dv.kmv(w.B, 0), orc.kmv_dense(w.X, w.ell, w.a, w.kind, w.B)) <= KMV_TOL
    finally:
        dv.close()


def test_cg_breakdown_is_reported_not_hung():
    """sigma = 0 with duplicated rows makes H singular; a right-hand side outside its range either
    converges in the least-squares sense or is reported as breakdown / not converged, and the call returns."""
    w = make("config5", n=400, s=2)
    X = w.X.copy()
    X[1::2] = X[0::2]                                     # every row duplicated
    dv = Dev(X, w.kind, w.ell, 1.0, 0.0)
    try:
        rc = None
        try:
            rc, iters, _, relres, _ = dv.solve(w.B, 1e-6, max_iters=50)
        except dv.gp.GpError as e:
            assert e.code == dv.gp.GP_ERR_BREAKDOWN
        assert rc in (None, 0, 1)
    finally:
        dv.close()


# ------------------------------------------------------------------ optimiser traces (Section 4, hyperparameter traces)
@pytest.mark.parametrize("solver", ["cg", "ap", "sgd"])
def test_optimiser_trace_tracks_the_exact_gradient_trace(solver):
    """The paper's end-to-end claim (Section 4, hyperparameter-trace figures): with warm starts and the
    solver tolerances of Appendix B the hyperparameters follow the trace obtained with exact (Cholesky)
    gradients.  Three traces from the same start (every hyperparameter 1.0, Adam lr 0.1):
      exact       oracle, closed-form gradient of the marginal likelihood;
      same probes oracle, the stochastic estimator with exact solves and the probes the GPU run uses
                  (differs from `exact` by the estimator's noise only, s = 16 probes);
      gpu         the library: warm-started solver to tolerance 0.01 / 0.1, fp32.
    The gpu trace must stay within 10 % of `same probes` in every hyperparameter at every step (what solves
    stopped at relative residuals 0.01 / 0.1 add; observed 3.3 % with CG, 5.3 % with alternating
    projections, 8.4 % with SGD, which stops on its residual estimate), and no further from `exact` than the estimator's
    own noise (measured oracle against oracle: up to ~15 % on single lengthscales at s = 16) plus 5 %."""
    from paper_2405_18328_amd.mll import MllOptimizer
    w = make("config1", n=1000)
    d, s, steps = w.d, w.s, 20
    y = np.asarray(w.y, dtype=np.float64)
    B = np.concatenate([y[:, None], np.asarray(w.Z, dtype=np.float64)], axis=1)
    raw0 = orc.softplus_inverse(np.ones(d + 2))
    exact = np.array(orc.adam_ascent(raw0, lambda th: orc.mll_grad_exact(w.X, y, th[:d], th[d], th[d + 1], w.kind), steps))
    same = np.array(orc.adam_ascent(
        raw0, lambda th: orc.mll_grad_hutchinson(w.X, th[:d], th[d], th[d + 1], w.kind, B), steps))
    tol = np.array([0.01] + [0.1] * s, dtype=np.float32)
    opt = MllOptimizer(w.X, w.y, w.Z, w.kind, np.ones(d), 1.0, 1.0, tol, warm=True, max_iters=100000,
                       solver=solver, block=250, batch=250, sgd_lr=12.5)
    try:
        recs = [opt.step() for _ in range(steps)]
        gpu = np.array([r.theta for r in recs[1:]] + [opt.theta])     # theta after every step
        assert all(r.rc == 0 for r in recs)
        dev_same = np.abs(gpu - same) / same
        dev_exact = np.abs(gpu - exact) / exact
        print(f"[trace] {solver}: max deviation from same-probe trace {dev_same.max():.4f}, from exact trace "
              f"{dev_exact.max():.4f}; iterations {[r.iters for r in recs]}", flush=True)
        assert np.abs(recs[0].theta - 1.0).max() == 0.0
        assert dev_same.max() <= 0.10
        noise = np.abs(same - exact) / exact               # what the estimator alone adds (oracle vs oracle)
        assert dev_exact.max() <= 0.25 and (dev_exact <= noise.max() + 0.05).all()
        # the hyperparameters moved (the comparison is not between three constant traces)
        assert np.abs(gpu[-1] - 1.0).max() > 0.3
        # warm starts: later solves are cheaper than the first
        assert np.mean([r.iters for r in recs[5:]]) < recs[0].iters
    finally:
        opt.close()


def test_optimiser_trace_on_the_papers_kernel_and_shape():
    """The trace experiment of Section 4 on the kernel and input shape the paper runs (Matern-3/2 with
    per-dimension lengthscales, d = 26, inputs uniform in [-1, 1]^d like the pol-shaped benchmark
    configuration), CG with the tolerances of Appendix B (0.01 for y, 0.1 for the probes), warm starts,
    15 Adam steps from 1.0.  Reference: the oracle's trace with exact (Cholesky) solves and the same fixed
    probes, its estimator evaluated row block by row block (n = 3000: each of the 28 derivative matrices
    would be 72 MB dense).  The library's trace must stay within 10 % of it in every hyperparameter at
    every step, the same bar as for the squared-exponential case above (observed there 3.3 %)."""
    from paper_2405_18328_amd.mll import MllOptimizer
    w = make("config2", n=3000, s=16)
    d, s, steps = w.d, w.s, 15
    y = np.asarray(w.y, dtype=np.float64)
    B = np.concatenate([y[:, None], np.asarray(w.Z, dtype=np.float64)], axis=1)

    def estimator(th):
        ell, a, sigma = th[:d], th[d], th[d + 1]
        V = orc.chol_solve(orc.coefficient_matrix(w.X, ell, a, sigma, w.kind), B)
        return orc.mll_grad_hutchinson_rows(w.X, ell, a, sigma, w.kind, B, V, row_block=64, workers=8)

    print("[trace] oracle trace (15 steps of Cholesky solve + estimator)", flush=True)
    same = np.array(orc.adam_ascent(orc.softplus_inverse(np.ones(d + 2)), estimator, steps))
    tol = np.array([0.01] + [0.1] * s, dtype=np.float32)
    opt = MllOptimizer(w.X, w.y, w.Z, w.kind, np.ones(d), 1.0, 1.0, tol, warm=True, max_iters=2000)
    try:
        recs = [opt.step() for _ in range(steps)]
        gpu = np.array([r.theta for r in recs[1:]] + [opt.theta])     # theta after every step
        assert all(r.rc == 0 for r in recs)
        dev_same = np.abs(gpu - same) / same
        print(f"[trace] matern d=26: max deviation from the same-probe oracle trace {dev_same.max():.4f}; "
              f"iterations {[r.iters for r in recs]}", flush=True)
        assert dev_same.max() <= 0.10
        assert np.abs(gpu[-1] - 1.0).max() > 0.3          # the hyperparameters moved
        assert np.mean([r.iters for r in recs[5:]]) < recs[0].iters     # warm starts pay
    finally:
        opt.close()


def test_probe_laws_gaussian_and_rademacher_give_unbiased_gradients():
    """Section 2.1 allows Gaussian and Rademacher probes (any law with E[z z^T] = I); the laws differ in the
    fourth moment (3 against 1), which is what enters the spread of the trace estimate: z^T A z has
    variance 2 ||A||_F^2 for Gaussian probes and 2 (||A||_F^2 - sum_i A_ii^2) for Rademacher probes, so
    Rademacher is never worse and is much better where H^-1 dH/dtheta_k has a heavy diagonal (the signal
    and noise scales).  Measured on the GPU path: 40 draws of s = 8 probes per law, tight solves, gradient
    against the oracle's exact (Cholesky) gradient: both unbiased, spread ratio as the formula says."""
    from paper_2405_18328_amd.inputs import draw_probes
    w = make("config1", n=800)
    d, s, draws = w.d, 8, 40
    y = np.asarray(w.y, dtype=np.float64)
    exact = orc.mll_grad_exact(w.X, y, w.ell, w.a, w.sigma, w.kind)
    dv = _dev(w)
    try:
        stats = {}
        for law in ("gaussian", "rademacher"):
            rng = np.random.default_rng(77)
            errs = []
            for _ in range(draws):
                Z = draw_probes(rng, w.n, s, law)
                B = np.concatenate([np.asarray(w.y, dtype=np.float32)[:, None], Z.astype(np.float32)], axis=1)
                rc, _, _, _, Vd = dv.solve(B, 1e-5)
                assert rc == 0
                errs.append(dv.grad(Vd, dv.to(B)) - exact)
            errs = np.array(errs)
            stats[law] = (errs.mean(axis=0), errs.std(axis=0, ddof=1))
            bias, sd = stats[law]
            # unbiased: the mean error over the draws is within 4 standard errors, component by component
            assert (np.abs(bias) <= 4.0 * sd / np.sqrt(draws) + 1e-3 * np.abs(exact)).all(), (law, bias, sd)
        ratio = stats["rademacher"][1] / stats["gaussian"][1]
        print(f"[probes] spread ratio rademacher / gaussian per component: {np.round(ratio, 2)}", flush=True)
        # 40 draws fix a standard deviation to about 11 %: never worse beyond that noise, and clearly
        # better on the two scale components (observed 0.09 and 0.44)
        assert (ratio < 1.35).all() and (ratio[d:] < 0.7).all()
    finally:
        dv.close()


def test_cg_large_n_product_not_split_over_columns():
    """n = 70000: enough row blocks that the product inside the solver is not split over column ranges
    (the solver then reads H P straight from the product's output instead of summing partials).  Cold
    and warm solve, true residual on sampled rows from the oracle."""
    w = make("config3", n=70000, s=2)
    a, sigma = 1.0, 1.0
    dv = Dev(w.X, w.kind, w.ell, a, sigma)
    try:
        tol = 1e-3
        rc, it, kmv, rr, Vd = dv.solve(w.B, tol, max_iters=500)
        assert rc == 0 and kmv == it and (rr < tol).all()
        rows = np.sort(np.random.default_rng(3).choice(w.n, size=256, replace=False))
        B = np.asarray(w.B, dtype=np.float64)

        def sampled_rel(V):
            HV = orc.kmv_rows(w.X, w.ell, a, w.kind, V.astype(np.float64), rows, sigma=sigma)
            return np.linalg.norm(HV - B[rows], axis=0) * np.sqrt(w.n / rows.size) / np.linalg.norm(B, axis=0)

        rel = sampled_rel(Vd.cpu().numpy())
        print(f"[large-n cg] {it} iterations, sampled true relative residual {rel.max():.2e}", flush=True)
        assert rel.max() <= 2.0 * tol
        # warm start from the solution at slightly different hyperparameters: one extra product, fewer iterations
        dv.set_theta(np.asarray(w.ell) * 1.02, a, sigma)
        rc2, it2, kmv2, rr2, Vd2 = dv.solve(w.B, tol, max_iters=500, X0=Vd.clone())
        assert rc2 == 0 and kmv2 == it2 + 1 and it2 < it
    finally:
        dv.close()
