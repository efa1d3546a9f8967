"""GPU parity of the alternating-projections solver (gp_ap_solve) against the fp64 CPU oracle.

What is unique is compared tightly: the block chosen at every step (while the oracle's own margin
between the best and second-best block is wide enough that fp32 cannot flip it), the iterate after a
fixed number of steps, the stopping decision.  Tolerances:
  iterate after k steps   normwise relative error <= 2e-4 per column: the block solve multiplies the
                          residual by an fp32 copy of H[I,I]^-1, error ~ eps32 * kappa(H[I,I]) per step
                          (kappa <= 1 + block * a^2 / sigma^2, a few thousand in these cases);
  converged solve         tracked residual < tol (reported); the true residual recomputed in fp64 may exceed
                          it by the fp32 drift of the tracked residual, one rounding of size
                          ~eps32 |H[:,I] d| per step: <= tol * (1 + 1e-3) + 5e-7 * max(steps, 40);
  step counts             within 10% (or 2 steps) of the oracle's: after a near-tie flips a block choice
                          the two runs follow different but equally valid greedy paths.
"""
import numpy as np
import pytest

from oracle import gp_oracle as orc
from paper_2405_18328_amd.inputs import make
from tests.gpu_util import Dev

pytestmark = pytest.mark.gpu

STEP_TOL = 2e-4


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    yield


def _drift(steps):
    return 5e-7 * max(steps, 40)


def _colrel(got, ref):
    num = np.linalg.norm(got.astype(np.float64) - ref, axis=0)
    den = np.maximum(np.linalg.norm(ref, axis=0), 1e-300)
    return num / den


def _margin_ok(H, B, V, block, live, rel=1e-3):
    """True when the oracle's best block beats the runner-up by a relative margin fp32 cannot flip."""
    R = B - H @ V
    sc = np.array([np.sum(R[j0:j1][:, live] ** 2) for (j0, j1) in orc.ap_blocks(B.shape[0], block)])
    if len(sc) < 2:
        return True
    top = np.sort(sc)[::-1]
    return top[0] - top[1] > rel * top[0]


@pytest.mark.parametrize("name,kw,block", [
    ("config1", dict(n=300, s=4), 70),       # SE d=8: five blocks, the last one of 20 rows, blocks cut chunks of 32
    ("config2", dict(n=500, s=6), 96),       # Matern d=26, six blocks (last 20)
    ("config3", dict(n=450, s=2), 64),       # SE d=3, blocks aligned with the chunks
])
def test_ap_steps_match_oracle(name, kw, block):
    w = make(name, **kw)
    a, sigma = 1.1, 0.5
    H = orc.coefficient_matrix(w.X, w.ell, a, sigma, w.kind)
    B = np.asarray(w.B, dtype=np.float64)
    t = B.shape[1]
    rng = np.random.default_rng(5)
    X0 = (0.3 * rng.standard_normal(B.shape)).astype(np.float32)
    dv = Dev(w.X, w.kind, w.ell, a, sigma)
    try:
        for x0 in (None, X0):
            for k in (1, 2, 3, 5, 8):
                Vo, ito, rro, pko = orc.ap_batched(H, B, X0=x0, tol=1e-12, block=block, max_iters=k)
                assert ito == k
                # follow the oracle's own path to see where a choice could flip
                Vs = np.zeros_like(B) if x0 is None else x0.astype(np.float64)
                safe = True
                for step in range(k):
                    safe = safe and _margin_ok(H, B, Vs, block, np.ones(t, bool))
                    Vs, _, _, _ = orc.ap_batched(H, B, X0=Vs, tol=1e-12, block=block, max_iters=1)
                rc, it, kmv, rr, pk, Vd = dv.ap_solve(w.B, 1e-12, block, max_iters=k,
                                                      X0=None if x0 is None else dv.to(x0), picks=True)
                assert rc == 1 and it == k and kmv == (0 if x0 is None else 1)
                if not safe:
                    continue
                assert list(pk) == pko, (k, list(pk), pko)
                got = Vd.cpu().numpy()
                assert np.isfinite(got).all()
                assert (_colrel(got, Vo) <= STEP_TOL).all(), (k, _colrel(got, Vo))
                np.testing.assert_allclose(rr, rro, rtol=2e-3)
    finally:
        dv.close()


@pytest.mark.parametrize("name,kw,block", [
    ("config1", dict(n=700, s=8), 130),
    ("config2", dict(n=900, s=3), 200),
    ("config5", dict(n=1000, s=5), 96),      # duplicated rows: blocks with (numerically) repeated points
])
def test_ap_converged_solve_two_tolerances(name, kw, block):
    """Appendix B tolerances (0.01 for y, 0.1 for the probes), a zero right-hand side in the batch."""
    w = make(name, **kw)
    a, sigma = 1.0, 0.4
    H = orc.coefficient_matrix(w.X, w.ell, a, sigma, w.kind)
    B = np.asarray(w.B, dtype=np.float64).copy()
    B[:, -1] = 0.0
    t = B.shape[1]
    tol = np.array([0.01] + [0.1] * (t - 1))
    Vo, ito, rro, pko = orc.ap_batched(H, B, tol=tol, block=block, max_iters=100000)
    dv = Dev(w.X, w.kind, w.ell, a, sigma)
    try:
        rc, it, kmv, rr, pk, Vd = dv.ap_solve(B.astype(np.float32), tol, block, picks=True)
        got = Vd.cpu().numpy().astype(np.float64)
        assert rc == 0 and kmv == 0 and len(pk) == it
        assert (rr[:-1] < tol[:-1]).all() and rr[-1] == 0.0 and (got[:, -1] == 0.0).all()
        true_rel = np.linalg.norm(H @ got[:, :-1] - B[:, :-1], axis=0) / np.linalg.norm(B[:, :-1], axis=0)
        assert (true_rel <= tol[:-1] * 1.001 + _drift(it)).all(), (true_rel, it)
        assert abs(it - ito) <= max(2, 0.1 * ito), (it, ito)
        assert list(pk[:3]) == pko[:3]
        # every step picked a different block from the one before (its residual was just zeroed)
        assert all(pk[i] != pk[i + 1] for i in range(len(pk) - 1))
    finally:
        dv.close()


def test_ap_paper_block_size_and_warm_start():
    """Block size 2000 (Appendix B) on n = 4500: blocks of 2000, 2000 and 500 rows, 32 x 32 tiles of
    64 in the factorisation.  Then the warm start of Section 3: the solution at nearby
    hyperparameters as x0 needs fewer steps, and an x0 that already solves the system needs none."""
    w = make("config2", n=4500, s=3)
    a, sigma = 1.0, 0.5
    ell = np.asarray(w.ell_truth, dtype=np.float64)
    H = orc.coefficient_matrix(w.X, ell, a, sigma, w.kind)
    B = np.asarray(w.B, dtype=np.float64)
    tol = 1e-3
    Vo, ito, rro, pko = orc.ap_batched(H, B, tol=tol, block=2000, max_iters=5000)
    dv = Dev(w.X, w.kind, ell, a, sigma)
    try:
        rc, it, kmv, rr, pk, Vd = dv.ap_solve(w.B, tol, 2000, picks=True)
        got = Vd.cpu().numpy().astype(np.float64)
        assert rc == 0 and (rr < tol).all()
        true_rel = np.linalg.norm(H @ got - B, axis=0) / np.linalg.norm(B, axis=0)
        assert (true_rel <= tol * 1.001 + _drift(it)).all(), true_rel
        assert abs(it - ito) <= max(2, 0.1 * ito), (it, ito)
        assert list(pk[:2]) == pko[:2]
        # one step from a random start against the oracle: the 2000 x 2000 inverse at work
        rng = np.random.default_rng(8)
        X0 = (0.2 * rng.standard_normal(B.shape)).astype(np.float32)
        V1, _, _, p1 = orc.ap_batched(H, B, X0=X0, tol=1e-12, block=2000, max_iters=1)
        rc, it1, kmv1, _, pk1, Vd1 = dv.ap_solve(w.B, 1e-12, 2000, max_iters=1, X0=dv.to(X0), picks=True)
        assert rc == 1 and it1 == 1 and kmv1 == 1 and list(pk1) == p1
        assert (_colrel(Vd1.cpu().numpy(), V1) <= STEP_TOL).all()
        # warm start at slightly different hyperparameters
        ell2 = ell * 1.03
        H2 = orc.coefficient_matrix(w.X, ell2, a, sigma, w.kind)
        dv.set_theta(ell2, a, sigma)
        _, ito_cold, _, _ = orc.ap_batched(H2, B, tol=tol, block=2000, max_iters=5000)
        _, ito_warm, _, _ = orc.ap_batched(H2, B, X0=Vo, tol=tol, block=2000, max_iters=5000)
        rc, it_cold, _, _, _, _ = dv.ap_solve(w.B, tol, 2000)
        rc2, it_warm, kmvw, rrw, _, Vw = dv.ap_solve(w.B, tol, 2000, X0=Vd.clone())
        assert rc == 0 and rc2 == 0 and kmvw == 1
        assert it_warm < it_cold and ito_warm < ito_cold
        assert abs(it_warm - ito_warm) <= max(2, 0.1 * ito_warm) and abs(it_cold - ito_cold) <= max(2, 0.1 * ito_cold)
        gw = Vw.cpu().numpy().astype(np.float64)
        true_rel = np.linalg.norm(H2 @ gw - B, axis=0) / np.linalg.norm(B, axis=0)
        assert (true_rel <= tol * 1.001 + _drift(it_warm)).all()
        # x0 = the solution itself (in place): nothing to do
        Vs = dv.to(np.linalg.solve(H2, B))
        keep = Vs.clone()
        rc, it0, kmv0, rr0, _, Vout = dv.ap_solve(w.B, tol, 2000, X0=Vs, Vd=Vs)
        assert rc == 0 and it0 == 0 and kmv0 == 1 and (rr0 < tol).all()
        assert (Vout == keep).all()
    finally:
        dv.close()


@pytest.mark.parametrize("path", ["fp32", "f16x2", "f16x3"])
def test_ap_every_product_path(monkeypatch, path):
    monkeypatch.setenv("GPWS_PATH", path)
    w = make("config5", n=800, s=4)
    a, sigma = 0.9, 0.3
    H = orc.coefficient_matrix(w.X, w.ell, a, sigma, w.kind)
    B = np.asarray(w.B, dtype=np.float64)
    dv = Dev(w.X, w.kind, w.ell, a, sigma)
    try:
        V3, _, _, p3 = orc.ap_batched(H, B, tol=1e-12, block=150, max_iters=3)
        rc, it, _, _, pk, Vd = dv.ap_solve(w.B, 1e-12, 150, max_iters=3, picks=True)
        assert rc == 1 and it == 3 and list(pk) == p3
        assert (_colrel(Vd.cpu().numpy(), V3) <= STEP_TOL).all()
        rc, it, _, rr, _, Vd = dv.ap_solve(w.B, 0.01, 150)
        got = Vd.cpu().numpy().astype(np.float64)
        true_rel = np.linalg.norm(H @ got - B, axis=0) / np.linalg.norm(B, axis=0)
        assert rc == 0 and (true_rel <= 0.01 * 1.001 + _drift(it)).all(), (true_rel, it)
    finally:
        dv.close()


def test_ap_one_block_is_a_direct_solve_and_extreme_shapes():
    w = make("config1", n=150, s=2)
    a, sigma = 1.2, 0.7
    H = orc.coefficient_matrix(w.X, w.ell, a, sigma, w.kind)
    B = np.asarray(w.B, dtype=np.float64)
    dv = Dev(w.X, w.kind, w.ell, a, sigma)
    try:
        # the largest block size with a block that is mostly padding
        rc, it, _, rr, pk, Vd = dv.ap_solve(w.B, 1e-4, 2048, picks=True)
        assert rc == 0 and it == 1 and list(pk) == [0]
        assert (_colrel(Vd.cpu().numpy(), np.linalg.solve(H, B)) <= 1e-4).all()
        # blocks of one row: greedy coordinate descent, many tiny steps
        Vo, ito, _, pko = orc.ap_batched(H, B, tol=1e-12, block=1, max_iters=40)
        rc, it, _, _, pk, Vd = dv.ap_solve(w.B, 1e-12, 1, max_iters=40, picks=True)
        assert rc == 1 and it == 40
        same = 0
        while same < 40 and pk[same] == pko[same]:
            same += 1
        assert same >= 10, (list(pk), pko)         # scalar residuals tie more easily than block norms
        if same == 40:
            assert (_colrel(Vd.cpu().numpy(), Vo) <= STEP_TOL).all()
        # max_iters = 0 returns the start
        rc, it, _, rr, _, Vd = dv.ap_solve(w.B, 1e-3, 64, max_iters=0)
        assert rc == 1 and it == 0 and (Vd.cpu().numpy() == 0).all() and np.allclose(rr, 1.0)
    finally:
        dv.close()
    # n = 1, t = 1
    X = np.array([[0.3, -0.2]], dtype=np.float32)
    dv = Dev(X, "se", np.array([1.0, 2.0]), 1.5, 0.5)
    try:
        rc, it, _, rr, _, Vd = dv.ap_solve(np.array([[2.0]], dtype=np.float32), 1e-5, 2000)
        assert rc == 0 and it == 1
        assert abs(float(Vd.cpu().numpy()[0, 0]) - 2.0 / (1.5 ** 2 + 0.25)) < 1e-6
    finally:
        dv.close()


def test_ap_argument_errors():
    import torch
    w = make("config1", n=200, s=2)
    dv = Dev(w.X, w.kind, w.ell, 1.0, 0.5)
    gp = dv.gp
    try:
        Bd = dv.to(w.B)
        Vd = torch.zeros_like(Bd)
        t = Bd.shape[1]
        assert gp.gp_ap_workspace_bytes(dv.ctx, t, 0) == 0 and gp.gp_ap_workspace_bytes(dv.ctx, t, 2049) == 0
        need = gp.gp_ap_workspace_bytes(dv.ctx, t, 64)
        assert need > 0
        wk = torch.empty(need + 256, dtype=torch.uint8, device=dv.dev)
        for bad_block in (0, -3, 2049):
            with pytest.raises(gp.GpError) as e:
                gp.gp_ap_solve(dv.ctx, Bd, t, None, Vd, t, t, 0.01, bad_block, 10, wk, wk.numel())
            assert e.value.code == -1
        with pytest.raises(gp.GpError) as e:
            gp.gp_ap_solve(dv.ctx, Bd, t, None, Vd, t, t, 0.01, 64, 10, wk, need - 1)
        assert e.value.code == -3
        with pytest.raises(gp.GpError) as e:
            gp.gp_ap_solve(dv.ctx, Bd, t, None, Vd, t, t, 0.01, 64, 10, wk[16:], need)
        assert e.value.code == -3
        with pytest.raises(gp.GpError) as e:
            gp.gp_ap_solve(dv.ctx, Bd, t, None, Vd, t, t, -1.0, 64, 10, wk, wk.numel())
        assert e.value.code == -1
        with pytest.raises(gp.GpError) as e:
            gp.gp_ap_solve(dv.ctx, Bd, t, None, Vd, t, t, 0.01, 64, -1, wk, wk.numel())
        assert e.value.code == -1
        # the context still works afterwards
        rc, it, _, rr, _ = gp.gp_ap_solve(dv.ctx, Bd, t, None, Vd, t, t, 0.05, 64, 1000, wk, wk.numel())
        assert rc == 0 and (rr < 0.05).all()
    finally:
        dv.close()


def test_ap_many_columns_and_padded_leading_dimensions():
    """t = 300 (more than one pass of 256 columns in the block solve and of the streaming kernels) with
    leading dimensions larger than t for B, x0 and V; the padding columns of V must not be written."""
    import torch
    w = make("config3", n=420, s=4)
    a, sigma = 1.0, 0.5
    t, block = 300, 128
    rng = np.random.default_rng(3)
    B = rng.standard_normal((w.n, t))
    X0 = 0.2 * rng.standard_normal((w.n, t))
    H = orc.coefficient_matrix(w.X, w.ell, a, sigma, w.kind)
    dv = Dev(w.X, w.kind, w.ell, a, sigma)
    gp = dv.gp
    try:
        ldb, ldv = t + 5, t + 9
        Bd = torch.full((w.n, ldb), 7.0, device=dv.dev)
        Bd[:, :t] = dv.to(B)
        Vd = torch.full((w.n, ldv), -777.0, device=dv.dev)
        Vd[:, :t] = dv.to(X0)
        need = gp.gp_ap_workspace_bytes(dv.ctx, t, block)
        wk = torch.empty(need, dtype=torch.uint8, device=dv.dev)
        Bf, X0f = B.astype(np.float32).astype(np.float64), X0.astype(np.float32).astype(np.float64)
        for k in (1, 4):
            Vd[:, :t] = dv.to(X0)
            Vo, _, rro, pko = orc.ap_batched(H, Bf, X0=X0f, tol=1e-12, block=block, max_iters=k)
            rc, it, kmv, rr, pk = gp.gp_ap_solve(dv.ctx, Bd, ldb, Vd, Vd, ldv, t, 1e-12, block, k, wk, wk.numel(),
                                                 want_picks=True)
            assert rc == 1 and it == k and kmv == 1 and list(pk) == pko
            got = Vd.cpu().numpy()
            assert (got[:, t:] == -777.0).all()
            assert (_colrel(got[:, :t], Vo) <= STEP_TOL).all()
            np.testing.assert_allclose(rr, rro, rtol=2e-3)
    finally:
        dv.close()


def test_ap_random_small_shapes():
    """Twelve seeded combinations of n, d, t, block size and kernel (odd sizes, blocks that cut chunks of 32,
    a last block of a single row, t = 1): three steps against the oracle."""
    rng = np.random.default_rng(2024)
    for case in range(12):
        n = int(rng.integers(33, 700))
        d = int(rng.integers(1, 20))
        t = int(rng.integers(1, 40))
        block = int(rng.integers(1, 300)) if case else n - 1          # case 0: last block is one row
        kind = "se" if case % 2 else "matern32"
        X = rng.standard_normal((n, d)).astype(np.float32)
        ell = rng.uniform(0.8, 2.5, size=d) * np.sqrt(d)
        a, sigma = float(rng.uniform(0.5, 1.5)), float(rng.uniform(0.3, 1.0))
        B = rng.standard_normal((n, t)).astype(np.float32)
        print(f"[ap-shape] case {case}: n={n} d={d} t={t} block={block} {kind}", flush=True)
        H = orc.coefficient_matrix(X, ell, a, sigma, kind)
        Bf = B.astype(np.float64)
        dv = Dev(X, kind, ell, a, sigma)
        try:
            k = 3
            Vo, ito, rro, pko = orc.ap_batched(H, Bf, tol=1e-12, block=block, max_iters=k)
            Vs, safe = np.zeros_like(Bf), True
            for _ in range(ito):
                safe = safe and _margin_ok(H, Bf, Vs, block, np.ones(t, bool))
                Vs, _, _, _ = orc.ap_batched(H, Bf, X0=Vs, tol=1e-12, block=block, max_iters=1)
            # a single block solves the system in one step: fp64 then meets even this tolerance and stops,
            # fp32 cannot, so the library is held to the oracle's number of steps
            rc, it, _, rr, pk, Vd = dv.ap_solve(B, 1e-12, block, max_iters=ito, picks=True)
            assert it == ito
            if safe:
                assert list(pk) == pko
                assert (_colrel(Vd.cpu().numpy(), Vo) <= STEP_TOL).all(), case
                np.testing.assert_allclose(rr, rro, rtol=2e-3, atol=2e-5)   # a single-block solve leaves an fp32 rounding-level residual
        finally:
            dv.close()


def test_ap_shapes_at_the_solve_kernels_tile_boundaries():
    """Right-hand-side counts around the block solve's 64-column workgroups and 4-column lanes (63..66, 128,
    129), block sizes around its 16-row tiles and the factorisation's 64-row tiles (16, 17, 127..129, 500),
    and the largest blocks the library takes (2047, 2048): three steps against the oracle."""
    rng = np.random.default_rng(77)
    cases = [(300, 63, 100), (300, 64, 128), (300, 65, 129), (300, 66, 16), (300, 128, 17), (260, 129, 127),
             (1100, 65, 500), (4200, 65, 2047), (4300, 9, 2048)]
    for case, (n, t, block) in enumerate(cases):
        d = 5
        kind = "se" if case % 2 else "matern32"
        X = rng.standard_normal((n, d)).astype(np.float32)
        ell = rng.uniform(0.8, 2.5, size=d) * np.sqrt(d)
        a, sigma = float(rng.uniform(0.5, 1.5)), float(rng.uniform(0.4, 1.0))
        # rows growing in size keep the blocks' residual norms apart, so that the greedy order is unambiguous
        B = (rng.standard_normal((n, t)) * (1.0 + np.arange(n)[:, None] / n)).astype(np.float32)
        print(f"[ap-shape] case {case}: n={n} t={t} block={block} {kind}", flush=True)
        H = orc.coefficient_matrix(X, ell, a, sigma, kind)
        Bf = B.astype(np.float64)
        dv = Dev(X, kind, ell, a, sigma)
        try:
            k = 3
            Vo, ito, rro, pko = orc.ap_batched(H, Bf, tol=1e-12, block=block, max_iters=k)
            Vs, safe = np.zeros_like(Bf), True
            for _ in range(ito):
                safe = safe and _margin_ok(H, Bf, Vs, block, np.ones(t, bool))
                Vs, _, _, _ = orc.ap_batched(H, Bf, X0=Vs, tol=1e-12, block=block, max_iters=1)
            rc, it, _, rr, pk, Vd = dv.ap_solve(B, 1e-12, block, max_iters=ito, picks=True)
            assert it == ito
            if safe:
                assert list(pk) == pko
                assert (_colrel(Vd.cpu().numpy(), Vo) <= STEP_TOL).all(), (case, _colrel(Vd.cpu().numpy(), Vo).max())
                np.testing.assert_allclose(rr, rro, rtol=2e-3, atol=2e-5)
            else:
                print(f"[ap-shape] case {case}: block margins too narrow for a step-by-step comparison", flush=True)
        finally:
            dv.close()
