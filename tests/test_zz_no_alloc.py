"""gp_kmv_static, the K V entry point for callers that cannot allocate: same results as gp_kmv.

Two calls in a row through the C ABI, the second on a smaller problem (the file-scope scratch then
still holds the first call's contents), each compared bit for bit with gp_kmv (same kernels, no
atomics on floats) and with the fp64 oracle at the 1e-5 normwise bar of the K V parity tests; a product
whose scratch would not fit is refused before anything is launched.  Collected last on purpose.
"""
import numpy as np
import pytest
import torch

from oracle import gp_oracle as orc
from paper_2405_18328_amd import binding as gp
from paper_2405_18328_amd.inputs import make
from tests.gpu_util import Dev, relerr

pytestmark = pytest.mark.gpu

KMV_TOL = 1e-5


def _both(dv, w, add_noise):
    """(gp_kmv_static output, gp_kmv output) on the workload's right-hand sides, padded leading dimensions."""
    t = w.s + 1
    ldv, ldo = t + 3, t + 2
    Vd = torch.full((w.n, ldv), float("nan"), device=dv.dev)
    Vd[:, :t] = dv.to(w.B)
    outs = []
    for fn in (gp.gp_kmv_static, gp.gp_kmv):
        out = torch.full((w.n, ldo), -777.0, device=dv.dev)
        print(f"[no-alloc] {fn.__name__} n={w.n} d={w.d} t={t} kind={w.kind}", flush=True)
        fn(dv.ctx, Vd, ldv, t, out, ldo, add_noise)
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        assert (o[:, t:] == -777.0).all(), "padding columns of the output were written"
        outs.append(o[:, :t])
    return outs


def test_static_scratch_product_equals_gp_kmv_twice_in_a_row_second_call_smaller():
    cases = [("config2", dict(n=6000, s=64)),     # Matern-3/2, d = 26, t = 65: column-split partials, two N-tiles + y column
             ("config1", dict(n=1500, s=16)),     # SE, d = 8, t = 17: smaller in every dimension than the call before
             ("config2", dict(n=6000, s=64))]     # and the larger one again over what the small one left
    for name, kw in cases:
        w = make(name, **kw)
        dv = Dev(w.X, w.kind, w.ell, w.a, w.sigma)
        try:
            got, ref_gpu = _both(dv, w, 1)
            assert np.array_equal(got, ref_gpu), "gp_kmv_static differs from gp_kmv"
            ref = orc.kmv_dense(w.X, w.ell, w.a, w.kind, w.B, sigma=w.sigma)
            assert relerr(got, ref) <= KMV_TOL
            # a second call on the same context, without the noise term, reusing the scratch at once
            got0, ref0 = _both(dv, w, 0)
            assert np.array_equal(got0, ref0)
            assert relerr(got0, orc.kmv_dense(w.X, w.ell, w.a, w.kind, w.B)) <= KMV_TOL
        finally:
            dv.close()


def test_static_scratch_product_on_every_product_path(monkeypatch):
    w = make("config3", n=3000, s=8)
    for path in ("fp32", "f16x2", "f16x3"):
        monkeypatch.setenv("GPWS_PATH", path)
        dv = Dev(w.X, w.kind, w.ell, w.a, w.sigma)
        try:
            got, ref_gpu = _both(dv, w, 1)
            assert np.array_equal(got, ref_gpu), path
            assert relerr(got, orc.kmv_dense(w.X, w.ell, w.a, w.kind, w.B, sigma=w.sigma)) <= KMV_TOL
        finally:
            dv.close()


def test_static_scratch_product_refuses_what_does_not_fit_and_bad_arguments():
    n, d, t = 300000, 3, 65      # the packed images of V alone take 77 MB here (256 bytes per row)
    X = torch.zeros((n, d), device="cuda:0")
    ctx = gp.gp_create(gp.GP_SE_ARD, n, d, X, torch.cuda.current_stream().cuda_stream)
    try:
        gp.gp_set_theta(ctx, np.ones(d), 1.0, 0.1)
        V = torch.zeros((n, t), device="cuda:0")
        out = torch.full((n, t), 5.0, device="cuda:0")
        with pytest.raises(gp.GpError) as e:
            gp.gp_kmv_static(ctx, V, t, t, out, t, 1)
        assert e.value.code == gp.GP_ERR_WORKSPACE and "static" in str(e.value)
        torch.cuda.synchronize()
        assert (out == 5.0).all(), "a refused call wrote its output"
        with pytest.raises(gp.GpError) as e:
            gp.gp_kmv_static(ctx, V, t, t, V, t, 0)
        assert e.value.code == gp.GP_ERR_ARG
        with pytest.raises(gp.GpError) as e:
            gp.gp_kmv_static(ctx, V, t - 1, t, out, t, 0)
        assert e.value.code == gp.GP_ERR_ARG
    finally:
        gp.gp_destroy(ctx)
