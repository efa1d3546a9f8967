"""Seeded synthetic regression workloads shaped like the paper's experiments.

This module only draws inputs.  It holds none of the method's arithmetic (no
kernel matrix, no solver, no gradient): targets are drawn with random Fourier
features of the kernel's spectral density, which needs only cosines of random
projections.  Both the HIP path and the CPU oracle consume what is generated
here; neither is imported.

The paper (Section 4, Appendix C) measures on five UCI regression sets with
n between 13.5k and 44k and d between 9 and 26; those are not reproduced.  The
workloads below have the same structure (dense real-valued inputs, a scalar
target, s probe vectors) at the sizes the benchmark contract names.

Everything is generated in float64 with numpy's default_rng(seed) and rounded
once to float32; the oracle upcasts those float32 values exactly.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

SE = "se"
MATERN32 = "matern32"


@dataclass
class Workload:
    name: str
    kind: str                 # "se" | "matern32"
    X: np.ndarray             # (n, d) float32
    y: np.ndarray             # (n,)  float32, centred, unit variance
    Z: np.ndarray             # (n, s) float32 probes
    ell: np.ndarray           # (d,) float64 lengthscales to start from
    a: float                  # signal scale (amplitude) to start from
    sigma: float              # noise scale to start from (H = K + sigma^2 I)
    tol: float                # relative-residual tolerance for every column
    ell_truth: np.ndarray = field(default=None)   # lengthscales that generated y
    probe_law: str = "gaussian"

    @property
    def n(self):
        return self.X.shape[0]

    @property
    def d(self):
        return self.X.shape[1]

    @property
    def s(self):
        return self.Z.shape[1]

    @property
    def B(self):
        """Right-hand sides [y, z_1..z_s], (n, s+1) float32."""
        return np.concatenate([self.y[:, None], self.Z], axis=1).astype(np.float32)


def draw_probes(rng, n, s, law):
    """s probe vectors of length n with E[z z^T] = I (Section 2.1)."""
    if law == "gaussian":
        return rng.standard_normal((n, s))
    if law == "rademacher":
        return rng.integers(0, 2, size=(n, s)).astype(np.float64) * 2.0 - 1.0
    raise ValueError(law)


def _rff_draw(rng, X, ell, a, sigma, kind, m=512, block=65536):
    """Approximate GP prior draw at X plus N(0, sigma^2) noise.

    f(x) = a sqrt(2/m) sum_i w_i cos(omega_i^T x + b_i) with w ~ N(0, I),
    b ~ U[0, 2pi] and omega drawn from the kernel's spectral density:
    Gaussian N(0, diag(1/ell^2)) for the squared exponential, multivariate
    Student-t with 3 degrees of freedom for Matern-3/2.
    """
    n, d = X.shape
    g = rng.standard_normal((m, d))
    if kind == MATERN32:
        u = rng.chisquare(3.0, size=(m, 1))
        g = g * np.sqrt(3.0 / u)
    omega = g / ell[None, :]
    phase = rng.uniform(0.0, 2.0 * np.pi, size=m)
    w = rng.standard_normal(m)
    f = np.empty(n)
    for r0 in range(0, n, block):
        r1 = min(r0 + block, n)
        f[r0:r1] = np.cos(X[r0:r1] @ omega.T + phase[None, :]) @ w
    f *= a * np.sqrt(2.0 / m)
    return f + sigma * rng.standard_normal(n)


def _standardise(v):
    v = v - v.mean(axis=0)
    sd = v.std(axis=0)
    return v / np.where(sd > 0, sd, 1.0)


def _finish(name, kind, X, y, Z, ell, a, sigma, tol, ell_truth, law):
    X32 = np.ascontiguousarray(X, dtype=np.float32)
    y32 = np.ascontiguousarray(_standardise(y), dtype=np.float32)
    Z32 = np.ascontiguousarray(Z, dtype=np.float32)
    return Workload(name, kind, X32, y32, Z32, np.asarray(ell, dtype=np.float64), float(a),
                    float(sigma), float(tol), np.asarray(ell_truth, dtype=np.float64), law)


def config1(n=2048, d=8, s=16, seed=1001):
    """Small SE-ARD case: X ~ N(0, I), ell = 1, a = 1, sigma^2 = 0.1, Rademacher probes."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, d))
    ell = np.ones(d)
    sigma = np.sqrt(0.1)
    y = _rff_draw(rng, X, ell, 1.0, sigma, SE)
    Z = draw_probes(rng, n, s, "rademacher")
    return _finish("config1", SE, X, y, Z, ell, 1.0, sigma, 1e-6, ell, "rademacher")


def config2(n=16384, d=26, s=64, seed=1002):
    """pol-shaped Matern-3/2 case: X ~ U[-1, 1]; y generated with lengthscales
    log-uniform in [0.3, 3] and sigma^2 = 0.05; optimisation starts at 1.0 for
    every hyperparameter, as in Section 4."""
    rng = np.random.default_rng(seed)
    X = rng.uniform(-1.0, 1.0, size=(n, d))
    ell_truth = 0.3 * 10.0 ** rng.uniform(0.0, 1.0, size=d)
    y = _rff_draw(rng, X, ell_truth, 1.0, np.sqrt(0.05), MATERN32)
    Z = draw_probes(rng, n, s, "gaussian")
    return _finish("config2", MATERN32, X, y, Z, np.ones(d), 1.0, 1.0, 0.01, ell_truth, "gaussian")


def config3(n=400000, d=3, s=64, seed=1003):
    """Low-d SE-ARD case: X from a 3-component Gaussian mixture, standardised;
    y = sum_k sin(w_k x_k + p_k) + N(0, 0.1^2); sigma^2 = 0.01."""
    rng = np.random.default_rng(seed)
    weights = np.array([0.5, 0.3, 0.2])
    means = 2.0 * rng.standard_normal((3, d))
    comp = rng.choice(3, size=n, p=weights)
    X = np.empty((n, d))
    for c in range(3):
        A = rng.standard_normal((d, d))
        cov_root = np.linalg.cholesky(A @ A.T / d + 0.25 * np.eye(d))
        idx = np.nonzero(comp == c)[0]
        X[idx] = means[c] + rng.standard_normal((idx.size, d)) @ cov_root.T
    X = _standardise(X)
    freq = rng.uniform(1.0, 3.0, size=d)
    phase = rng.uniform(0.0, 2.0 * np.pi, size=d)
    y = np.sin(X * freq[None, :] + phase[None, :]).sum(axis=1) + 0.1 * rng.standard_normal(n)
    Z = draw_probes(rng, n, s, "gaussian")
    ell = np.ones(d)
    return _finish("config3", SE, X, y, Z, ell, 1.0, 0.1, 0.01, ell, "gaussian")


def config4(n=500000, d=90, s=64, seed=1004, ell_value=None):
    """High-d Matern-3/2 case: X ~ N(0, I) standardised, sigma^2 = 0.5.

    ell_value = 1.0 is the literal configuration (r^2 ~ 2d, K is numerically the
    identity); ell_value = sqrt(d) gives r^2 = O(1).  Default: sqrt(d).
    """
    rng = np.random.default_rng(seed)
    X = _standardise(rng.standard_normal((n, d)))
    ell = np.full(d, np.sqrt(d) if ell_value is None else float(ell_value))
    sigma = np.sqrt(0.5)
    y = _rff_draw(rng, X, ell, 1.0, sigma, MATERN32)
    Z = draw_probes(rng, n, s, "gaussian")
    return _finish("config4", MATERN32, X, y, Z, ell, 1.0, sigma, 0.01, ell, "gaussian")


def config5(n=2000000, d=11, s=64, seed=1005):
    """Largest SE-ARD case: X ~ U[0, 1] with 5% of the rows overwritten by copies
    of other rows; ell = 1, a = 1, sigma^2 = 0.01."""
    rng = np.random.default_rng(seed)
    X = rng.uniform(0.0, 1.0, size=(n, d))
    ndup = n // 20
    dst = rng.choice(n, size=ndup, replace=False)
    keep = np.ones(n, dtype=bool)
    keep[dst] = False
    src = rng.choice(np.nonzero(keep)[0], size=ndup, replace=True)
    X[dst] = X[src]
    ell = np.ones(d)
    y = _rff_draw(rng, X, ell, 1.0, 0.1, SE)
    Z = draw_probes(rng, n, s, "gaussian")
    return _finish("config5", SE, X, y, Z, ell, 1.0, 0.1, 0.01, ell, "gaussian")


CONFIGS = {"config1": config1, "config2": config2, "config3": config3,
           "config4": config4, "config5": config5}


def make(name, **overrides):
    """Build a workload by name; n, d, s, seed can be overridden for scaled-down tests."""
    return CONFIGS[name](**overrides)
