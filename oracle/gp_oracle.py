"""fp64 CPU oracle for warm-started iterative GP marginal-likelihood optimisation.

TEST INFRASTRUCTURE ONLY.  This module is the slow, dense, obviously-correct
definition of what the GPU hot path computes.  Only tests, the smoke check and
the benchmark's cpu_baseline leg may import it; the product path never does,
and nothing here imports the product package or its HIP library.

Everything is NumPy/SciPy in float64.  Inputs that arrive as float32 are upcast
exactly, so input rounding is never charged as an error of either side.

Notation follows the paper (Section 2):
    theta = (ell_1..ell_d, a, sigma)      lengthscales, signal scale, noise scale
    K     = k(x, x; ell, a)               n x n kernel matrix
    H     = K + sigma^2 I                 coefficient matrix
    B     = [y, z_1..z_s]                 right-hand sides, column 0 is y
    V     = [v_y, v_1..v_s] = H^{-1} B    solutions

Readings where the paper is silent (it names the Matern-3/2 kernel with
per-dimension lengthscales and a scalar signal scale in Section 4, prints no
formula, and never mentions the squared exponential):
    r^2_ij   = sum_k (x_ik - x_jk)^2 / ell_k^2        by explicit differences
    SE-ARD   : K_ij = a^2 exp(-r^2_ij / 2)
    Matern32 : K_ij = a^2 (1 + sqrt(3) r_ij) exp(-sqrt(3) r_ij)
    the signal scale a is an amplitude (K is proportional to a^2);
    the noise parameter is sigma with H = K + sigma^2 I (Section 2);
    gradients are with respect to the constrained (ell, a, sigma).

Pin status: every function below is pinned by tests/test_oracle_pins.py against
something other than itself (scikit-learn / SciPy library routines, hand values,
closed forms, finite differences, brute force).  The only unpinned quantity is
the warm-vs-cold iteration *count* of the solvers (the paper gives it only as
stripped figures): "parity unpinned" for iteration numbers; the solutions
themselves are pinned.
"""
from __future__ import annotations

import numpy as np
import scipy.linalg as sla

SE = "se"
MATERN32 = "matern32"
_SQRT3 = np.sqrt(3.0)


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


# --------------------------------------------------------------------------
# Kernel matrix and its derivatives (Section 2: k(x, x; vartheta); Section 4
# names the Matern-3/2 ARD kernel with a scalar signal scale)
# --------------------------------------------------------------------------
def scaled_sqdist(Xa, Xb, ell):
    """r^2_ij = sum_k (xa_ik - xb_jk)^2 / ell_k^2 by explicit differences."""
    Xa, Xb, ell = _f64(Xa), _f64(Xb), _f64(ell)
    r2 = np.zeros((Xa.shape[0], Xb.shape[0]))
    for k in range(Xa.shape[1]):
        diff = (Xa[:, k][:, None] - Xb[:, k][None, :]) / ell[k]
        r2 += diff * diff
    return r2


def kernel_from_sqdist(r2, a, kind):
    if kind == SE:
        return a * a * np.exp(-0.5 * r2)
    if kind == MATERN32:
        r = np.sqrt(r2)
        return a * a * (1.0 + _SQRT3 * r) * np.exp(-_SQRT3 * r)
    raise ValueError(f"unknown kernel kind {kind!r}")


def kernel_cross(Xa, Xb, ell, a, kind):
    """k(Xa, Xb): pairwise evaluations, |Xa| x |Xb| (Section 2)."""
    return kernel_from_sqdist(scaled_sqdist(Xa, Xb, ell), float(a), kind)


def kernel_matrix(X, ell, a, kind):
    """K = k(x, x; vartheta), n x n (Section 2)."""
    return kernel_cross(X, X, ell, a, kind)


def coefficient_matrix(X, ell, a, sigma, kind):
    """H_theta = k(x, x) + sigma^2 I (Section 2)."""
    K = kernel_matrix(X, ell, a, kind)
    K[np.diag_indices_from(K)] += float(sigma) ** 2
    return K


def dK_dell(X, ell, a, kind, k):
    """dK/d ell_k, n x n.

    SE      : K_ij * D_ijk / ell_k^3                 with D_ijk = (x_ik - x_jk)^2
    Matern32: 3 a^2 exp(-sqrt(3) r_ij) D_ijk / ell_k^3
    (the Matern form has r cancelled, so coincident points give 0, not 0/0).
    """
    X, ell = _f64(X), _f64(ell)
    a = float(a)
    r2 = scaled_sqdist(X, X, ell)
    D = (X[:, k][:, None] - X[:, k][None, :]) ** 2
    if kind == SE:
        return a * a * np.exp(-0.5 * r2) * D / ell[k] ** 3
    if kind == MATERN32:
        return 3.0 * a * a * np.exp(-_SQRT3 * np.sqrt(r2)) * D / ell[k] ** 3
    raise ValueError(kind)


def dK_da(X, ell, a, kind):
    """dK/da = 2 K / a (K is proportional to a^2)."""
    return 2.0 * kernel_matrix(X, ell, a, kind) / float(a)


# --------------------------------------------------------------------------
# Dense products and Cholesky solves (Section 2, the tractable-n route)
# --------------------------------------------------------------------------
def kmv_dense(X, ell, a, kind, V, sigma=None):
    """K V, or (K + sigma^2 I) V when sigma is given.  Dense fp64 matmul."""
    V = _f64(V)
    out = kernel_matrix(X, ell, a, kind) @ V
    if sigma is not None:
        out = out + float(sigma) ** 2 * V
    return out


def kmv_rows(X, ell, a, kind, V, rows, sigma=None, col_block=32768):
    """Exact rows (K V)[rows, :] against all n columns, never forming K.

    For n too large for a dense K: O(len(rows) * n * (d + t)) work, column
    blocks bound the memory.  Same definition as kmv_dense.
    """
    X, V = _f64(X), _f64(V)
    rows = np.asarray(rows, dtype=np.int64)
    Xr = X[rows]
    out = np.zeros((rows.size, V.shape[1]))
    for c0 in range(0, X.shape[0], col_block):
        c1 = min(c0 + col_block, X.shape[0])
        out += kernel_cross(Xr, X[c0:c1], ell, a, kind) @ V[c0:c1]
    if sigma is not None:
        out += float(sigma) ** 2 * V[rows]
    return out


def cross_kmv(Xstar, X, ell, a, kind, V):
    """k(X*, X) V, m x t.  With V = v_y = H^{-1} y this is the posterior mean at the
    inputs X* (Section 2, Eq. 1); dense fp64, the definition."""
    return kernel_cross(_f64(Xstar), _f64(X), ell, a, kind) @ _f64(V)


def chol_solve(H, B):
    """V* = H^{-1} B via Cholesky and two triangular solves (Section 2)."""
    c, low = sla.cho_factor(_f64(H), lower=True)
    return sla.cho_solve((c, low), _f64(B))


# --------------------------------------------------------------------------
# Log marginal likelihood and its exact gradient (Section 2, the equations
# for L(theta) and grad L(theta))
# --------------------------------------------------------------------------
def mll(X, y, ell, a, sigma, kind):
    """L = -1/2 y^T H^{-1} y - 1/2 log det H - n/2 log 2 pi."""
    y = _f64(y).reshape(-1)
    H = coefficient_matrix(X, ell, a, sigma, kind)
    L = sla.cholesky(H, lower=True)
    w = sla.solve_triangular(L, y, lower=True)
    logdet = 2.0 * np.sum(np.log(np.diag(L)))
    return -0.5 * (w @ w) - 0.5 * logdet - 0.5 * y.size * np.log(2.0 * np.pi)


def dH_list(X, ell, a, sigma, kind):
    """Yield dH/d theta_k for theta = (ell_1..ell_d, a, sigma), each n x n."""
    X = _f64(X)
    n, d = X.shape
    for k in range(d):
        yield dK_dell(X, ell, a, kind, k)
    yield dK_da(X, ell, a, kind)
    yield 2.0 * float(sigma) * np.eye(n)


def mll_grad_exact(X, y, ell, a, sigma, kind):
    """grad L = 1/2 (H^{-1}y)^T dH (H^{-1}y) - 1/2 tr(H^{-1} dH), d+2 entries."""
    y = _f64(y).reshape(-1)
    H = coefficient_matrix(X, ell, a, sigma, kind)
    Hinv = chol_solve(H, np.eye(H.shape[0]))
    alpha = Hinv @ y
    g = []
    for dH in dH_list(X, ell, a, sigma, kind):
        g.append(0.5 * alpha @ (dH @ alpha) - 0.5 * np.sum(Hinv * dH))
    return np.array(g)


# --------------------------------------------------------------------------
# Hutchinson gradient estimator (Section 2.1, "Gradient Estimator" and
# "Linear System Solver": trace estimator substituted into grad L)
# --------------------------------------------------------------------------
def mll_grad_hutchinson(X, ell, a, sigma, kind, B, V=None):
    """Stochastic gradient with probes Z = B[:, 1:], y = B[:, 0].

    g_k = 1/2 v_y^T dH_k v_y - 1/(2s) sum_j v_j^T dH_k z_j
    using z_j^T H^{-1} dH_k z_j = v_j^T dH_k z_j (H symmetric), 1/s as in the
    trace-estimator equation.  V = H^{-1} B from Cholesky when not given; when
    given (for example an iterative solver's output) the same formula is
    evaluated at that V.
    """
    B = _f64(B)
    if V is None:
        V = chol_solve(coefficient_matrix(X, ell, a, sigma, kind), B)
    V = _f64(V)
    s = B.shape[1] - 1
    vy, Vz, Z = V[:, 0], V[:, 1:], B[:, 1:]
    g = []
    for dH in dH_list(X, ell, a, sigma, kind):
        quad = 0.5 * vy @ (dH @ vy)
        tr = 0.0
        if s > 0:
            tr = np.sum(Vz * (dH @ Z)) / s
        g.append(quad - 0.5 * tr)
    return np.array(g)


def mll_grad_hutchinson_rows(X, ell, a, sigma, kind, B, V, rows=None, row_block=256, workers=1):
    """The estimator of mll_grad_hutchinson at a given V, summed over rows i of the derivative matrices:

        g_k = sum_i [ 1/2 v_y,i (dH_k v_y)_i - 1/(2s) sum_j v_j,i (dH_k z_j)_i ]

    Rows i of every dH_k are formed a block at a time against all n columns and dropped again, so
    nothing n x n is ever held and n of several 10^4 fits in memory.  rows = None sums over all n rows
    (that is the estimator); an index array sums those rows' terms only, which is the whole estimator
    whenever V is zero outside them.  workers > 1 only spreads the row blocks over threads.
    """
    X, B, V, ell = _f64(X), _f64(B), _f64(V), _f64(ell)
    a, sigma = float(a), float(sigma)
    n, d = X.shape
    s = B.shape[1] - 1
    rows = np.arange(n) if rows is None else np.asarray(rows, dtype=np.int64)
    vy, Vz, Z = V[:, 0], V[:, 1:], B[:, 1:]

    def term(I, M):
        """The rows I of one derivative matrix (M = dH_k[I, :]) entered into both parts of g_k."""
        quad = 0.5 * vy[I] @ (M @ vy)
        tr = np.sum(Vz[I] * (M @ Z)) / s if s > 0 else 0.0
        return quad - 0.5 * tr

    def block(I):
        g = np.zeros(d + 2)
        r2 = scaled_sqdist(X[I], X, ell)
        if kind == SE:
            psi = a * a * np.exp(-0.5 * r2)
        elif kind == MATERN32:
            psi = 3.0 * a * a * np.exp(-_SQRT3 * np.sqrt(r2))
        else:
            raise ValueError(kind)
        for k in range(d):
            D = (X[I, k][:, None] - X[:, k][None, :]) ** 2
            g[k] = term(I, psi * D / ell[k] ** 3)                      # rows of dK/d ell_k, as in dK_dell
        g[d] = term(I, 2.0 * kernel_from_sqdist(r2, a, kind) / a)      # rows of dK/da
        E = np.zeros((I.size, n))
        E[np.arange(I.size), I] = 2.0 * sigma                          # rows of dH/dsigma = 2 sigma I
        g[d + 1] = term(I, E)
        return g

    blocks = [rows[i0:i0 + row_block] for i0 in range(0, rows.size, row_block)]
    if workers > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=workers) as ex:
            parts = list(ex.map(block, blocks))
    else:
        parts = [block(I) for I in blocks]
    return np.sum(parts, axis=0) if parts else np.zeros(d + 2)


# --------------------------------------------------------------------------
# Batched conjugate gradients, no preconditioner (Section 2.1 "Linear System
# Solver", Appendix B stopping rule)
# --------------------------------------------------------------------------
def cg_batched(matvec, B, X0=None, tol=0.01, max_iters=1000):
    """One independent Hestenes-Stiefel CG per column, run in lock step.

    matvec(P) returns H P for an n x t block.  Per column c the iteration stops
    ("freezes") once the recursively updated residual satisfies
    ||r_c|| / ||b_c|| < tol_c (strict); the solve ends when every column is
    frozen or after max_iters products.  A column with b_c = 0 has solution 0.

    Returns (V, iters, relres) with iters = number of matvecs inside the loop
    (the warm start's initial-residual product is not counted) and relres the
    final recursive relative residuals.
    """
    B = _f64(B)
    n, t = B.shape
    tol = np.broadcast_to(np.asarray(tol, dtype=np.float64), (t,)).copy()
    bnorm = np.sqrt(np.sum(B * B, axis=0))
    if X0 is None:
        X = np.zeros_like(B)
        R = B.copy()
    else:
        X = _f64(X0).copy()
        R = B - matvec(X)
    zero_rhs = bnorm == 0.0
    X[:, zero_rhs] = 0.0
    R[:, zero_rhs] = 0.0
    safe = np.where(zero_rhs, 1.0, bnorm)
    rho = np.sum(R * R, axis=0)
    relres = np.sqrt(rho) / safe
    frozen = zero_rhs | (relres < tol)
    P = R.copy()
    iters = 0
    while not frozen.all() and iters < max_iters:
        AP = matvec(P)
        iters += 1
        gamma = np.sum(P * AP, axis=0)
        live = ~frozen
        alpha = np.zeros(t)
        alpha[live] = rho[live] / gamma[live]
        X += alpha * P
        R -= alpha * AP
        rho_new = np.where(live, np.sum(R * R, axis=0), rho)
        relres = np.sqrt(rho_new) / safe
        beta = np.zeros(t)
        beta[live] = rho_new[live] / rho[live]
        rho = rho_new
        frozen = frozen | (relres < tol)
        P = R + beta * P
    return X, iters, relres


def dense_matvec(H):
    H = _f64(H)
    return lambda P: H @ P


# --------------------------------------------------------------------------
# Alternating projections as the linear system solver (Section 2.1 names it and
# cites Wu et al., 2024; Appendix B fixes the block size 2000 and the stopping
# rule; the steps below are that published method as read here:
#   - the n indices are cut into consecutive blocks of `block` indices (the last
#     one may be shorter);
#   - every step picks ONE block for the whole batch, the one whose residual
#     rows have the largest squared norm summed over the columns still being
#     updated (greedy rule), lowest index on a tie;
#   - the block's sub-system H[I,I] d = R[I,:] is solved exactly through the
#     Cholesky factor of H[I,I]; then V[I,:] += d and R -= H[:,I] d, so R stays
#     the residual B - H V and the quadratic objective of Section 2.1 is
#     minimised exactly over the coordinates I;
#   - a column stops being updated once ||r_c|| / ||b_c|| < tol_c (strict), as
#     in cg_batched; max_iters caps the number of block updates.)
# --------------------------------------------------------------------------
def ap_blocks(n, block):
    """[(start, stop)] of the consecutive index blocks."""
    return [(j, min(n, j + block)) for j in range(0, n, block)]


def ap_batched(H, B, X0=None, tol=0.01, block=2000, max_iters=10000):
    """Alternating projections on the dense coefficient matrix H (n x n).

    Returns (V, iters, relres, picks): iters = block updates done, relres = final
    relative residuals (R is updated, never recomputed, as in the method), picks =
    the block index chosen at every step.
    """
    H = _f64(H)
    B = _f64(B)
    n, t = B.shape
    tol = np.broadcast_to(np.asarray(tol, dtype=np.float64), (t,)).copy()
    blocks = ap_blocks(n, block)
    factors = [sla.cho_factor(H[j0:j1, j0:j1], lower=True) for (j0, j1) in blocks]
    bnorm = np.sqrt(np.sum(B * B, axis=0))
    if X0 is None:
        V = np.zeros_like(B)
        R = B.copy()
    else:
        V = _f64(X0).copy()
        R = B - H @ V
    zero_rhs = bnorm == 0.0
    V[:, zero_rhs] = 0.0
    R[:, zero_rhs] = 0.0
    safe = np.where(zero_rhs, 1.0, bnorm)
    relres = np.sqrt(np.sum(R * R, axis=0)) / safe
    frozen = zero_rhs | (relres < tol)
    iters = 0
    picks = []
    while not frozen.all() and iters < max_iters:
        live = ~frozen
        score = np.array([np.sum(R[j0:j1][:, live] ** 2) for (j0, j1) in blocks])
        k = int(np.argmax(score))
        j0, j1 = blocks[k]
        D = np.zeros((j1 - j0, t))
        D[:, live] = sla.cho_solve(factors[k], R[j0:j1][:, live])
        V[j0:j1] += D
        R -= H[:, j0:j1] @ D
        iters += 1
        picks.append(k)
        relres = np.where(live, np.sqrt(np.sum(R * R, axis=0)) / safe, relres)
        frozen = frozen | (relres < tol)
    return V, iters, relres, picks


# --------------------------------------------------------------------------
# Stochastic gradient descent as the linear system solver (Section 2.1 lists it,
# citing Lin et al.; Appendix B gives what is fixed: mini-batches of 1000 data
# points, momentum 0.9, no iterate averaging, a residual vector kept in memory
# and refreshed on the mini-batch rows only, "the gradient is equal to the
# residual").  The steps as read here, one recurrence per column, all columns
# sharing each mini-batch I (distinct row indices, given by the caller):
#   G      = H[I,:] U - B[I,:]        gradient of the quadratic of Section 2.1 on the rows I
#   R[I,:] = -G                       the residual estimate, refreshed on I only
#   M      = rho M ;  M[I,:] -= (lr / |I|) G        (momentum; lr / |I| is the step on a sampled row:
#   U     += M                         Appendix B's rates 20..100 with |I| = 1000 are steps of 0.02..0.1)
# Column c stops being updated (its momentum is dropped) once the ESTIMATED
# residual satisfies ||R_c|| / ||b_c|| < tol_c; the test is made after every step.
# --------------------------------------------------------------------------
def sgd_batched(H, B, batches, X0=None, tol=0.01, lr=50.0, momentum=0.9, max_iters=None):
    """batches: sequence of 1-D integer arrays (distinct indices each); step k uses batches[k].

    Returns (U, iters, relres_est): iters = steps done (at most len(batches) or max_iters),
    relres_est = the final estimated relative residuals.
    """
    H = _f64(H)
    B = _f64(B)
    n, t = B.shape
    tol = np.broadcast_to(np.asarray(tol, dtype=np.float64), (t,)).copy()
    bnorm = np.sqrt(np.sum(B * B, axis=0))
    if X0 is None:
        U = np.zeros_like(B)
        R = B.copy()
    else:
        U = _f64(X0).copy()
        R = B - H @ U
    zero_rhs = bnorm == 0.0
    U[:, zero_rhs] = 0.0
    R[:, zero_rhs] = 0.0
    safe = np.where(zero_rhs, 1.0, bnorm)
    relres = np.sqrt(np.sum(R * R, axis=0)) / safe
    frozen = zero_rhs | (relres < tol)
    M = np.zeros_like(B)
    limit = len(batches) if max_iters is None else min(max_iters, len(batches))
    iters = 0
    while not frozen.all() and iters < limit:
        I = np.asarray(batches[iters], dtype=np.int64)
        live = ~frozen
        G = H[I, :] @ U - B[I, :]
        R[np.ix_(I, live)] = -G[:, live]
        M[:, live] *= momentum
        M[np.ix_(I, live)] -= (lr / I.size) * G[:, live]
        M[:, frozen] = 0.0
        U += M
        iters += 1
        relres = np.where(live, np.sqrt(np.sum(R * R, axis=0)) / safe, relres)
        frozen = frozen | (relres < tol)
    return U, iters, relres


# --------------------------------------------------------------------------
# Positivity transform and Adam, as used by the outer loop (Section 4 and
# Appendix B: softplus constraints, Adam with learning rate 0.1)
# --------------------------------------------------------------------------
def softplus(raw):
    raw = _f64(raw)
    return np.logaddexp(0.0, raw)


def softplus_inverse(theta):
    theta = _f64(theta)
    return theta + np.log(-np.expm1(-theta))


def softplus_grad(raw):
    """d softplus(raw) / d raw = 1 / (1 + exp(-raw))."""
    raw = _f64(raw)
    return 1.0 / (1.0 + np.exp(-raw))


def adam_ascent(raw0, grad_fn, steps, lr=0.1, b1=0.9, b2=0.999, eps=1e-8):
    """Bias-corrected Adam maximising L over raw = softplus^{-1}(theta).

    grad_fn(theta) returns dL/dtheta (constrained); the chain rule through the
    softplus is applied here.  Returns the list of theta after every step.
    """
    raw = _f64(raw0).copy()
    m = np.zeros_like(raw)
    v = np.zeros_like(raw)
    trace = []
    for it in range(1, steps + 1):
        g = grad_fn(softplus(raw)) * softplus_grad(raw)
        m = b1 * m + (1 - b1) * g
        v = b2 * v + (1 - b2) * g * g
        raw = raw + lr * (m / (1 - b1 ** it)) / (np.sqrt(v / (1 - b2 ** it)) + eps)
        trace.append(softplus(raw))
    return trace
