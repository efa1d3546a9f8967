/*
 * gpws.h -- C ABI of libgpws: the hot path of warm-started marginal-likelihood
 * optimisation for iterative Gaussian processes on one AMD MI355X (gfx950).
 *
 * The path (paper Section 2.1): a first-order optimiser needs estimates of the
 * gradient of the log marginal likelihood; the estimate needs
 * H^{-1}[y, z_1..z_s] for H = k(x,x) + sigma^2 I; an iterative solver (conjugate
 * gradients, alternating projections or stochastic gradient descent, the three
 * the paper runs) obtains it from products with H or with blocks of its rows or
 * columns, all evaluated matrix-free (K is never stored).  The warm start
 * (Section 3) passes the previous outer step's solution as x0.
 *
 * Conventions
 *   - Every pointer named d* is DEVICE memory owned by the caller; every
 *     pointer named h* is HOST memory owned by the caller.  The library owns
 *     only what lives inside gp_ctx and frees it in gp_destroy.
 *   - Matrices are row-major fp32: element (i, c) of an n x t block is
 *     p[i*ld + c], ld >= t.  Column 0 of a right-hand-side block is y, columns
 *     1..s are the probes z_j; t = s + 1.
 *   - All work is enqueued on the HIP stream given to gp_create.  Calls that
 *     return host results (the solvers, gp_mll_grad) synchronise that stream
 *     before returning; gp_set_theta waits for earlier work on the stream and
 *     may synchronise once more (see there); gp_kmv is asynchronous.
 *   - theta = (ell_1..ell_d, a, sigma): lengthscales, signal scale (amplitude,
 *     K is proportional to a^2), noise scale (H = K + sigma^2 I).
 *   - No call aborts or throws.  Return value: 0 = GP_OK, > 0 = result usable
 *     but a condition is flagged, < 0 = error (nothing useful was written);
 *     gp_last_error gives the text.  Arguments are validated before any launch.
 *   - One context must not be used from two host threads at once.
 */
#ifndef GPWS_H
#define GPWS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gp_ctx gp_ctx;

enum { GP_SE_ARD = 0, GP_MATERN32_ARD = 1 };

enum {
  GP_OK = 0,
  GP_NOT_CONVERGED = 1,   /* max_iters reached before every column met its tolerance */
  GP_ERR_ARG = -1,        /* NULL pointer, bad size, bad leading dimension, theta not set */
  GP_ERR_HIP = -2,        /* a HIP runtime call failed */
  GP_ERR_WORKSPACE = -3,  /* dWork too small or misaligned */
  GP_ERR_BREAKDOWN = -4   /* CG met p^T H p <= 0 or a non-finite value */
};

/* Largest input dimension and right-hand-side count the kernels are built for. */
#define GP_MAX_D 126
#define GP_MAX_T 1024

/*
 * Create a context for n training inputs of dimension d (paper Section 2: the
 * inputs x of the regression model).  dX: device, row-major n x d fp32; it is
 * read at every gp_set_theta and must stay valid and unchanged until
 * gp_destroy.  hip_stream: a hipStream_t (NULL = the default stream).
 * kernel: GP_SE_ARD      k = a^2 exp(-r^2/2)
 *         GP_MATERN32_ARD k = a^2 (1 + sqrt(3) r) exp(-sqrt(3) r)
 *         with r^2 = sum_k (x_ik - x_jk)^2 / ell_k^2  (Section 4 names the
 *         Matern-3/2 kernel with per-dimension lengthscales and a scalar
 *         signal scale; the formulas are the standard ones).
 * Errors: GP_ERR_ARG for n < 1, d < 1, d > GP_MAX_D, unknown kernel, NULL
 * pointers; GP_ERR_HIP if device allocation fails.
 */
int gp_create(gp_ctx** out, int kernel, int64_t n, int d, const float* dX, void* hip_stream);

/* Free everything the context owns.  NULL is accepted. */
int gp_destroy(gp_ctx* ctx);

/*
 * Set the hyperparameters theta (Section 2: theta = {vartheta, sigma}).
 * h_lengthscale: d positive doubles; signal_scale > 0; noise_scale >= 0.
 * Rebuilds the scaled copies of the inputs the tile kernels read (O(n d) device
 * work) and chooses the arithmetic of the tile pass (see gp_product_path) from
 * the largest scaled squared norm.  Waits for earlier work on the stream (a
 * pinned staging block is reused); the packing itself is left running unless
 * the norm has to be read back, which happens only when a bound kept on the
 * host does not already settle the choice.  Must be called before any of the
 * calls below.  Errors: GP_ERR_ARG for non-positive or non-finite values, or
 * inputs that are not finite after scaling.
 */
int gp_set_theta(gp_ctx* ctx, const double* h_lengthscale, double signal_scale, double noise_scale);

/*
 * OUT = K V (add_noise = 0) or (K + sigma^2 I) V (add_noise = 1): the
 * matrix-free product at the heart of every solver iteration (Section 2.1,
 * "Linear System Solver").  dV: n x t, leading dimension ldv; dOut: n x t,
 * leading dimension ldo; the byte ranges of dOut and dV must not overlap
 * (GP_ERR_ARG otherwise).  1 <= t <= GP_MAX_T.
 * Asynchronous on the context's stream, except that the first call, and any call
 * that needs more scratch than an earlier one (larger t), waits for the stream
 * and reallocates the context's scratch block with hipMalloc.
 */
int gp_kmv(gp_ctx* ctx, const float* dV, int64_t ldv, int t, float* dOut, int64_t ldo, int add_noise);

/*
 * gp_kmv for callers that cannot allocate: code between hipStreamBeginCapture and
 * hipStreamEndCapture, serving loops that must never reach hipMalloc, harnesses that forbid it.
 * Same arguments, same kernels and bit-identical results as gp_kmv, but the scratch of the product
 * (column maxima, the packed images of V, column-split partial sums) is a file-scope device array
 * of GP_KMV_STATIC_SCRATCH_BYTES bytes that every GPU the library is used on holds until the
 * process ends, and the call reaches no hipMalloc, hipFree, stream synchronisation or memset
 * command.  A product whose scratch does not fit (256 bytes per row for the packed images of V,
 * plus n t floats per column split, of which there are up to 64 when n is small: n = 16384, t = 65
 * needs 39 MB, n = 200000 needs 52 MB, n = 300000 does not fit) is refused with GP_ERR_WORKSPACE
 * and nothing is launched: use gp_kmv for it.
 * All calls on one GPU, from any context, share that GPU's array: two such calls must not be in
 * flight on one GPU at the same time (calls on one stream are ordered and safe; calls on different
 * streams race).  Nothing in it needs to survive between calls; what must start at zero is cleared
 * by the call itself.
 */
#define GP_KMV_STATIC_SCRATCH_BYTES (64u << 20)
int gp_kmv_static(gp_ctx* ctx, const float* dV, int64_t ldv, int t, float* dOut, int64_t ldo, int add_noise);

/* Bytes of device workspace gp_cg_solve needs for t right-hand sides (0 on bad arguments). */
size_t gp_workspace_bytes(const gp_ctx* ctx, int t);

/*
 * Solve H [v_y, v_1..v_s] = [y, z_1..z_s] (the batched system of Section 2.1)
 * by conjugate gradients without a preconditioner (Appendix B), one
 * Hestenes-Stiefel recurrence per column run in lock step so that all columns
 * share each product H P.
 *   dB   : n x t right-hand sides (ldb).
 *   dX0  : n x t initial guess (same leading dimension ldv as dV) or NULL for
 *          zeros.  Passing the previous outer step's solution is the warm start
 *          of Section 3.  dX0 may be the same pointer as dV.
 *   dV   : n x t solution out (ldv).
 *   h_tol: t relative-residual tolerances; column c stops being updated once
 *          its recursively updated residual satisfies ||r_c|| / ||b_c|| < tol_c
 *          (Appendix B: 0.01 for the y system, 0.1 for the probe systems).
 *          A column with b_c = 0 gets the solution 0.
 *   max_iters >= 0: cap on the products inside the loop.
 *   dWork/work_bytes: device scratch, at least gp_workspace_bytes(ctx, t),
 *          256-byte aligned.  Nothing of size n x t is allocated by the call.
 *   h_iters     : out, products H P done inside the loop.
 *   h_kmv_count : out, all products including the warm start's initial residual.
 *   h_relres    : out, t final recursive relative residuals.
 * Returns GP_OK, GP_NOT_CONVERGED (dV holds the last iterate), or an error.
 * Synchronises the stream.
 */
int gp_cg_solve(gp_ctx* ctx, const float* dB, int64_t ldb, const float* dX0, float* dV, int64_t ldv,
                int t, const float* h_tol, int max_iters, void* dWork, size_t work_bytes,
                int* h_iters, int* h_kmv_count, float* h_relres);

/*
 * The same batched system solved by alternating projections (Section 2.1 names the method and cites
 * Wu et al., 2024; Appendix B: block size 2000, the same stopping rule as for conjugate gradients).
 * The n indices are cut into consecutive blocks of `block` indices (the last may be shorter).  Each
 * step picks, for the whole batch, the block whose residual rows have the largest squared norm over
 * the columns still being updated (lowest index on a tie), solves that block's sub-system
 * H[I,I] d = R[I,:] exactly, adds d to V[I,:] and subtracts H[:,I] d from the residual, which is
 * therefore tracked, never recomputed.  Column c is no longer updated once
 * ||r_c|| / ||b_c|| < tol_c; a column with b_c = 0 gets the solution 0.
 *   dB, dX0, dV, ldb, ldv, t, h_tol, h_relres: as for gp_cg_solve (dX0 != NULL is the warm start of
 *          Section 3 and costs one full product for the initial residual).
 *   block : 1 .. GP_AP_MAX_BLOCK.
 *   max_iters >= 0: cap on the number of block updates.
 *   dWork/work_bytes: device scratch, at least gp_ap_workspace_bytes(ctx, t, block), 256-byte
 *          aligned.  It holds, besides the solver's vectors, the inverse of every diagonal block
 *          (about 4 * n * block bytes), rebuilt by every call for the current theta.
 *   h_iters     : out, block updates done.
 *   h_kmv_count : out, full n x n products done (0, or 1 for a warm start).
 *   h_picks     : out or NULL, max_iters ints: the block index chosen at every step.
 * Returns GP_OK, GP_NOT_CONVERGED (dV holds the last iterate), GP_ERR_BREAKDOWN when a diagonal
 * block is not numerically positive definite, or an argument/workspace/HIP error.
 * Synchronises the stream.
 */
#define GP_AP_MAX_BLOCK 2048
size_t gp_ap_workspace_bytes(const gp_ctx* ctx, int t, int block);
int gp_ap_solve(gp_ctx* ctx, const float* dB, int64_t ldb, const float* dX0, float* dV, int64_t ldv,
                int t, const float* h_tol, int block, int max_iters, void* dWork, size_t work_bytes,
                int* h_iters, int* h_kmv_count, float* h_relres, int* h_picks);

/*
 * The same batched system solved by stochastic gradient descent on the quadratic objective of
 * Section 2.1 (the paper lists the solver, citing Lin et al.; Appendix B: mini-batches of 1000 data
 * points, momentum 0.9, no iterate averaging, a residual vector kept in memory and refreshed on the
 * mini-batch rows only).  Step k, with I = the k-th mini-batch, for all t columns at once:
 *   G = H[I,:] U - B[I,:];  R[I,:] = -G;  M = momentum * M;  M[I,:] -= (lr / batch) * G;  U += M.
 * Column c is no longer updated once the ESTIMATED residual satisfies ||R_c|| / ||b_c|| < tol_c (the
 * test is made after every step); a column with b_c = 0 gets the solution 0.  R starts as the true
 * residual (B, or B - H x0 for a warm start, which costs one full product).
 *   dB, dX0, dV, ldb, ldv, t, h_tol, h_relres, h_kmv_count: as for gp_cg_solve; h_relres are the
 *          estimated relative residuals.
 *   dBatches: device, max_iters x batch int32, row k = the indices of mini-batch k, each in [0, n) and
 *          distinct within a row (not checked: repeated indices lose updates; an index outside
 *          [0, n) is never dereferenced and makes the call return GP_ERR_ARG).  The library draws no
 *          random numbers.
 *   batch : 1 .. min(n, GP_SGD_MAX_BATCH).   lr > 0: the step on a sampled row is lr / batch
 *          (Appendix B's rates are 20 .. 100 with batch 1000).   0 <= momentum < 1.
 *   max_iters >= 0: cap on the number of steps.   h_iters: out, steps done.
 *   dWork/work_bytes: device scratch, at least gp_sgd_workspace_bytes(ctx, t, batch), 256-byte aligned.
 * Returns GP_OK, GP_NOT_CONVERGED (dV holds the last iterate), GP_ERR_BREAKDOWN when the residual
 * estimate stops being finite (learning rate too large), or an argument/workspace/HIP error.
 * Synchronises the stream.
 */
#define GP_SGD_MAX_BATCH 65536
size_t gp_sgd_workspace_bytes(const gp_ctx* ctx, int t, int batch);
int gp_sgd_solve(gp_ctx* ctx, const float* dB, int64_t ldb, const float* dX0, float* dV, int64_t ldv,
                 int t, const float* h_tol, const int32_t* dBatches, int batch, int max_iters, double lr,
                 double momentum, void* dWork, size_t work_bytes, int* h_iters, int* h_kmv_count,
                 float* h_relres);

/*
 * Stochastic estimate of the gradient of the log marginal likelihood (Section 2
 * gradient equation with the trace replaced by the s-probe estimator of
 * Section 2.1, normalised by 1/s):
 *   g_k = 1/2 v_y^T (dH/dtheta_k) v_y - 1/(2s) sum_j v_j^T (dH/dtheta_k) z_j
 * evaluated matrix-free in one tile pass over all pairs (i, j).
 *   dV: n x t solutions [v_y, v_1..v_s] (ldv); dB: n x t [y, z_1..z_s] (ldb);
 *   t = s + 1 >= 1 (s = 0 leaves only the quadratic term).
 *   h_grad: out, d + 2 doubles: dL/d ell_1..ell_d, dL/da, dL/dsigma, with
 *   respect to the constrained parameters (a softplus chain rule is the caller's).
 * Synchronises the stream.
 */
int gp_mll_grad(gp_ctx* ctx, const float* dV, int64_t ldv, const float* dB, int64_t ldb, int t,
                double* h_grad);

/*
 * Cross-covariance product OUT = K(X*, X) V between m other inputs X* and the context's n
 * inputs, for the current theta, matrix-free with the same tile pass as gp_kmv (Section 2,
 * Eq. 1: with V = v_y = H^{-1} y, t = 1, this is the posterior mean at X*; with the columns
 * of a solved batch it gives the data-dependent term of each posterior sample).
 *   dXstar: device, m x d row-major fp32, 1 <= m <= 2^30; read during the call only.
 *   dV: device, n x t, leading dimension ldv >= t.  dOut: device, m x t, ldo >= t; written.
 * No noise term is added.  Synchronises the stream once (to read the largest scaled norm of
 * X*, which together with the training inputs' selects the arithmetic of the product).
 */
int gp_predict(gp_ctx* ctx, const float* dXstar, int64_t m, const float* dV, int64_t ldv, int t, float* dOut,
               int64_t ldo);

/*
 * Instrumentation for roofline reports (not part of the method): while enabled, every launch of
 * the chosen kinds of kernel made through this context is bracketed by a pair of HIP events on the
 * context's stream.  gp_profile(ctx, mask) resets the counters and starts recording the kinds whose
 * bit (1 << GP_PROF_*) is set in mask -- mask 1 records the K V tile-pass kernel only, whether
 * launched by gp_kmv, gp_predict or inside a solver; gp_profile(ctx, 0) stops.
 * gp_profile_read_kind synchronises the stream and returns the number of bracketed launches of
 * one kind and the sum of their durations in milliseconds; gp_profile_read is the same for
 * GP_PROF_TILE.  At most 8192 launches are recorded per enable, later ones are not counted.
 * Either output pointer may be NULL.  Bracketing costs a few microseconds per launch, which
 * shows in the wall time of latency-bound solves: record the small kernels only where the
 * measurement is about them.
 */
enum {
  GP_PROF_TILE = 0,      /* K V tile pass (either arithmetic path) */
  GP_PROF_CG_DOT = 1,    /* gp_cg_solve: p^T (H p) */
  GP_PROF_CG_XR = 2,     /* gp_cg_solve: x += alpha p, r -= alpha H p, r^T r */
  GP_PROF_CG_P = 3,      /* gp_cg_solve: p = r + beta p */
  GP_PROF_GRAD_TILE = 4, /* gp_mll_grad: the gradient tile pass */
  GP_PROF_KINDS = 5
};
int gp_profile(gp_ctx* ctx, int enable);
int gp_profile_read(gp_ctx* ctx, int* h_launches, double* h_total_ms);
int gp_profile_read_kind(gp_ctx* ctx, int kind, int* h_launches, double* h_total_ms);

/*
 * Which arithmetic the K V tile pass uses for the current theta (Section 2.1 leaves the
 * arithmetic of the product open; all three meet the same accuracy bar).  gp_set_theta
 * picks it from the largest scaled squared norm max_i |(x_i - mean)/ell|^2:
 *   0  fp32 matrix-core products throughout,
 *   1  fp16 matrix-core products on operands split into two fp16 pieces (fp32 accumulation),
 *   2  the same with three pieces for the distance operands.
 * Returns the code, or GP_ERR_ARG for a NULL context or before the first gp_set_theta.
 */
int gp_product_path(const gp_ctx* ctx);

/* Text of the last error on this context ("" if none).  Never NULL. */
const char* gp_last_error(const gp_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* GPWS_H */
