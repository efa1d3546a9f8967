// C ABI entry points of libgpws: argument validation, context lifetime and
// dispatch to the kernel launchers.  Nothing crosses this boundary but plain
// pointers and sizes.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <cmath>
#include <cstdlib>
#include <mutex>
#include <new>

#include "gpws_internal.h"

int gp_fail(gp_ctx* ctx, int code, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return code;
}

int gp_ensure_scratch(gp_ctx* ctx, size_t bytes) {
  if (bytes <= ctx->scratch_bytes) return GP_OK;
  // not stream-ordered: make sure no kernel still uses the old block
  GP_HIP(ctx, hipStreamSynchronize(ctx->stream));
  if (ctx->dScratch) GP_HIP(ctx, hipFree(ctx->dScratch));
  ctx->dScratch = nullptr;
  ctx->scratch_bytes = 0;
  GP_HIP(ctx, hipMalloc(&ctx->dScratch, bytes));
  ctx->scratch_bytes = bytes;
  return GP_OK;
}

// ---- scratch of gp_kmv_static -------------------------------------------------------------------
// A file-scope device array instead of an allocation: every GPU the library runs on holds its own
// copy from the moment the code object is loaded until the process ends.  In host code the array's
// name is only a stand-in for the symbol, not a device address; the address on a given device comes
// from hipGetSymbolAddress with that device current, and only that pointer is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[GP_KMV_STATIC_SCRATCH_BYTES];

namespace {
constexpr int GP_MAX_DEVICES = 64;
std::mutex g_static_lock;
void* g_static_ptr[GP_MAX_DEVICES];   // per device: where `scratch` lives there (NULL until resolved)

// Address of the static scratch on device `dev`, which must be the current device; resolved once.
hipError_t static_scratch_on(int dev, void** out) {
  *out = nullptr;
  if (dev < 0 || dev >= GP_MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(g_static_lock);
  if (!g_static_ptr[dev]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_static_ptr[dev] = ptr;
  }
  *out = g_static_ptr[dev];
  return hipSuccess;
}
}  // namespace

extern "C" {

int gp_create(gp_ctx** out, int kernel, int64_t n, int d, const float* dX, void* hip_stream) {
  if (!out) return GP_ERR_ARG;
  *out = nullptr;
  if (kernel != GP_SE_ARD && kernel != GP_MATERN32_ARD) return GP_ERR_ARG;
  if (n < 1 || n > ((int64_t)1 << 31) - 4096 || d < 1 || d > GP_MAX_D || !dX) return GP_ERR_ARG;
  gp_ctx* ctx = new (std::nothrow) gp_ctx();
  if (!ctx) return GP_ERR_ARG;
  memset(ctx, 0, sizeof(*ctx));
  ctx->kernel = kernel;
  ctx->n = n;
  ctx->d = d;
  ctx->KS = gp_ks_bucket(d);
  ctx->KH = gp_kh_bucket(d, kernel);
  ctx->f16_ok = ctx->KH > 0;
  if (!ctx->f16_ok) ctx->KH = 8;   // operands are still allocated and packed, the product stays on the fp32 path
  ctx->path_forced = -1;
  if (const char* f = getenv("GPWS_PATH")) {      // testing aid: pin the product path
    if (!strcmp(f, "fp32")) ctx->path_forced = GP_PATH_FP32;
    else if (!strcmp(f, "f16x2")) ctx->path_forced = GP_PATH_F16X2;
    else if (!strcmp(f, "f16x3")) ctx->path_forced = GP_PATH_F16X3;
  }
  // tuning aids of the tile pass, read once here and never in a launch path
  if (const char* e = getenv("GPWS_MI")) ctx->mi_forced = atoi(e) == 2 ? 2 : 1;
  if (const char* e = getenv("GPWS_W")) ctx->w_forced = atoi(e) == 8 ? 8 : 4;
  ctx->n_pad = (n + GP_ROW_ALIGN - 1) / GP_ROW_ALIGN * GP_ROW_ALIGN;
  ctx->stream = (hipStream_t)hip_stream;
  ctx->dX = dX;
  *out = ctx;   // handed out even on failure below so the caller can read the error, then destroy

  int dev = 0;
  hipDeviceProp_t prop;
  GP_HIP(ctx, hipGetDevice(&dev));
  GP_HIP(ctx, hipGetDeviceProperties(&prop, dev));
  ctx->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
    return gp_fail(ctx, GP_ERR_HIP, "libgpws is built for gfx950 only, device is %s", prop.gcnArchName);
  GP_HIP(ctx, static_scratch_on(dev, &ctx->static_scratch));

  const size_t packed = ((size_t)(ctx->n_pad / GP_CHUNK) * ctx->KS * 64 + GP_PACK_SLACK) * sizeof(float);
  GP_HIP(ctx, hipMalloc((void**)&ctx->dXA, packed));
  GP_HIP(ctx, hipMalloc((void**)&ctx->dXB, packed));
  GP_HIP(ctx, hipMalloc((void**)&ctx->dXs, (size_t)n * d * sizeof(float)));
  GP_HIP(ctx, hipMalloc((void**)&ctx->dNorm, (size_t)ctx->n_pad * sizeof(float)));
  GP_HIP(ctx, hipMalloc((void**)&ctx->dMaxNorm, 256));
  {
    const size_t units = (size_t)(ctx->n_pad / GP_CHUNK) * ctx->KH * 64;
    for (int pc = 0; pc < 3; ++pc) {
      GP_HIP(ctx, hipMalloc(&ctx->dXAh[pc], units * 16));
      GP_HIP(ctx, hipMalloc(&ctx->dXBh[pc], units * 16));
    }
  }
  GP_HIP(ctx, hipMalloc((void**)&ctx->dMean, sizeof(double) * d));
  GP_HIP(ctx, hipMalloc((void**)&ctx->dTheta, sizeof(double) * (d + 2)));
  ctx->red_bytes = (size_t)1 << 22;
  GP_HIP(ctx, hipMalloc((void**)&ctx->dRed, ctx->red_bytes));
  ctx->pinned_bytes = (size_t)1 << 16;
  GP_HIP(ctx, hipHostMalloc(&ctx->hPinned, ctx->pinned_bytes, hipHostMallocDefault));
  GP_HIP(ctx, hipHostGetDevicePointer(&ctx->dPinned, ctx->hPinned, 0));
  return gp_launch_column_means(ctx);
}

int gp_destroy(gp_ctx* ctx) {
  if (!ctx) return GP_OK;
  (void)hipStreamSynchronize(ctx->stream);
  if (ctx->dXA) (void)hipFree(ctx->dXA);
  if (ctx->dXB) (void)hipFree(ctx->dXB);
  if (ctx->dXs) (void)hipFree(ctx->dXs);
  if (ctx->dNorm) (void)hipFree(ctx->dNorm);
  if (ctx->dMaxNorm) (void)hipFree(ctx->dMaxNorm);
  for (int pc = 0; pc < 3; ++pc) {
    if (ctx->dXAh[pc]) (void)hipFree(ctx->dXAh[pc]);
    if (ctx->dXBh[pc]) (void)hipFree(ctx->dXBh[pc]);
  }
  if (ctx->dMean) (void)hipFree(ctx->dMean);
  if (ctx->dTheta) (void)hipFree(ctx->dTheta);
  if (ctx->dRed) (void)hipFree(ctx->dRed);
  if (ctx->dScratch) (void)hipFree(ctx->dScratch);
  if (ctx->hPinned) (void)hipHostFree(ctx->hPinned);
  if (ctx->prof_ev) {
    for (int i = 0; i < 2 * GP_PROF_MAX; ++i) (void)hipEventDestroy(ctx->prof_ev[i]);
    delete[] ctx->prof_ev;
  }
  delete[] ctx->prof_kind;
  delete ctx;
  return GP_OK;
}

int gp_set_theta(gp_ctx* ctx, const double* h_lengthscale, double signal_scale, double noise_scale) {
  if (!ctx) return GP_ERR_ARG;
  if (!ctx->dXA) return gp_fail(ctx, GP_ERR_ARG, "gp_set_theta: context was not created successfully");
  if (!h_lengthscale) return gp_fail(ctx, GP_ERR_ARG, "gp_set_theta: NULL lengthscales");
  for (int k = 0; k < ctx->d; ++k)
    if (!(h_lengthscale[k] > 0.0) || !std::isfinite(h_lengthscale[k]))
      return gp_fail(ctx, GP_ERR_ARG, "gp_set_theta: lengthscale %d = %g is not positive and finite", k, h_lengthscale[k]);
  if (!(signal_scale > 0.0) || !std::isfinite(signal_scale))
    return gp_fail(ctx, GP_ERR_ARG, "gp_set_theta: signal scale %g is not positive and finite", signal_scale);
  if (!(noise_scale >= 0.0) || !std::isfinite(noise_scale))
    return gp_fail(ctx, GP_ERR_ARG, "gp_set_theta: noise scale %g is negative or not finite", noise_scale);
  // the staging region is this call's alone; the copy a previous call queued from it must have run
  GP_HIP(ctx, hipStreamSynchronize(ctx->stream));
  double* stage = (double*)((char*)ctx->hPinned + GP_PIN_THETA);
  for (int k = 0; k < ctx->d; ++k) {
    ctx->ell[k] = h_lengthscale[k];
    stage[k] = 1.0 / h_lengthscale[k];
  }
  stage[ctx->d] = signal_scale;
  stage[ctx->d + 1] = noise_scale;
  ctx->a = signal_scale;
  ctx->sigma = noise_scale;
  GP_HIP(ctx, hipMemcpyAsync(ctx->dTheta, stage, sizeof(double) * (ctx->d + 2), hipMemcpyHostToDevice, ctx->stream));
  GP_HIP(ctx, hipMemsetAsync(ctx->dMaxNorm, 0, sizeof(unsigned), ctx->stream));
  int rc = gp_launch_pack(ctx);
  if (rc < 0) return rc;
  // The largest scaled squared norm decides which product path holds the error budget.  The host-side
  // bound sum_k (xabs_k / ell_k)^2 >= max_i |xs_i|^2 settles the common case (two fp16 pieces) without a
  // read-back; otherwise the exact maximum found by the packing kernel is fetched.
  double bound = 0.0;
  for (int k = 0; k < ctx->d; ++k) bound += (ctx->xabs[k] / ctx->ell[k]) * (ctx->xabs[k] / ctx->ell[k]);
  bound *= 1.0 + 1e-5;   // fp32 rounding of the scaled inputs
  if (bound <= (double)GP_NORM_X2_MAX && ctx->path_forced < 0) {
    ctx->max_norm = (float)bound;
  } else {
    float* hmax = (float*)((char*)ctx->hPinned + GP_PIN_NORM);
    GP_HIP(ctx, hipMemcpyAsync(hmax, ctx->dMaxNorm, sizeof(float), hipMemcpyDeviceToHost, ctx->stream));
    GP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    ctx->max_norm = *hmax;
  }
  if (!std::isfinite(ctx->max_norm))
    return gp_fail(ctx, GP_ERR_ARG, "gp_set_theta: inputs scaled by the lengthscales are not finite");
  int path = ctx->max_norm <= GP_NORM_X2_MAX ? GP_PATH_F16X2
             : ctx->max_norm <= GP_NORM_X3_MAX ? GP_PATH_F16X3 : GP_PATH_FP32;
  if (ctx->path_forced >= 0 && !(ctx->path_forced != GP_PATH_FP32 && ctx->max_norm > GP_NORM_X3_MAX))
    path = ctx->path_forced;
  if (!ctx->f16_ok) path = GP_PATH_FP32;
  ctx->path = path;
  ctx->XP = path == GP_PATH_F16X3 ? 3 : 2;
  ctx->theta_set = true;
  return GP_OK;
}

static int check_block(gp_ctx* ctx, const char* who, const void* p, int64_t ld, int t) {
  if (!p) return gp_fail(ctx, GP_ERR_ARG, "%s: NULL device pointer", who);
  if (ld < t) return gp_fail(ctx, GP_ERR_ARG, "%s: leading dimension %lld < t = %d", who, (long long)ld, t);
  return GP_OK;
}

// argument checks shared by gp_kmv and gp_kmv_static
static int kmv_check(gp_ctx* ctx, const char* who, const float* dV, int64_t ldv, int t, float* dOut, int64_t ldo) {
  if (!ctx) return GP_ERR_ARG;
  if (!ctx->theta_set) return gp_fail(ctx, GP_ERR_ARG, "%s: gp_set_theta has not been called", who);
  if (t < 1 || t > GP_MAX_T) return gp_fail(ctx, GP_ERR_ARG, "%s: t = %d outside [1, %d]", who, t, GP_MAX_T);
  int rc;
  if ((rc = check_block(ctx, who, dV, ldv, t)) < 0) return rc;
  if ((rc = check_block(ctx, who, dOut, ldo, t)) < 0) return rc;
  // byte ranges the two blocks span (last row ends after t elements, not after a full leading dimension)
  const uintptr_t v0 = (uintptr_t)dV, v1 = v0 + ((size_t)(ctx->n - 1) * (size_t)ldv + (size_t)t) * sizeof(float);
  const uintptr_t o0 = (uintptr_t)dOut, o1 = o0 + ((size_t)(ctx->n - 1) * (size_t)ldo + (size_t)t) * sizeof(float);
  if (v0 < o1 && o0 < v1) return gp_fail(ctx, GP_ERR_ARG, "%s: dOut overlaps dV", who);
  return GP_OK;
}

int gp_kmv(gp_ctx* ctx, const float* dV, int64_t ldv, int t, float* dOut, int64_t ldo, int add_noise) {
  int rc = kmv_check(ctx, "gp_kmv", dV, ldv, t, dOut, ldo);
  if (rc < 0) return rc;
  const size_t need = gp_kmv_scratch_bytes(ctx, t);
  if ((rc = gp_ensure_scratch(ctx, need)) < 0) return rc;
  return gp_kmv_launch(ctx, dV, ldv, t, dOut, ldo, add_noise ? 1 : 0, ctx->dScratch, ctx->scratch_bytes, nullptr);
}

int gp_kmv_static(gp_ctx* ctx, const float* dV, int64_t ldv, int t, float* dOut, int64_t ldo, int add_noise) {
  int rc = kmv_check(ctx, "gp_kmv_static", dV, ldv, t, dOut, ldo);
  if (rc < 0) return rc;
  if (!ctx->static_scratch) return gp_fail(ctx, GP_ERR_HIP, "gp_kmv_static: the static scratch was not resolved on this device");
  const size_t need = gp_kmv_scratch_bytes(ctx, t);
  if (need > (size_t)GP_KMV_STATIC_SCRATCH_BYTES)
    return gp_fail(ctx, GP_ERR_WORKSPACE, "gp_kmv_static: n = %lld, t = %d need %zu bytes of scratch, the static block holds %zu; use gp_kmv",
                   (long long)ctx->n, t, need, (size_t)GP_KMV_STATIC_SCRATCH_BYTES);
  return gp_kmv_launch(ctx, dV, ldv, t, dOut, ldo, add_noise ? 1 : 0, ctx->static_scratch, (size_t)GP_KMV_STATIC_SCRATCH_BYTES, nullptr);
}

int gp_predict(gp_ctx* ctx, const float* dXstar, int64_t m, const float* dV, int64_t ldv, int t, float* dOut,
               int64_t ldo) {
  if (!ctx) return GP_ERR_ARG;
  if (!ctx->theta_set) return gp_fail(ctx, GP_ERR_ARG, "gp_predict: gp_set_theta has not been called");
  if (t < 1 || t > GP_MAX_T) return gp_fail(ctx, GP_ERR_ARG, "gp_predict: t = %d outside [1, %d]", t, GP_MAX_T);
  if (m < 1 || m > ((int64_t)1 << 30)) return gp_fail(ctx, GP_ERR_ARG, "gp_predict: m = %lld outside [1, 2^30]", (long long)m);
  if (!dXstar) return gp_fail(ctx, GP_ERR_ARG, "gp_predict: NULL dXstar");
  int rc;
  if ((rc = check_block(ctx, "gp_predict(dV)", dV, ldv, t)) < 0) return rc;
  if ((rc = check_block(ctx, "gp_predict(dOut)", dOut, ldo, t)) < 0) return rc;
  const size_t pack_bytes = gp_pack_rows_bytes(ctx, m);
  const size_t kmv_bytes = (gp_kmv_rect_scratch_bytes(ctx, t, m) + 255) / 256 * 256;
  if ((rc = gp_ensure_scratch(ctx, pack_bytes + kmv_bytes)) < 0) return rc;
  KmvRows rows;
  if ((rc = gp_pack_rows(ctx, dXstar, m, ctx->dScratch, &rows)) < 0) return rc;
  return gp_kmv_launch(ctx, dV, ldv, t, dOut, ldo, 0, (char*)ctx->dScratch + pack_bytes, kmv_bytes, nullptr, &rows);
}

size_t gp_workspace_bytes(const gp_ctx* ctx, int t) {
  if (!ctx || t < 1 || t > GP_MAX_T) return 0;
  return gp_cg_workspace_bytes(ctx, t);
}

int gp_cg_solve(gp_ctx* ctx, const float* dB, int64_t ldb, const float* dX0, float* dV, int64_t ldv, int t,
                const float* h_tol, int max_iters, void* dWork, size_t work_bytes, int* h_iters,
                int* h_kmv_count, float* h_relres) {
  if (!ctx) return GP_ERR_ARG;
  if (!ctx->theta_set) return gp_fail(ctx, GP_ERR_ARG, "gp_cg_solve: gp_set_theta has not been called");
  if (t < 1 || t > GP_MAX_T) return gp_fail(ctx, GP_ERR_ARG, "gp_cg_solve: t = %d outside [1, %d]", t, GP_MAX_T);
  int rc;
  if ((rc = check_block(ctx, "gp_cg_solve(dB)", dB, ldb, t)) < 0) return rc;
  if ((rc = check_block(ctx, "gp_cg_solve(dV)", dV, ldv, t)) < 0) return rc;
  if (!h_tol) return gp_fail(ctx, GP_ERR_ARG, "gp_cg_solve: NULL tolerances");
  for (int c = 0; c < t; ++c)
    if (!(h_tol[c] > 0.0f) || !std::isfinite(h_tol[c]))
      return gp_fail(ctx, GP_ERR_ARG, "gp_cg_solve: tolerance %d = %g is not positive and finite", c, (double)h_tol[c]);
  if (max_iters < 0) return gp_fail(ctx, GP_ERR_ARG, "gp_cg_solve: max_iters < 0");
  if (!dWork) return gp_fail(ctx, GP_ERR_WORKSPACE, "gp_cg_solve: NULL workspace");
  return gp_cg_run(ctx, dB, ldb, dX0, dV, ldv, t, h_tol, max_iters, dWork, work_bytes, h_iters, h_kmv_count,
                   h_relres);
}

size_t gp_ap_workspace_bytes(const gp_ctx* ctx, int t, int block) {
  if (!ctx || t < 1 || t > GP_MAX_T || block < 1 || block > GP_AP_MAX_BLOCK) return 0;
  return gp_ap_workspace_bytes_impl(ctx, t, block);
}

int gp_ap_solve(gp_ctx* ctx, const float* dB, int64_t ldb, const float* dX0, float* dV, int64_t ldv, int t,
                const float* h_tol, int block, int max_iters, void* dWork, size_t work_bytes, int* h_iters,
                int* h_kmv_count, float* h_relres, int* h_picks) {
  if (!ctx) return GP_ERR_ARG;
  if (!ctx->theta_set) return gp_fail(ctx, GP_ERR_ARG, "gp_ap_solve: gp_set_theta has not been called");
  if (t < 1 || t > GP_MAX_T) return gp_fail(ctx, GP_ERR_ARG, "gp_ap_solve: t = %d outside [1, %d]", t, GP_MAX_T);
  if (block < 1 || block > GP_AP_MAX_BLOCK)
    return gp_fail(ctx, GP_ERR_ARG, "gp_ap_solve: block = %d outside [1, %d]", block, GP_AP_MAX_BLOCK);
  if ((ctx->n + block - 1) / block > (1 << 20))
    return gp_fail(ctx, GP_ERR_ARG, "gp_ap_solve: more than 2^20 blocks");
  int rc;
  if ((rc = check_block(ctx, "gp_ap_solve(dB)", dB, ldb, t)) < 0) return rc;
  if ((rc = check_block(ctx, "gp_ap_solve(dV)", dV, ldv, t)) < 0) return rc;
  if (!h_tol) return gp_fail(ctx, GP_ERR_ARG, "gp_ap_solve: NULL tolerances");
  for (int c = 0; c < t; ++c)
    if (!(h_tol[c] > 0.0f) || !std::isfinite(h_tol[c]))
      return gp_fail(ctx, GP_ERR_ARG, "gp_ap_solve: tolerance %d = %g is not positive and finite", c, (double)h_tol[c]);
  if (max_iters < 0) return gp_fail(ctx, GP_ERR_ARG, "gp_ap_solve: max_iters < 0");
  if (!dWork) return gp_fail(ctx, GP_ERR_WORKSPACE, "gp_ap_solve: NULL workspace");
  return gp_ap_run(ctx, dB, ldb, dX0, dV, ldv, t, h_tol, block, max_iters, dWork, work_bytes, h_iters, h_kmv_count,
                   h_relres, h_picks);
}

size_t gp_sgd_workspace_bytes(const gp_ctx* ctx, int t, int batch) {
  if (!ctx || t < 1 || t > GP_MAX_T || batch < 1 || batch > GP_SGD_MAX_BATCH || batch > ctx->n) return 0;
  return gp_sgd_workspace_bytes_impl(ctx, t, batch);
}

int gp_sgd_solve(gp_ctx* ctx, const float* dB, int64_t ldb, const float* dX0, float* dV, int64_t ldv, int t,
                 const float* h_tol, const int32_t* dBatches, int batch, int max_iters, double lr, double momentum,
                 void* dWork, size_t work_bytes, int* h_iters, int* h_kmv_count, float* h_relres) {
  if (!ctx) return GP_ERR_ARG;
  if (!ctx->theta_set) return gp_fail(ctx, GP_ERR_ARG, "gp_sgd_solve: gp_set_theta has not been called");
  if (t < 1 || t > GP_MAX_T) return gp_fail(ctx, GP_ERR_ARG, "gp_sgd_solve: t = %d outside [1, %d]", t, GP_MAX_T);
  if (batch < 1 || batch > GP_SGD_MAX_BATCH || batch > ctx->n)
    return gp_fail(ctx, GP_ERR_ARG, "gp_sgd_solve: batch = %d outside [1, min(n, %d)]", batch, GP_SGD_MAX_BATCH);
  int rc;
  if ((rc = check_block(ctx, "gp_sgd_solve(dB)", dB, ldb, t)) < 0) return rc;
  if ((rc = check_block(ctx, "gp_sgd_solve(dV)", dV, ldv, t)) < 0) return rc;
  if (!h_tol) return gp_fail(ctx, GP_ERR_ARG, "gp_sgd_solve: NULL tolerances");
  for (int c = 0; c < t; ++c)
    if (!(h_tol[c] > 0.0f) || !std::isfinite(h_tol[c]))
      return gp_fail(ctx, GP_ERR_ARG, "gp_sgd_solve: tolerance %d = %g is not positive and finite", c, (double)h_tol[c]);
  if (max_iters < 0) return gp_fail(ctx, GP_ERR_ARG, "gp_sgd_solve: max_iters < 0");
  if (max_iters > 0 && !dBatches) return gp_fail(ctx, GP_ERR_ARG, "gp_sgd_solve: NULL mini-batch indices");
  if (!(lr > 0.0) || !std::isfinite(lr)) return gp_fail(ctx, GP_ERR_ARG, "gp_sgd_solve: learning rate %g is not positive and finite", lr);
  if (!(momentum >= 0.0) || !(momentum < 1.0)) return gp_fail(ctx, GP_ERR_ARG, "gp_sgd_solve: momentum %g outside [0, 1)", momentum);
  if (!dWork) return gp_fail(ctx, GP_ERR_WORKSPACE, "gp_sgd_solve: NULL workspace");
  return gp_sgd_run(ctx, dB, ldb, dX0, dV, ldv, t, h_tol, dBatches, batch, max_iters, lr, momentum, dWork, work_bytes,
                    h_iters, h_kmv_count, h_relres);
}

int gp_mll_grad(gp_ctx* ctx, const float* dV, int64_t ldv, const float* dB, int64_t ldb, int t, double* h_grad) {
  if (!ctx) return GP_ERR_ARG;
  if (!ctx->theta_set) return gp_fail(ctx, GP_ERR_ARG, "gp_mll_grad: gp_set_theta has not been called");
  if (t < 1 || t > GP_MAX_T) return gp_fail(ctx, GP_ERR_ARG, "gp_mll_grad: t = %d outside [1, %d]", t, GP_MAX_T);
  int rc;
  if ((rc = check_block(ctx, "gp_mll_grad(dV)", dV, ldv, t)) < 0) return rc;
  if ((rc = check_block(ctx, "gp_mll_grad(dB)", dB, ldb, t)) < 0) return rc;
  if (!h_grad) return gp_fail(ctx, GP_ERR_ARG, "gp_mll_grad: NULL output");
  return gp_grad_run(ctx, dV, ldv, dB, ldb, t, h_grad);
}

int gp_profile(gp_ctx* ctx, int enable) {
  if (!ctx) return GP_ERR_ARG;
  if (enable < 0 || enable >= (1 << GP_PROF_KINDS)) return gp_fail(ctx, GP_ERR_ARG, "gp_profile: unknown kinds in mask %d", enable);
  if (enable && !ctx->prof_ev) {
    ctx->prof_ev = new (std::nothrow) hipEvent_t[2 * GP_PROF_MAX];
    ctx->prof_kind = new (std::nothrow) unsigned char[GP_PROF_MAX];
    if (!ctx->prof_ev || !ctx->prof_kind) return gp_fail(ctx, GP_ERR_ARG, "gp_profile: out of host memory");
    for (int i = 0; i < 2 * GP_PROF_MAX; ++i) GP_HIP(ctx, hipEventCreate(&ctx->prof_ev[i]));
  }
  if (enable) ctx->prof_count = 0;
  ctx->prof_mask = (unsigned)enable;
  return GP_OK;
}

int gp_product_path(const gp_ctx* ctx) {
  if (!ctx || !ctx->theta_set) return GP_ERR_ARG;
  return ctx->path;
}

int gp_profile_read_kind(gp_ctx* ctx, int kind, int* h_launches, double* h_total_ms) {
  if (!ctx) return GP_ERR_ARG;
  if (kind < 0 || kind >= GP_PROF_KINDS) return gp_fail(ctx, GP_ERR_ARG, "gp_profile_read_kind: kind %d", kind);
  GP_HIP(ctx, hipStreamSynchronize(ctx->stream));
  double tot = 0.0;
  int count = 0;
  for (int i = 0; i < ctx->prof_count; ++i) {
    if (ctx->prof_kind[i] != kind) continue;
    float ms = 0.0f;
    GP_HIP(ctx, hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]));
    tot += (double)ms;
    ++count;
  }
  if (h_launches) *h_launches = count;
  if (h_total_ms) *h_total_ms = tot;
  return GP_OK;
}

int gp_profile_read(gp_ctx* ctx, int* h_launches, double* h_total_ms) {
  return gp_profile_read_kind(ctx, GP_PROF_TILE, h_launches, h_total_ms);
}

const char* gp_last_error(const gp_ctx* ctx) { return ctx ? ctx->err : "NULL context"; }

}  // extern "C"
