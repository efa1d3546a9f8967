// Internal declarations shared by the translation units of libgpws (gfx950 only).
#ifndef GPWS_INTERNAL_H
#define GPWS_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/gpws.h"

// ---------------------------------------------------------------------------
// Geometry of the tile pass.  A wavefront (64 lanes) owns MI sub-tiles of 32
// rows i and walks over the columns j in chunks of 32; one 32x32 tile of
// pairs is one v_mfma_f32_32x32x2_f32 accumulator (16 VGPRs per lane).
// ---------------------------------------------------------------------------
constexpr int GP_CHUNK = 32;          // rows per packed operand chunk
constexpr int GP_WAVES = 4;           // wavefronts per workgroup
constexpr int GP_THREADS = 64 * GP_WAVES;
constexpr int GP_ROW_ALIGN = 512;     // packed operand arrays are padded to this many rows
constexpr int GP_VEC_PAD = 4;         // solver arrays are padded to a multiple of 4 rows (float4 streams)
constexpr float GP_PAD_NORM = 1.0e30f; // squared norm given to padding rows of XA (phi underflows to 0)
constexpr int GP_PACK_SLACK = 256;    // floats allocated past the packed arrays: staging loads overrun by < 256
constexpr float GP_PAD_NORM_H = 60000.0f;  // same for the fp16 operands (must fit fp16)
enum { GP_PATH_FP32 = 0, GP_PATH_F16X2 = 1, GP_PATH_F16X3 = 2 };
// fp16 distance pieces: two pieces carry 22 bits, so r^2 has an absolute error ~2^-22 (|xs_i|^2+|xs_j|^2);
// past this squared norm three pieces (33 bits) are used, and past fp16's range the fp32 MFMA path
constexpr float GP_NORM_X2_MAX = 64.0f;
constexpr float GP_NORM_X3_MAX = 16000.0f;
constexpr int GP_FLUSH_CHUNKS = 1024; // tile kernels add their fp32 accumulators into OUT every this many column chunks (power of 2)
constexpr int GP_PROF_MAX = 8192;     // event pairs available to gp_profile
// Regions of the context's pinned host block (64 KB).  A region the host writes before an asynchronous
// host-to-device copy must not be written again until that copy has run, so gp_set_theta has one no
// other call touches (it waits for the stream before writing it); the solvers stage their tolerances
// and read results back in the first region and synchronise before they return.
constexpr size_t GP_PIN_SOLVER = 0;       // flags, tolerances in, residuals / gradient sums out
constexpr size_t GP_PIN_THETA = 16384;    // gp_set_theta: 1/ell, a, sigma staged for the device copy
constexpr size_t GP_PIN_NORM = 24576;     // largest scaled squared norm read back
constexpr size_t GP_PIN_POST = 32768;     // flags the solvers' finalise kernels post for the host loop

// Operands of the distance contraction, packed so that one wave-wide dword
// load is one MFMA operand: P[(chunk*KS + ks)*64 + lane] holds, for row
// 32*chunk + lane%32, the component k = 2*ks + lane/32 of
//   XA (column side j): [ xs_j(0..d-1), |xs_j|^2, 1, 0.. ]
//   XB (row side i)   : g * [ -2 xs_i(0..d-1), 1, |xs_i|^2, 0.. ]
// with xs = (x - mean)/ell and g = -log2(e)/2 (SE) or 3 (Matern-3/2), so that
// XA_j . XB_i = g * r^2_ij comes straight out of the MFMA chain.
struct gp_ctx {
  int kernel;
  int64_t n;
  int d;
  int KS;                 // k-steps (of 2) of the distance chain, bucketed
  int64_t n_pad;          // n rounded up to GP_ROW_ALIGN
  hipStream_t stream;
  const float* dX;        // caller-owned
  float* dXA;             // packed, n_pad/32 * KS * 64
  float* dXB;
  float* dXs;             // scaled centred inputs, row-major n x d (gradient pass)
  float* dNorm;           // |xs_i|^2, n_pad entries
  unsigned* dMaxNorm;     // bit pattern of max_i |xs_i|^2 (device), refreshed by gp_set_theta
  // split-fp16 operands of the matrix-core path: three pieces (hi, mid, lo) per side, 16-byte units
  // [(chunk*KH + kh)*64 + lane], element e of a unit = component 16 kh + 8 (lane/32) + e
  void* dXAh[3];
  void* dXBh[3];
  int KH;                 // 16-wide k-steps of the fp16 distance chain, bucketed
  int XP;                 // pieces used per operand of the distance chain (2 or 3)
  int path;               // GP_PATH_* chosen by gp_set_theta
  int path_forced;        // -1, or a GP_PATH_* forced through the GPWS_PATH environment variable
  int mi_forced;          // 0, or the sub-tiles per wave forced through GPWS_MI (tuning aid, read at gp_create)
  int w_forced;           // 0, or the wavefronts per workgroup forced through GPWS_W (tuning aid, read at gp_create)
  bool f16_ok;            // false when d + 3 components do not fit the widest fp16 operand bucket (SE, d = 126)
  float max_norm;         // host copy of max_i |xs_i|^2
  double* dMean;          // d column means of X
  double* dTheta;         // device copy: 1/ell (d), then a, sigma
  bool theta_set;
  double xabs[GP_MAX_D];  // max_i |x_ik - mean_k| per dimension (host copy, fixed at gp_create)
  double ell[GP_MAX_D];
  double a, sigma;
  // lazily grown scratch for split-column partial sums of gp_kmv / gp_mll_grad
  void* dScratch;
  size_t scratch_bytes;
  void* static_scratch;   // this device's address of the file-scope scratch gp_kmv_static uses (never freed)
  // small device + pinned host blocks for scalars
  double* dRed;           // reduction partials
  size_t red_bytes;
  void* hPinned;          // pinned host staging for scalar read-back
  void* dPinned;          // the same block as the device addresses it (kernels post small results there)
  size_t pinned_bytes;
  int num_cu;
  // event pairs bracketing kernel launches while profiling is on (gp_profile): prof_mask has bit k set
  // when launches of kind k (GP_PROF_* of gpws.h) are bracketed
  unsigned prof_mask;
  int prof_count;
  hipEvent_t* prof_ev;    // 2 * GP_PROF_MAX events, created on first enable
  unsigned char* prof_kind;   // kind of every recorded pair
  char err[256];
};

// Row side of a rectangular product K(X*, X) V: m other points packed like the context's own rows
// (same centring, lengthscales and scaling).  NULL everywhere below means the square product.
struct KmvRows {
  int64_t m;
  const float* XB;        // fp32 packed row operands, [m_pad/32][KS][64]
  const void* XBh[3];     // fp16 pieces, [m_pad/32][KH][64] 16-byte units
  int path;               // GP_PATH_* to use (covers the norms of both point sets)
};

// Column-split partial results of a product whose final sum the caller takes over (the CG dot-product
// kernel adds the partials while it reads H P anyway): OUT_ic = sum_k part[k stride + i t + c].
// JS == 1 means the launcher wrote OUT itself.
struct KmvDeferred {
  const float* part;
  int64_t stride;
  int JS;
};

// Contraction restricted to the context's points 32 chunk0 .. min(n, 32 (chunk0 + nchunks)) - 1 (a
// column block of K): OUT = K[:, window] V[window, :].  V is still the full-height n x t array; only
// the window's rows are read.  Coincident pairs get no special treatment (as in a rectangular product)
// and no noise term can be asked for.
struct KmvWindow {
  int chunk0;
  int nchunks;
};

int gp_fail(gp_ctx* ctx, int code, const char* fmt, ...);
#define GP_HIP(ctx, call)                                                              \
  do {                                                                                 \
    hipError_t e__ = (call);                                                           \
    if (e__ != hipSuccess)                                                             \
      return gp_fail(ctx, GP_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e__)); \
  } while (0)

// Bracket one kernel launch of the given kind with an event pair when that kind is being profiled:
//   const bool pr = gp_prof_begin(ctx, kind);  launch;  gp_prof_end(ctx, pr);
inline bool gp_prof_begin(gp_ctx* ctx, int kind) {
  if (!((ctx->prof_mask >> kind) & 1u) || ctx->prof_count >= GP_PROF_MAX) return false;
  if (hipEventRecord(ctx->prof_ev[2 * ctx->prof_count], ctx->stream) != hipSuccess) return false;
  ctx->prof_kind[ctx->prof_count] = (unsigned char)kind;
  return true;
}
inline void gp_prof_end(gp_ctx* ctx, bool begun) {
  if (!begun) return;
  if (hipEventRecord(ctx->prof_ev[2 * ctx->prof_count + 1], ctx->stream) == hipSuccess) ++ctx->prof_count;
}

int gp_ks_bucket(int d);   // -1 if d is out of range
int gp_ensure_scratch(gp_ctx* ctx, size_t bytes);

// ---- prep_kernels.hip
int gp_launch_column_means(gp_ctx* ctx);
int gp_launch_pack(gp_ctx* ctx);
// packs m other points (device, row-major m x d) against the context's centring and theta into
// caller-provided buffers sized by gp_pack_rows_bytes; fills rows (path from the larger of the two
// sets' scaled norms; synchronises the stream to read that norm back)
size_t gp_pack_rows_bytes(const gp_ctx* ctx, int64_t m);
int gp_pack_rows(gp_ctx* ctx, const float* dXstar, int64_t m, void* buf, KmvRows* rows);

// ---- tile_pass.hip
struct KmvPlan {
  int MI;        // 32-row sub-tiles per wave
  int W;         // wavefronts per workgroup (fp16 path; the fp32 path always uses GP_WAVES)
  int JS;        // column-range splits
  int row_blocks;
  int cps;       // chunks per split
};
KmvPlan gp_plan_kmv(const gp_ctx* ctx, int64_t rows, int64_t col_chunks = 0);   // col_chunks = 0: all of the context's
size_t gp_kmv_scratch_bytes(const gp_ctx* ctx, int t);   // square product, worst case over the paths gp_set_theta may choose
size_t gp_kmv_rect_scratch_bytes(const gp_ctx* ctx, int t, int64_t rows);
size_t gp_kmv_window_scratch_bytes(const gp_ctx* ctx, int t, int col_chunks);   // product over any column window of at most that many chunks
// OUT = K V (+ sigma^2 V).  colmax: optional device array of t bit patterns of max_i |V_ic| that the
// caller already holds (the split-fp16 path then skips its own reduction over V); NULL otherwise.
// rows: NULL, or the row side of a rectangular product (add_noise must then be 0).
// defer: NULL, or where to report column-split partials instead of summing them into OUT.
int gp_kmv_launch(gp_ctx* ctx, const float* dV, int64_t ldv, int t, float* dOut, int64_t ldo,
                  int add_noise, void* scratch, size_t scratch_bytes, const unsigned* colmax,
                  const KmvRows* rows = nullptr, KmvDeferred* defer = nullptr, const KmvWindow* win = nullptr);

// ---- tile_pass_f16.hip
int gp_kh_bucket(int d, int kernel);
KmvPlan gp_plan_kmv_f16(const gp_ctx* ctx, int64_t rows, int64_t col_chunks = 0);
size_t gp_kmv_f16_scratch_bytes(const gp_ctx* ctx, int t, int64_t rows, int64_t col_chunks = 0);
int gp_kmv_launch_f16(gp_ctx* ctx, const float* dV, int64_t ldv, int t, float* dOut, int64_t ldo,
                      int add_noise, void* scratch, size_t scratch_bytes, const unsigned* colmax,
                      const KmvRows* rows, KmvDeferred* defer, const KmvWindow* win);

// colmax[c] = bit pattern of max_i |V_ic| for c < t, stream-ordered; optionally the same for a second
// n x t matrix in the same launch.  cleared = true: the caller has already zeroed the output words.
int gp_launch_colmax(gp_ctx* ctx, const float* dV, int64_t ldv, int t, unsigned* colmax, const float* dV2 = nullptr,
                     int64_t ldv2 = 0, unsigned* colmax2 = nullptr, bool cleared = false);

// ---- ap_kernels.hip
size_t gp_ap_workspace_bytes_impl(const gp_ctx* ctx, int t, int block);
int gp_ap_run(gp_ctx* ctx, const float* dB, int64_t ldb, const float* dX0, float* dV, int64_t ldv, int t,
              const float* h_tol, int block, int max_iters, void* dWork, size_t work_bytes, int* h_iters,
              int* h_kmv_count, float* h_relres, int* h_picks);

// ---- sgd_kernels.hip
size_t gp_sgd_workspace_bytes_impl(const gp_ctx* ctx, int t, int batch);
int gp_sgd_run(gp_ctx* ctx, const float* dB, int64_t ldb, const float* dX0, float* dV, int64_t ldv, int t,
               const float* h_tol, const int* dBatches, int batch, int max_iters, double lr, double momentum,
               void* dWork, size_t work_bytes, int* h_iters, int* h_kmv_count, float* h_relres);

// ---- cg_kernels.hip
int gp_cg_run(gp_ctx* ctx, const float* dB, int64_t ldb, const float* dX0, float* dV, int64_t ldv,
              int t, const float* h_tol, int max_iters, void* dWork, size_t work_bytes,
              int* h_iters, int* h_kmv_count, float* h_relres);
size_t gp_cg_workspace_bytes(const gp_ctx* ctx, int t);

// ---- grad_pass.hip
int gp_grad_run(gp_ctx* ctx, const float* dV, int64_t ldv, const float* dB, int64_t ldb, int t,
                double* h_grad);
// fp64 reduction of one right-hand-side block's tile-pass output OUT[JS][n][nq] into acc[d + 2]
// (part: G x (d + 2) workgroup partials); first_block adds the sigma component sum_i w_ii
int gp_grad_reduce_launch(gp_ctx* ctx, const float* OUT, int64_t split_stride, int JS, int nq, const float* dV,
                          int64_t ldv, const float* dB, int64_t ldb, int t, float half_w, float probe_w,
                          int first_block, double* part, int G, double* acc);

// ---- grad_pass_f16.hip
int gp_grad_run_f16(gp_ctx* ctx, const float* dV, int64_t ldv, const float* dB, int64_t ldb, int t,
                    double* h_grad);

#endif
