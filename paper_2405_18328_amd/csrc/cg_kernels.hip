// Batched conjugate gradients without a preconditioner (paper Section 2.1
// "Linear System Solver", Appendix B): one Hestenes-Stiefel recurrence per
// column, all columns sharing each matrix-free product H P.  A column is frozen
// (no further updates) once its recursive relative residual is below its
// tolerance; the solve ends when every column is frozen.
//
// The vector part is HBM-bound streaming.  X, R, P, HP live in the caller's
// workspace as contiguous n4 x t fp32 arrays (n4 = n rounded up to 4, padding
// rows kept at zero), so every kernel walks them as one flat float4 stream.
// The grid is a multiple of t workgroups, which makes each thread's stride a
// multiple of t: a thread always sees the same 4 columns and keeps their
// partial dot products in registers.  Per-column sums go thread -> LDS
// (fixed-order gather) -> per-workgroup fp64 partials -> a one-workgroup
// finalise kernel; nothing uses atomics, so a solve is bit-reproducible.
#include "gpws_internal.h"

typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int VT = 256;                 // threads per workgroup in the streaming kernels
constexpr int VW = 4 * VT;              // flat elements one workgroup covers per step
constexpr int FT = 1024;                // threads of the finalise kernels

struct CgFlags {
  int all_done;
  int breakdown;
  int iters;
  int seq;          // host mirror only: number of finalise steps posted so far (written last)
};

struct CgDev {
  CgFlags* flags;
  CgFlags* post;    // pinned host memory: the finalise kernels post the flags there for the host loop
  double* rho;      // [t] current r^T r
  double* bn2;      // [t] ||b||^2
  float* alpha;     // [t]
  float* beta;      // [t]
  float* tol;       // [t]
  float* relres;    // [t]
  int* frozen;      // [t]
  int* zero_rhs;    // [t]
  unsigned* colmax; // [t] bit patterns of max |P_ic|, kept current for the split-fp16 product
  double* part;     // [G][t] workgroup partials
  double* part2;    // [G][t] second set (init only)
};

// Sum, for every column c, the per-thread values of the threads that hold c.
// Thread `tid` holds flat positions 4*tid..4*tid+3 of a 1024-wide window that
// starts at flat offset `base`; position p belongs to column (base + p) % t.
__device__ __forceinline__ void block_column_sums(const float v[4], int t, int base_mod, double* out,
                                                  float* sh /* [VW] */) {
  const int tid = threadIdx.x;
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 4; ++q) sh[4 * tid + q] = v[q];
  __syncthreads();
  for (int c = tid; c < t; c += VT) {
    int p0 = c - base_mod;
    if (p0 < 0) p0 += t;
    double s = 0.0;
    for (int p = p0; p < VW; p += t) s += (double)sh[p];
    out[c] = s;
  }
}

// colmax[c] = max(colmax[c], max over this workgroup's elements of |.|) for the thread's four columns;
// non-negative floats order like unsigned ints, and max does not depend on the order of the updates
__device__ __forceinline__ void block_column_max(const float m[4], const int c[4], int t, unsigned* colmax,
                                                 unsigned* smax /* [t] */) {
  for (int k = threadIdx.x; k < t; k += VT) smax[k] = 0u;
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 4; ++q) atomicMax(&smax[c[q]], __float_as_uint(m[q]));
  __syncthreads();
  for (int k = threadIdx.x; k < t; k += VT)
    if (smax[k]) atomicMax(&colmax[k], smax[k]);
}

__device__ __forceinline__ void thread_columns(int t, int64_t e0, int c[4]) {
  int c0 = (int)(e0 % t);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    c[q] = c0;
    c0 = (c0 + 1 == t) ? 0 : c0 + 1;
  }
}

// H p (or H x0) at flat positions e..e+3 as the fixed-order sum of the JS column-split partials the
// product left (flat index e = i t + c in every partial; positions at or past `valid` are padding: 0).
__device__ __forceinline__ f32x4 sum_split_partials(const float* __restrict__ part_in, int64_t part_stride, int JS,
                                                    int64_t e, int64_t valid) {
  f32x4 hp = f32x4{0.f, 0.f, 0.f, 0.f};
  if ((part_stride & 3) == 0 && e + 4 <= valid) {
#pragma unroll 4
    for (int k = 0; k < JS; ++k) hp += *reinterpret_cast<const f32x4*>(part_in + (int64_t)k * part_stride + e);
  } else {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (e + q < valid)
        for (int k = 0; k < JS; ++k) hp[q] += part_in[(int64_t)k * part_stride + e + q];
  }
  return hp;
}

// X <- X0 (or 0), R <- B, partial ||b||^2.  Rows >= n of the padded arrays are zeroed.
__global__ __launch_bounds__(VT) void cg_load_kernel(const float* __restrict__ B, int64_t ldb,
                                                     const float* __restrict__ X0, int64_t ldx, int64_t n,
                                                     int64_t n4, int t, float* __restrict__ X,
                                                     float* __restrict__ R, double* __restrict__ part,
                                                     unsigned* __restrict__ colmax) {
  __shared__ float sh[VW];
  __shared__ unsigned smax[GP_MAX_T];
  const int64_t total = n4 * t;
  const int64_t stride = (int64_t)gridDim.x * VW;   // a multiple of t: a thread keeps its four columns
  const int64_t e0 = ((int64_t)blockIdx.x * VT + threadIdx.x) * 4;
  float acc[4] = {0.f, 0.f, 0.f, 0.f}, mx[4] = {0.f, 0.f, 0.f, 0.f};
  for (int64_t e = e0; e < total; e += stride) {
    f32x4 b, x;
    int64_t i = e / t;
    int c = (int)(e - i * t);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const bool live = i < n;
      b[q] = live ? B[i * ldb + c] : 0.0f;
      x[q] = (live && X0) ? X0[i * ldx + c] : 0.0f;
      acc[q] = fmaf(b[q], b[q], acc[q]);
      mx[q] = fmaxf(mx[q], fabsf(x[q]));
      if (++c == t) { c = 0; ++i; }
    }
    *reinterpret_cast<f32x4*>(X + e) = x;
    *reinterpret_cast<f32x4*>(R + e) = b;
  }
  block_column_sums(acc, t, (int)(((int64_t)blockIdx.x * VW) % t), part + (int64_t)blockIdx.x * t, sh);
  if (X0) {   // max |X0| per column for the warm start's product H x0
    int cq[4];
    thread_columns(t, e0, cq);
    block_column_max(mx, cq, t, colmax, smax);
  }
}

// R <- R - HX (warm start: initial residual), then (both cases) P <- R, partial r^T r.  HX is read from
// the product's column-split partials when it left them unsummed (JS > 1).
__global__ __launch_bounds__(VT) void cg_resid_kernel(float* __restrict__ R, const float* __restrict__ HX,
                                                      const float* __restrict__ part_in, int64_t part_stride,
                                                      int JS, int64_t valid, int subtract,
                                                      float* __restrict__ P, int64_t total, int t,
                                                      double* __restrict__ part, unsigned* __restrict__ colmax) {
  __shared__ float sh[VW];
  __shared__ unsigned smax[GP_MAX_T];
  const int64_t e0 = ((int64_t)blockIdx.x * VT + threadIdx.x) * 4;
  const int64_t stride = (int64_t)gridDim.x * VW;
  int c[4];
  thread_columns(t, e0, c);
  float acc[4] = {0.f, 0.f, 0.f, 0.f}, mx[4] = {0.f, 0.f, 0.f, 0.f};
  for (int64_t e = e0; e < total; e += stride) {
    f32x4 r = *reinterpret_cast<const f32x4*>(R + e);
    if (subtract) {
      const f32x4 hx = JS > 1 ? sum_split_partials(part_in, part_stride, JS, e, valid)
                              : *reinterpret_cast<const f32x4*>(HX + e);
      r -= hx;
      *reinterpret_cast<f32x4*>(R + e) = r;
    }
    *reinterpret_cast<f32x4*>(P + e) = r;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      acc[q] = fmaf(r[q], r[q], acc[q]);
      mx[q] = fmaxf(mx[q], fabsf(r[q]));
    }
  }
  block_column_sums(acc, t, (int)(((int64_t)blockIdx.x * VW) % t), part + (int64_t)blockIdx.x * t, sh);
  block_column_max(mx, c, t, colmax, smax);   // max |P| per column for the product that follows
}

// partial p^T (H p).  When the product left column-split partials (JS > 1), H p is first formed here as
// their fixed-order sum and written to HP (flat index e = i t + c, identical in both layouts; elements
// at or past n t are padding and stay zero).
__global__ __launch_bounds__(VT) void cg_dot_kernel(const float* __restrict__ P, float* __restrict__ HP,
                                                    const float* __restrict__ part_in, int64_t part_stride, int JS,
                                                    int64_t valid, int64_t total, int t,
                                                    const CgFlags* __restrict__ flags, double* __restrict__ part) {
  __shared__ float sh[VW];
  if (flags->all_done) return;
  const int64_t stride = (int64_t)gridDim.x * VW;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int64_t e = ((int64_t)blockIdx.x * VT + threadIdx.x) * 4; e < total; e += stride) {
    const f32x4 p = *reinterpret_cast<const f32x4*>(P + e);
    f32x4 hp;
    if (JS > 1) {
      hp = sum_split_partials(part_in, part_stride, JS, e, valid);
      *reinterpret_cast<f32x4*>(HP + e) = hp;
    } else {
      hp = *reinterpret_cast<const f32x4*>(HP + e);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] = fmaf(p[q], hp[q], acc[q]);
  }
  block_column_sums(acc, t, (int)(((int64_t)blockIdx.x * VW) % t), part + (int64_t)blockIdx.x * t, sh);
}

// x += alpha p ; r -= alpha Hp ; partial r^T r
__global__ __launch_bounds__(VT) void cg_update_xr_kernel(float* __restrict__ X, float* __restrict__ R,
                                                          const float* __restrict__ P,
                                                          const float* __restrict__ HP, int64_t total, int t,
                                                          const float* __restrict__ alpha,
                                                          const CgFlags* __restrict__ flags,
                                                          double* __restrict__ part) {
  __shared__ float sh[VW];
  if (flags->all_done) return;
  const int64_t e0 = ((int64_t)blockIdx.x * VT + threadIdx.x) * 4;
  const int64_t stride = (int64_t)gridDim.x * VW;
  int c[4];
  thread_columns(t, e0, c);
  float al[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) al[q] = alpha[c[q]];
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int64_t e = e0; e < total; e += stride) {
    const f32x4 p = *reinterpret_cast<const f32x4*>(P + e);
    const f32x4 hp = *reinterpret_cast<const f32x4*>(HP + e);
    f32x4 x = *reinterpret_cast<const f32x4*>(X + e);
    f32x4 r = *reinterpret_cast<const f32x4*>(R + e);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      x[q] = fmaf(al[q], p[q], x[q]);
      r[q] = fmaf(-al[q], hp[q], r[q]);
      acc[q] = fmaf(r[q], r[q], acc[q]);
    }
    *reinterpret_cast<f32x4*>(X + e) = x;
    *reinterpret_cast<f32x4*>(R + e) = r;
  }
  block_column_sums(acc, t, (int)(((int64_t)blockIdx.x * VW) % t), part + (int64_t)blockIdx.x * t, sh);
}

// p = r + beta p
__global__ __launch_bounds__(VT) void cg_update_p_kernel(float* __restrict__ P, const float* __restrict__ R,
                                                         int64_t total, int t, const float* __restrict__ beta,
                                                         const CgFlags* __restrict__ flags,
                                                         unsigned* __restrict__ colmax) {
  __shared__ unsigned smax[GP_MAX_T];
  if (flags->all_done) return;
  const int64_t e0 = ((int64_t)blockIdx.x * VT + threadIdx.x) * 4;
  const int64_t stride = (int64_t)gridDim.x * VW;
  int c[4];
  thread_columns(t, e0, c);
  float be[4], mx[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int q = 0; q < 4; ++q) be[q] = beta[c[q]];
  for (int64_t e = e0; e < total; e += stride) {
    const f32x4 r = *reinterpret_cast<const f32x4*>(R + e);
    f32x4 p = *reinterpret_cast<const f32x4*>(P + e);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      p[q] = fmaf(be[q], p[q], r[q]);
      mx[q] = fmaxf(mx[q], fabsf(p[q]));
    }
    *reinterpret_cast<f32x4*>(P + e) = p;
  }
  block_column_max(mx, c, t, colmax, smax);   // max |P| per column for the next product (zeroed by the beta finalise)
}

// dV <- X (columns whose right-hand side is zero get 0)
__global__ __launch_bounds__(VT) void cg_store_kernel(const float* __restrict__ X, int64_t n, int t,
                                                      const int* __restrict__ zero_rhs, float* __restrict__ V,
                                                      int64_t ldv) {
  const int64_t total = n * t;
  for (int64_t e = (int64_t)blockIdx.x * VT + threadIdx.x; e < total; e += (int64_t)gridDim.x * VT) {
    const int64_t i = e / t;
    const int c = (int)(e - i * t);
    V[i * ldv + c] = zero_rhs[c] ? 0.0f : X[e];
  }
}

// ---- one-workgroup finalise kernels --------------------------------------
// column sums of the [G][t] workgroup partials, fixed order; result valid for tid < t
__device__ __forceinline__ double finalize_sum(const double* part, int G, int t, double* sh /* [FT] */) {
  const int tid = threadIdx.x;
  const int nparts = FT / t > 0 ? FT / t : 1;
  const int c = tid % t, pt = tid / t;
  // four independent partial sums keep several loads in flight (the order stays fixed)
  double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
  if (pt < nparts) {
    int g = pt;
    for (; g + 3 * nparts < G; g += 4 * nparts) {
      s0 += part[(int64_t)g * t + c];
      s1 += part[(int64_t)(g + nparts) * t + c];
      s2 += part[(int64_t)(g + 2 * nparts) * t + c];
      s3 += part[(int64_t)(g + 3 * nparts) * t + c];
    }
    for (; g < G; g += nparts) s0 += part[(int64_t)g * t + c];
  }
  const double s = (s0 + s1) + (s2 + s3);
  __syncthreads();
  sh[tid] = s;
  __syncthreads();
  double tot = 0.0;
  if (tid < t)
    for (int k = 0; k < nparts; ++k) tot += sh[k * t + c];
  return tot;
}

// Copy the flags to the host mirror; seq goes last, behind a system-scope fence, so that a host that
// sees the new seq also sees the flags that belong to it.  One thread.
__device__ __forceinline__ void post_flags(const CgDev& s, int seq) {
  volatile CgFlags* h = s.post;
  h->all_done = s.flags->all_done;
  h->breakdown = s.flags->breakdown;
  h->iters = s.flags->iters;
  __threadfence_system();
  h->seq = seq;
}

__global__ __launch_bounds__(FT) void cg_fin_init_kernel(CgDev s, int G, int t, int have_bn2) {
  __shared__ double sh[FT];
  __shared__ int live_count;
  if (threadIdx.x == 0) live_count = 0;
  double bn2 = 0.0;
  if (have_bn2) bn2 = finalize_sum(s.part2, G, t, sh);
  const double rho = finalize_sum(s.part, G, t, sh);
  const int c = threadIdx.x;
  if (c < t) {
    if (have_bn2) s.bn2[c] = bn2; else bn2 = s.bn2[c];
    const int zero = !(bn2 > 0.0);
    const double rel = zero ? 0.0 : sqrt(rho / bn2);
    const int fr = zero || rel < (double)s.tol[c];
    s.rho[c] = rho;
    s.relres[c] = (float)rel;
    s.zero_rhs[c] = zero;
    s.frozen[c] = fr;
    s.alpha[c] = 0.0f;
    s.beta[c] = 0.0f;
    if (!fr) atomicAdd(&live_count, 1);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    s.flags->all_done = live_count == 0;
    s.flags->breakdown = 0;
    s.flags->iters = 0;
    __threadfence();
    post_flags(s, 1);
  }
}

__global__ __launch_bounds__(FT) void cg_fin_alpha_kernel(CgDev s, int G, int t) {
  __shared__ double sh[FT];
  if (s.flags->all_done) return;
  const double gamma = finalize_sum(s.part, G, t, sh);
  const int c = threadIdx.x;
  if (c < t) {
    float al = 0.0f;
    if (!s.frozen[c]) {
      if (!(gamma > 0.0) || !isfinite(gamma)) {
        s.flags->breakdown = 1;
      } else {
        al = (float)(s.rho[c] / gamma);
      }
    }
    s.alpha[c] = al;
  }
}

__global__ __launch_bounds__(FT) void cg_fin_beta_kernel(CgDev s, int G, int t) {
  __shared__ double sh[FT];
  __shared__ int live_count;
  if (s.flags->all_done) return;
  if (threadIdx.x == 0) live_count = 0;
  const double rho_new = finalize_sum(s.part, G, t, sh);
  const int c = threadIdx.x;
  if (c < t) {
    float be = 0.0f;
    int fr = s.frozen[c];
    if (!fr) {
      const double rho = s.rho[c];
      const double rel = sqrt(rho_new / s.bn2[c]);
      if (!isfinite(rho_new)) s.flags->breakdown = 1;
      be = (float)(rho_new / rho);
      s.rho[c] = rho_new;
      s.relres[c] = (float)rel;
      fr = rel < (double)s.tol[c];
      s.frozen[c] = fr;
    }
    s.beta[c] = be;
    s.colmax[c] = 0u;          // the p update that follows accumulates the new column maxima
    if (!fr) atomicAdd(&live_count, 1);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    s.flags->iters += 1;
    if (live_count == 0 || s.flags->breakdown) s.flags->all_done = 1;
    __threadfence();
    post_flags(s, s.flags->iters + 1);
  }
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct CgLayout {
  int64_t n4;
  int G;
  size_t off_X, off_R, off_P, off_HP, off_state, off_part, off_part2, off_kmv, total;
  size_t kmv_bytes;
};

CgLayout cg_layout(const gp_ctx* ctx, int t) {
  CgLayout L;
  L.n4 = (ctx->n + GP_VEC_PAD - 1) / GP_VEC_PAD * GP_VEC_PAD;
  // grid of the streaming kernels: a multiple of t workgroups, enough to fill the chip on large
  // problems, fewer on small ones (about 8 float4 per thread) so the finalise kernels sum fewer partials
  const int64_t total4 = L.n4 * (int64_t)t / 4;
  int64_t per = (total4 + (int64_t)VT * 8 * t - 1) / ((int64_t)VT * 8 * t);
  const int per_max = (2 * ctx->num_cu + t - 1) / t;
  if (per > per_max) per = per_max;
  if (per < 1) per = 1;
  L.G = t * (int)per;
  const size_t arr = align_up((size_t)L.n4 * t * sizeof(float), 256);
  size_t o = 0;
  L.off_X = o; o += arr;
  L.off_R = o; o += arr;
  L.off_P = o; o += arr;
  L.off_HP = o; o += arr;
  L.off_state = o; o += align_up(sizeof(CgFlags) + (size_t)t * (2 * sizeof(double) + 4 * sizeof(float) + 3 * sizeof(int)) + 256, 256);
  L.off_part = o; o += align_up((size_t)L.G * t * sizeof(double), 256);
  L.off_part2 = o; o += align_up((size_t)L.G * t * sizeof(double), 256);
  L.off_kmv = o;
  L.kmv_bytes = align_up(gp_kmv_scratch_bytes(ctx, t), 256);
  o += L.kmv_bytes;
  L.total = o;
  return L;
}

}  // namespace

size_t gp_cg_workspace_bytes(const gp_ctx* ctx, int t) { return cg_layout(ctx, t).total; }

int gp_cg_run(gp_ctx* ctx, const float* dB, int64_t ldb, const float* dX0, float* dV, int64_t ldv, int t,
              const float* h_tol, int max_iters, void* dWork, size_t work_bytes, int* h_iters,
              int* h_kmv_count, float* h_relres) {
  const CgLayout L = cg_layout(ctx, t);
  if (work_bytes < L.total) return gp_fail(ctx, GP_ERR_WORKSPACE, "gp_cg_solve: workspace %zu < %zu bytes", work_bytes, L.total);
  if ((uintptr_t)dWork % 256) return gp_fail(ctx, GP_ERR_WORKSPACE, "gp_cg_solve: workspace not 256-byte aligned");
  hipStream_t st = ctx->stream;
  char* w = (char*)dWork;
  float* X = (float*)(w + L.off_X);
  float* R = (float*)(w + L.off_R);
  float* P = (float*)(w + L.off_P);
  float* HP = (float*)(w + L.off_HP);
  CgDev s;
  {
    char* q = w + L.off_state;
    s.flags = (CgFlags*)q; q += sizeof(CgFlags);
    s.rho = (double*)q; q += sizeof(double) * t;
    s.bn2 = (double*)q; q += sizeof(double) * t;
    s.alpha = (float*)q; q += sizeof(float) * t;
    s.beta = (float*)q; q += sizeof(float) * t;
    s.tol = (float*)q; q += sizeof(float) * t;
    s.relres = (float*)q; q += sizeof(float) * t;
    s.frozen = (int*)q; q += sizeof(int) * t;
    s.zero_rhs = (int*)q; q += sizeof(int) * t;
    s.colmax = (unsigned*)q; q += sizeof(unsigned) * t;
  }
  s.part = (double*)(w + L.off_part);
  s.part2 = (double*)(w + L.off_part2);
  void* kmv_scratch = w + L.off_kmv;
  const int64_t total = L.n4 * t;
  const dim3 grid(L.G), block(VT);

  // staging through pinned memory: tolerances in, flags and residuals out
  const size_t need_pinned = sizeof(CgFlags) + sizeof(float) * t * 2;
  if (need_pinned > GP_PIN_THETA) return gp_fail(ctx, GP_ERR_ARG, "gp_cg_solve: t too large for the pinned staging block");
  // this region is written by the host only here; every solver synchronises the stream before it
  // returns, so the copy a previous call queued from it has run (gp_set_theta stages elsewhere)
  CgFlags* hflags = (CgFlags*)((char*)ctx->hPinned + GP_PIN_SOLVER);
  float* htol = (float*)(hflags + 1);
  float* hrel = htol + t;
  for (int c = 0; c < t; ++c) htol[c] = h_tol[c];
  GP_HIP(ctx, hipMemcpyAsync(s.tol, htol, sizeof(float) * t, hipMemcpyHostToDevice, st));
  // HP padding rows are never written by the product; keep them zero
  GP_HIP(ctx, hipMemsetAsync(HP, 0, (size_t)total * sizeof(float), st));

  // The finalise kernels post the flags into pinned host memory themselves (no copy command in the
  // stream between iterations); the host polls the sequence number, and checks the stream now and
  // then so that a failed launch or a missing post ends the wait instead of hanging it.
  CgFlags* hpost = (CgFlags*)((char*)ctx->hPinned + GP_PIN_POST);
  s.post = (CgFlags*)((char*)ctx->dPinned + GP_PIN_POST);
  hpost->seq = 0;
  auto wait_seq = [&](int want) -> int {
    volatile CgFlags* h = hpost;
    for (unsigned spins = 1;; ++spins) {
      if (h->seq >= want) break;
      if ((spins & 4095u) == 0) {
        const hipError_t q = hipStreamQuery(st);
        if (q == hipSuccess) {          // nothing left to run: the post must be there by now
          if (h->seq >= want) break;
          return gp_fail(ctx, GP_ERR_HIP, "gp_cg_solve: the solver kernels did not report their state");
        }
        if (q != hipErrorNotReady) return gp_fail(ctx, GP_ERR_HIP, "gp_cg_solve: %s", hipGetErrorString(q));
      }
    }
    __atomic_thread_fence(__ATOMIC_ACQUIRE);
    return GP_OK;
  };

  // an error return leaves nothing of this solve running: kernels queued so far would otherwise post
  // their flags into the next solve's sequence
  auto drained = [&](int rc) -> int {
    (void)hipStreamSynchronize(st);
    return rc;
  };

  int kmv_count = 0;
  // the load kernel leaves max |X0| per column for the warm start's product, whose column-split
  // partials the residual kernel sums itself
  KmvDeferred df0 = {nullptr, 0, 1};
  if (dX0) GP_HIP(ctx, hipMemsetAsync(s.colmax, 0, sizeof(unsigned) * t, st));
  hipLaunchKernelGGL(cg_load_kernel, grid, block, 0, st, dB, ldb, dX0, ldv, ctx->n, L.n4, t, X, R, s.part2, s.colmax);
  GP_HIP(ctx, hipGetLastError());
  if (dX0) {
    int rc = gp_kmv_launch(ctx, X, t, t, HP, t, 1, kmv_scratch, L.kmv_bytes, s.colmax, nullptr, &df0);
    if (rc < 0) return drained(rc);
    ++kmv_count;
  }
  GP_HIP(ctx, hipMemsetAsync(s.colmax, 0, sizeof(unsigned) * t, st));
  hipLaunchKernelGGL(cg_resid_kernel, grid, block, 0, st, R, (const float*)HP, df0.part, df0.stride, df0.JS,
                     ctx->n * (int64_t)t, dX0 ? 1 : 0, P, total, t, s.part, s.colmax);
  hipLaunchKernelGGL(cg_fin_init_kernel, dim3(1), dim3(FT), 0, st, s, L.G, t, 1);
  GP_HIP(ctx, hipGetLastError());
  {
    const int rc = wait_seq(1);
    if (rc < 0) return drained(rc);
  }

  int it = 0;
  while (!hpost->all_done && it < max_iters) {
    KmvDeferred df = {nullptr, 0, 1};
    int rc = gp_kmv_launch(ctx, P, t, t, HP, t, 1, kmv_scratch, L.kmv_bytes, s.colmax, nullptr, &df);
    if (rc < 0) return drained(rc);
    ++kmv_count;
    bool pr = gp_prof_begin(ctx, GP_PROF_CG_DOT);
    hipLaunchKernelGGL(cg_dot_kernel, grid, block, 0, st, (const float*)P, HP, df.part, df.stride, df.JS,
                       ctx->n * (int64_t)t, total, t, s.flags, s.part);
    gp_prof_end(ctx, pr);
    hipLaunchKernelGGL(cg_fin_alpha_kernel, dim3(1), dim3(FT), 0, st, s, L.G, t);
    pr = gp_prof_begin(ctx, GP_PROF_CG_XR);
    hipLaunchKernelGGL(cg_update_xr_kernel, grid, block, 0, st, X, R, (const float*)P, (const float*)HP, total, t,
                       (const float*)s.alpha, s.flags, s.part);
    gp_prof_end(ctx, pr);
    hipLaunchKernelGGL(cg_fin_beta_kernel, dim3(1), dim3(FT), 0, st, s, L.G, t);
    pr = gp_prof_begin(ctx, GP_PROF_CG_P);
    hipLaunchKernelGGL(cg_update_p_kernel, grid, block, 0, st, P, (const float*)R, total, t, (const float*)s.beta, s.flags, s.colmax);
    gp_prof_end(ctx, pr);
    GP_HIP(ctx, hipGetLastError());
    rc = wait_seq(it + 2);
    if (rc < 0) return drained(rc);
    ++it;
  }

  int sblocks = (int)((ctx->n * (int64_t)t + VT - 1) / VT);
  if (sblocks > 8 * ctx->num_cu) sblocks = 8 * ctx->num_cu;
  hipLaunchKernelGGL(cg_store_kernel, dim3(sblocks), block, 0, st, (const float*)X, ctx->n, t, (const int*)s.zero_rhs, dV, ldv);
  GP_HIP(ctx, hipGetLastError());
  GP_HIP(ctx, hipMemcpyAsync(hrel, s.relres, sizeof(float) * t, hipMemcpyDeviceToHost, st));
  GP_HIP(ctx, hipMemcpyAsync(hflags, s.flags, sizeof(CgFlags), hipMemcpyDeviceToHost, st));
  GP_HIP(ctx, hipStreamSynchronize(st));
  if (h_iters) *h_iters = hflags->iters;
  if (h_kmv_count) *h_kmv_count = kmv_count;
  if (h_relres)
    for (int c = 0; c < t; ++c) h_relres[c] = hrel[c];
  if (hflags->breakdown) return gp_fail(ctx, GP_ERR_BREAKDOWN, "gp_cg_solve: p^T H p <= 0 or non-finite value at iteration %d", hflags->iters);
  // all_done is also raised by a breakdown; reaching here it means every column met its tolerance
  return hflags->all_done ? GP_OK : GP_NOT_CONVERGED;
}
