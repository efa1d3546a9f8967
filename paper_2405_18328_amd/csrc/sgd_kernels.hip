// Stochastic gradient descent as the linear system solver (Section 2.1 lists it beside conjugate
// gradients and alternating projections; Appendix B fixes mini-batches of 1000 data points, momentum
// 0.9, no iterate averaging, and a residual vector that is kept in memory and refreshed on the
// mini-batch rows only).
//
// One step, all t columns sharing the mini-batch I (distinct row indices supplied by the caller):
//   G = H[I,:] U - B[I,:];  R[I,:] = -G;  M = rho M;  M[I,:] -= (lr / |I|) G;  U += M.
// H[I,:] U is the tile pass with the batch's rows on the row side (their packed operands are gathered
// from the context's own packed arrays, 16 bytes at a time) and all n points on the column side.
// The squared norm of the residual estimate is kept per column in fp64 and corrected by
// sum_I (new^2 - old^2) each step, so the stopping test needs no pass over R.
// All sums have a fixed order; the only atomics are integer maxima.
#include <math.h>
#include <stdint.h>

#include "gpws_internal.h"
#include "col_streams.h"

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

struct SgdFlags {
  int all_done;
  int bad;          // 1: non-finite residual, 2: a batch index outside [0, n)
  int iters;
  int seq;          // host mirror only: finalise steps posted so far (written last)
};

struct SgdDev {
  SgdFlags* flags;
  SgdFlags* post;   // pinned host memory
  double* rr;       // [t] squared norm of the residual estimate
  double* bn2;      // [t]
  float* tol;       // [t]
  float* relres;    // [t]
  int* frozen;      // [t]
  int* zero_rhs;    // [t]
  unsigned* colmax; // [t] bit patterns of max |U| per column for the split-fp16 product
  double* part;     // [GW][t] workgroup partials
  double* part2;    // [GW][t]
};

__device__ __forceinline__ int clamp_index(int v, int64_t n, int* bad) {
  if (v < 0 || v >= n) {
    *bad = 2;
    return 0;
  }
  return v;
}

// rows [r0, r1) of workgroup w out of gridDim.x
__device__ __forceinline__ void wg_rows(int64_t n, int64_t* r0, int64_t* r1) {
  const int64_t per = (n + gridDim.x - 1) / gridDim.x;
  *r0 = (int64_t)blockIdx.x * per;
  const int64_t e = *r0 + per;
  *r1 = e < n ? e : n;
  if (*r0 > n) *r0 = n;
}

// U <- X0 (or 0), M <- 0, R <- B - HX0 (or B); partial squared norms of B and R; max |U| per column
__global__ __launch_bounds__(256) void sgd_init_kernel(const float* __restrict__ B, int64_t ldb,
                                                       const float* __restrict__ X0, int64_t ldx,
                                                       const float* __restrict__ HX0, int64_t n, int t,
                                                       float* __restrict__ U, float* __restrict__ M,
                                                       float* __restrict__ R, double* __restrict__ partB,
                                                       double* __restrict__ partR, unsigned* __restrict__ colmax) {
  __shared__ float red[256];
  int64_t r0, r1;
  wg_rows(n, &r0, &r1);
  const ColMap m = col_map(t);
  for (int cg = 0; cg < t; cg += m.tw) {
    const int c = cg + m.cl;
    const bool valid = c < t && m.rl < m.lanes;
    float accb = 0.0f, accr = 0.0f, mx = 0.0f;
    if (valid) {
      for (int64_t i = r0 + m.rl; i < r1; i += m.lanes) {
        const int64_t e = i * t + c;
        const float b = B[i * ldb + c];
        const float x = X0 ? X0[i * ldx + c] : 0.0f;
        const float r = X0 ? b - HX0[e] : b;
        U[e] = x;
        M[e] = 0.0f;
        R[e] = r;
        accb = fmaf(b, b, accb);
        accr = fmaf(r, r, accr);
        mx = fmaxf(mx, fabsf(x));
      }
      if (mx > 0.0f) atomicMax(&colmax[c], __float_as_uint(mx));   // once per solve: straight to memory
    }
    store_column_sums(m, valid, accb, cg, t, red, partB + (int64_t)blockIdx.x * t);
    store_column_sums(m, valid, accr, cg, t, red, partR + (int64_t)blockIdx.x * t);
  }
}

// packed row operands of the batch: slot s of the batch takes the place of row s.  fp32 operands:
// float (chunk * KS + ks) * 64 + lane belongs to row 32 chunk + lane % 32; fp16 operands: 16-byte unit
// (chunk * KH + kh) * 64 + lane likewise.  Slots past the batch repeat slot 0 (their output rows are
// never stored).
__global__ __launch_bounds__(256) void sgd_gather_kernel(const int* __restrict__ I, int b, int b_pad, int64_t n,
                                                         const float* __restrict__ srcXB, int KS,
                                                         const u32x4* __restrict__ s0, const u32x4* __restrict__ s1,
                                                         const u32x4* __restrict__ s2, int KH,
                                                         float* __restrict__ dstXB, u32x4* __restrict__ d0,
                                                         u32x4* __restrict__ d1, u32x4* __restrict__ d2,
                                                         const SgdFlags* __restrict__ flags, int* __restrict__ bad) {
  if (flags->all_done) return;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t n32 = (int64_t)(b_pad / 32) * KS * 64;
  const int64_t n16 = (int64_t)(b_pad / 32) * KH * 64;
  if (gid < n32) {
    const int lane = (int)(gid & 63);
    const int64_t q = gid >> 6;
    const int ks = (int)(q % KS);
    const int chunk = (int)(q / KS);
    const int slot = 32 * chunk + (lane & 31);
    const int idx = clamp_index(I[slot < b ? slot : 0], n, bad);
    dstXB[gid] = srcXB[((int64_t)(idx >> 5) * KS + ks) * 64 + (lane & 32) + (idx & 31)];
  }
  if (gid < n16) {
    const int lane = (int)(gid & 63);
    const int64_t q = gid >> 6;
    const int kh = (int)(q % KH);
    const int chunk = (int)(q / KH);
    const int slot = 32 * chunk + (lane & 31);
    const int idx = clamp_index(I[slot < b ? slot : 0], n, bad);
    const int64_t src = ((int64_t)(idx >> 5) * KH + kh) * 64 + (lane & 32) + (idx & 31);
    d0[gid] = s0[src];
    d1[gid] = s1[src];
    d2[gid] = s2[src];
  }
}

// On the batch rows: G = (H U)[I] - B[I] with the product's result (column-split partials summed here
// when JS > 1) plus sigma^2 U[I]; R[I] <- -G; Gs <- (lr / b) G for the columns still being updated
// (0 for the others); per-workgroup sums of new^2 - old^2 of the residual estimate.  Workgroup 0 also
// clears the column maxima, which the product has consumed by now.
__global__ __launch_bounds__(256) void sgd_batch_kernel(const int* __restrict__ I, int b, int64_t n, int t,
                                                        const float* __restrict__ OUT, const float* __restrict__ part,
                                                        int64_t stride, int JS, const float* __restrict__ U,
                                                        const float* __restrict__ B, int64_t ldb, float sigma2,
                                                        float step, float* __restrict__ R, float* __restrict__ Gs,
                                                        const int* __restrict__ frozen, unsigned* __restrict__ colmax,
                                                        const SgdFlags* __restrict__ flags, int* __restrict__ bad,
                                                        double* __restrict__ delta) {
  __shared__ double red[256];
  if (flags->all_done) return;
  if (blockIdx.x == 0)
    for (int c = threadIdx.x; c < t; c += 256) colmax[c] = 0u;
  int64_t r0, r1;
  wg_rows(b, &r0, &r1);
  const ColMap m = col_map(t);
  for (int cg = 0; cg < t; cg += m.tw) {
    const int c = cg + m.cl;
    const bool valid = c < t && m.rl < m.lanes;
    double acc = 0.0;
    if (valid) {
      const bool live = !frozen[c];
      for (int64_t s = r0 + m.rl; s < r1; s += m.lanes) {
        const int64_t e = s * t + c;
        const int64_t i = clamp_index(I[s], n, bad);
        float hx;
        if (JS > 1) {
          float h0 = 0.0f, h1 = 0.0f, h2 = 0.0f, h3 = 0.0f;      // four chains so that the loads overlap
          int q = 0;
          for (; q + 3 < JS; q += 4) {
            h0 += part[(int64_t)q * stride + e];
            h1 += part[(int64_t)(q + 1) * stride + e];
            h2 += part[(int64_t)(q + 2) * stride + e];
            h3 += part[(int64_t)(q + 3) * stride + e];
          }
          for (; q < JS; ++q) h0 += part[(int64_t)q * stride + e];
          hx = (h0 + h1) + (h2 + h3);
        } else {
          hx = OUT[e];
        }
        hx = fmaf(sigma2, U[i * t + c], hx);
        const float g = hx - B[i * ldb + c];
        if (live) {
          const float old = R[i * t + c];
          R[i * t + c] = -g;
          acc += (double)g * (double)g - (double)old * (double)old;
          Gs[e] = step * g;
        } else {
          Gs[e] = 0.0f;
        }
      }
    }
    if (m.rl < m.lanes) red[m.rl * m.tw + m.cl] = valid ? acc : 0.0;
    __syncthreads();
    if ((int)threadIdx.x < m.tw && cg + (int)threadIdx.x < t) {
      double sum = 0.0;
      for (int l = 0; l < m.lanes; ++l) sum += red[l * m.tw + threadIdx.x];
      delta[(int64_t)blockIdx.x * t + cg + threadIdx.x] = sum;
    }
    __syncthreads();
  }
}

// M <- rho M (0 for columns no longer updated), U += M; max |U| per column
__global__ __launch_bounds__(256) void sgd_stream_kernel(float* __restrict__ U, float* __restrict__ M, int64_t n, int t,
                                                         float rho, const int* __restrict__ frozen,
                                                         unsigned* __restrict__ colmax,
                                                         const SgdFlags* __restrict__ flags) {
  __shared__ unsigned smax[GP_MAX_T];
  if (flags->all_done) return;
  for (int c = threadIdx.x; c < t; c += 256) smax[c] = 0u;
  __syncthreads();
  int64_t r0, r1;
  wg_rows(n, &r0, &r1);
  const ColMap m = col_map(t);
  for (int cg = 0; cg < t; cg += m.tw) {
    const int c = cg + m.cl;
    if (c < t && m.rl < m.lanes) {
      const float f = frozen[c] ? 0.0f : rho;
      float mx = 0.0f;
      for (int64_t i = r0 + m.rl; i < r1; i += m.lanes) {
        const int64_t e = i * t + c;
        const float mm = f * M[e];
        const float u = U[e] + mm;
        M[e] = mm;
        U[e] = u;
        mx = fmaxf(mx, fabsf(u));
      }
      if (mx > 0.0f) atomicMax(&smax[c], __float_as_uint(mx));
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < t; c += 256)
    if (smax[c]) atomicMax(&colmax[c], smax[c]);
}

// the batch rows' own part of the step: M[I] -= Gs, U[I] -= Gs (indices are distinct)
__global__ __launch_bounds__(256) void sgd_scatter_kernel(const int* __restrict__ I, int b, int64_t n, int t,
                                                          const float* __restrict__ Gs, float* __restrict__ U,
                                                          float* __restrict__ M, unsigned* __restrict__ colmax,
                                                          const SgdFlags* __restrict__ flags, int* __restrict__ bad) {
  __shared__ unsigned smax[GP_MAX_T];
  if (flags->all_done) return;
  for (int c = threadIdx.x; c < t; c += 256) smax[c] = 0u;
  __syncthreads();
  const int64_t total = (int64_t)b * t;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
    const int64_t s = e / t;
    const int c = (int)(e - s * t);
    const float g = Gs[e];
    if (g != 0.0f) {
      const int64_t i = clamp_index(I[s], n, bad);
      M[i * t + c] -= g;
      const float u = U[i * t + c] - g;
      U[i * t + c] = u;
      atomicMax(&smax[c], __float_as_uint(fabsf(u)));
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < t; c += 256)
    if (smax[c]) atomicMax(&colmax[c], smax[c]);
}

// scol[c] = sum over the G workgroup partials of column c: 1024 / t segments of the partials are summed
// side by side and combined in a fixed order (t <= 1024; blockDim = 1024)
__device__ void sgd_column_totals(const double* __restrict__ part, int G, int t, double* spart, double* scol) {
  const int tid = threadIdx.x;
  const int nseg = 1024 / t;
  const int per = (G + nseg - 1) / nseg;
  const int seg = tid / t, c = tid - seg * t;
  if (seg < nseg) {
    double v = 0.0;
    const int w1 = (seg + 1) * per < G ? (seg + 1) * per : G;
    for (int w = seg * per; w < w1; ++w) v += part[(int64_t)w * t + c];
    spart[seg * t + c] = v;
  }
  __syncthreads();
  if (tid < t) {
    double v = 0.0;
    for (int g = 0; g < nseg; ++g) v += spart[g * t + tid];
    scol[tid] = v;
  }
  __syncthreads();
}

// per-column state: sums the workgroup partials in order, applies the stopping rule, posts the flags
__global__ __launch_bounds__(1024) void sgd_finalise_kernel(SgdDev s, int G, int t, int init, const int* __restrict__ bad) {
  __shared__ double spart[1024];
  __shared__ double scol[GP_MAX_T];
  __shared__ double scolb[GP_MAX_T];
  __shared__ int s_any, s_bad;
  const int tid = threadIdx.x;
  if (!init && s.flags->all_done) return;
  if (tid == 0) {
    s_any = 0;
    s_bad = *bad;
  }
  if (init) sgd_column_totals(s.part2, G, t, spart, scolb);
  sgd_column_totals(s.part, G, t, spart, scol);
  if (tid < t) {
    const int c = tid;
    const double acc = scol[c];
    int fr;
    double rr;
    if (init) {
      const double accb = scolb[c];
      s.bn2[c] = accb;
      const int zero = accb == 0.0 ? 1 : 0;
      s.zero_rhs[c] = zero;
      fr = zero;
      rr = acc;
      if (zero) s.relres[c] = 0.0f;
    } else {
      fr = s.frozen[c];
      rr = s.rr[c] + (fr ? 0.0 : acc);
    }
    if (rr < 0.0) rr = 0.0;
    s.rr[c] = rr;
    if (!fr) {
      const double rel = sqrt(rr / s.bn2[c]);
      if (!(rel == rel) || rel > 3.0e38) atomicOr(&s_bad, 1);
      s.relres[c] = (float)rel;
      if ((float)rel < s.tol[c]) fr = 1;
    }
    s.frozen[c] = fr;
    if (!fr) atomicOr(&s_any, 1);
  }
  __syncthreads();
  if (tid == 0) {
    SgdFlags f = *s.flags;
    if (!init) f.iters += 1;
    if (s_bad) f.bad = s_bad;
    f.all_done = (!s_any || f.bad) ? 1 : 0;
    *s.flags = f;
    s.post->all_done = f.all_done;
    s.post->bad = f.bad;
    s.post->iters = f.iters;
    __threadfence_system();
    s.post->seq = f.iters + 1;
    __threadfence_system();
  }
}

__global__ __launch_bounds__(256) void sgd_store_kernel(const float* __restrict__ U, int64_t n, int t,
                                                        const int* __restrict__ zero_rhs, float* __restrict__ out,
                                                        int64_t ldo) {
  const int64_t total = n * t;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
    const int64_t i = e / t;
    const int c = (int)(e - i * t);
    out[i * ldo + c] = zero_rhs[c] ? 0.0f : U[e];
  }
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct SgdLayout {
  int GW, GB, b_pad;
  size_t off_U, off_M, off_R, off_HX, off_OUT, off_Gs, off_xb, off_h[3], off_state, off_part, off_part2, off_kmv, total;
  size_t kmv_bytes;
};

SgdLayout sgd_layout(const gp_ctx* ctx, int t, int batch) {
  SgdLayout L;
  L.b_pad = (batch + GP_ROW_ALIGN - 1) / GP_ROW_ALIGN * GP_ROW_ALIGN;
  // streaming grid: enough workgroups to fill the chip, at least about 8 rows each
  int64_t gw = (ctx->n + 7) / 8;
  if (gw > 2 * ctx->num_cu) gw = 2 * ctx->num_cu;
  if (gw < 1) gw = 1;
  L.GW = (int)gw;
  int64_t gb = ((int64_t)batch + 3) / 4;
  if (gb > ctx->num_cu) gb = ctx->num_cu;
  if (gb < 1) gb = 1;
  L.GB = (int)gb;
  const int G = L.GW > L.GB ? L.GW : L.GB;
  const size_t arr = align_up((size_t)ctx->n * t * sizeof(float), 256);
  const size_t barr = align_up((size_t)batch * t * sizeof(float), 256);
  const size_t p32 = align_up(((size_t)(L.b_pad / 32) * ctx->KS * 64 + GP_PACK_SLACK) * sizeof(float), 256);
  const size_t p16 = align_up((size_t)(L.b_pad / 32) * ctx->KH * 64 * 16 + 4096, 256);
  size_t o = 0;
  L.off_U = o; o += arr;
  L.off_M = o; o += arr;
  L.off_R = o; o += arr;
  L.off_HX = o; o += arr;
  L.off_OUT = o; o += barr;
  L.off_Gs = o; o += barr;
  L.off_xb = o; o += p32;
  for (int pc = 0; pc < 3; ++pc) { L.off_h[pc] = o; o += p16; }
  L.off_state = o; o += align_up(sizeof(SgdFlags) + 64 + (size_t)t * (2 * sizeof(double) + 2 * sizeof(float) + 3 * sizeof(int)) + 256, 256);
  L.off_part = o; o += align_up((size_t)G * t * sizeof(double), 256);
  L.off_part2 = o; o += align_up((size_t)G * t * sizeof(double), 256);
  L.off_kmv = o;
  size_t kb = gp_kmv_scratch_bytes(ctx, t);
  const size_t rb = gp_kmv_rect_scratch_bytes(ctx, t, batch);
  if (rb > kb) kb = rb;
  L.kmv_bytes = align_up(kb, 256);
  o += L.kmv_bytes;
  L.total = o;
  return L;
}

}  // namespace

size_t gp_sgd_workspace_bytes_impl(const gp_ctx* ctx, int t, int batch) { return sgd_layout(ctx, t, batch).total; }

int gp_sgd_run(gp_ctx* ctx, const float* dB, int64_t ldb, const float* dX0, float* dV, int64_t ldv, int t,
               const float* h_tol, const int* dBatches, int batch, int max_iters, double lr, double momentum,
               void* dWork, size_t work_bytes, int* h_iters, int* h_kmv_count, float* h_relres) {
  const SgdLayout L = sgd_layout(ctx, t, batch);
  if (work_bytes < L.total) return gp_fail(ctx, GP_ERR_WORKSPACE, "gp_sgd_solve: workspace %zu < %zu bytes", work_bytes, L.total);
  if ((uintptr_t)dWork % 256) return gp_fail(ctx, GP_ERR_WORKSPACE, "gp_sgd_solve: workspace not 256-byte aligned");
  hipStream_t st = ctx->stream;
  const int64_t n = ctx->n;
  char* w = (char*)dWork;
  float* U = (float*)(w + L.off_U);
  float* M = (float*)(w + L.off_M);
  float* R = (float*)(w + L.off_R);
  float* HX = (float*)(w + L.off_HX);
  float* OUT = (float*)(w + L.off_OUT);
  float* Gs = (float*)(w + L.off_Gs);
  float* gXB = (float*)(w + L.off_xb);
  u32x4* gH[3];
  for (int pc = 0; pc < 3; ++pc) gH[pc] = (u32x4*)(w + L.off_h[pc]);
  SgdDev s;
  int* bad;
  {
    char* q = w + L.off_state;
    s.flags = (SgdFlags*)q; q += sizeof(SgdFlags);
    bad = (int*)q; q += 64;
    s.rr = (double*)q; q += sizeof(double) * t;
    s.bn2 = (double*)q; q += sizeof(double) * t;
    s.tol = (float*)q; q += sizeof(float) * t;
    s.relres = (float*)q; q += sizeof(float) * t;
    s.frozen = (int*)q; q += sizeof(int) * t;
    s.zero_rhs = (int*)q; q += sizeof(int) * t;
    s.colmax = (unsigned*)q; q += sizeof(unsigned) * t;
  }
  s.part = (double*)(w + L.off_part);
  s.part2 = (double*)(w + L.off_part2);
  void* kmv_scratch = w + L.off_kmv;

  const size_t need_pinned = sizeof(SgdFlags) + sizeof(float) * t * 2;
  if (ctx->pinned_bytes < GP_PIN_POST + sizeof(SgdFlags) || need_pinned > GP_PIN_THETA)
    return gp_fail(ctx, GP_ERR_ARG, "gp_sgd_solve: t too large for the pinned staging block");
  SgdFlags* hflags = (SgdFlags*)((char*)ctx->hPinned + GP_PIN_SOLVER);
  float* htol = (float*)((char*)ctx->hPinned + GP_PIN_SOLVER + sizeof(SgdFlags));
  float* hrel = htol + t;
  GP_HIP(ctx, hipStreamSynchronize(st));   // the pinned block may still be in use by an earlier call
  for (int c = 0; c < t; ++c) htol[c] = h_tol[c];
  GP_HIP(ctx, hipMemsetAsync(w + L.off_state, 0, L.off_part - L.off_state, st));
  GP_HIP(ctx, hipMemcpyAsync(s.tol, htol, sizeof(float) * t, hipMemcpyHostToDevice, st));

  SgdFlags* hpost = (SgdFlags*)((char*)ctx->hPinned + GP_PIN_POST);
  s.post = (SgdFlags*)((char*)ctx->dPinned + GP_PIN_POST);
  hpost->all_done = 0;      // the mirror still holds the previous call's last post
  hpost->bad = 0;
  hpost->iters = 0;
  hpost->seq = 0;
  auto wait_seq = [&](int want) -> int {
    volatile SgdFlags* h = hpost;
    for (unsigned spins = 1;; ++spins) {
      if (h->seq >= want || h->all_done) break;
      if ((spins & 4095u) == 0) {
        const hipError_t q = hipStreamQuery(st);
        if (q == hipSuccess) {          // nothing left to run: the post must be there by now
          if (h->seq >= want || h->all_done) break;
          return gp_fail(ctx, GP_ERR_HIP, "gp_sgd_solve: the solver kernels did not report their state");
        }
        if (q != hipErrorNotReady) return gp_fail(ctx, GP_ERR_HIP, "gp_sgd_solve: %s", hipGetErrorString(q));
      }
    }
    __atomic_thread_fence(__ATOMIC_ACQUIRE);
    return GP_OK;
  };

  int kmv_count = 0;
  if (dX0) {
    const int rc = gp_kmv_launch(ctx, dX0, ldv, t, HX, t, 1, kmv_scratch, L.kmv_bytes, nullptr);
    if (rc < 0) return rc;
    ++kmv_count;
  }
  hipLaunchKernelGGL(sgd_init_kernel, dim3(L.GW), dim3(256), 0, st, dB, ldb, dX0, ldv, (const float*)HX, n, t, U, M, R,
                     s.part2, s.part, s.colmax);
  hipLaunchKernelGGL(sgd_finalise_kernel, dim3(1), dim3(1024), 0, st, s, L.GW, t, 1, (const int*)bad);
  GP_HIP(ctx, hipGetLastError());
  {
    const int rc = wait_seq(1);
    if (rc < 0) return rc;
  }

  KmvRows rows;
  rows.m = batch;
  rows.XB = gXB;
  for (int pc = 0; pc < 3; ++pc) rows.XBh[pc] = gH[pc];
  rows.path = ctx->path;
  const float sigma2 = (float)(ctx->sigma * ctx->sigma);
  const float step = (float)(lr / (double)batch);
  const int64_t units32 = (int64_t)(L.b_pad / 32) * ctx->KS * 64;
  const int64_t units16 = (int64_t)(L.b_pad / 32) * ctx->KH * 64;
  const int64_t gunits = units32 > units16 ? units32 : units16;
  int sblocks = (int)(((int64_t)batch * t + 255) / 256);
  if (sblocks > 2 * ctx->num_cu) sblocks = 2 * ctx->num_cu;

  // The stopping test runs on the device after every step and kernels of steps launched after it has
  // fired return at once; the host looks at the posted flags every POLL steps only.
  const int POLL = 16;
  int it = 0;
  while (!hpost->all_done && it < max_iters) {
    const int* I = dBatches + (int64_t)it * batch;
    hipLaunchKernelGGL(sgd_gather_kernel, dim3((unsigned)((gunits + 255) / 256)), dim3(256), 0, st, I, batch, L.b_pad, n,
                       (const float*)ctx->dXB, ctx->KS, (const u32x4*)ctx->dXBh[0], (const u32x4*)ctx->dXBh[1],
                       (const u32x4*)ctx->dXBh[2], ctx->KH, gXB, gH[0], gH[1], gH[2], (const SgdFlags*)s.flags, bad);
    GP_HIP(ctx, hipGetLastError());
    KmvDeferred df = {nullptr, 0, 1};
    const int rc = gp_kmv_launch(ctx, U, t, t, OUT, t, 0, kmv_scratch, L.kmv_bytes, s.colmax, &rows, &df);
    if (rc < 0) return rc;
    hipLaunchKernelGGL(sgd_batch_kernel, dim3(L.GB), dim3(256), 0, st, I, batch, n, t, (const float*)OUT, df.part, df.stride,
                       df.JS, (const float*)U, dB, ldb, sigma2, step, R, Gs, (const int*)s.frozen, s.colmax,
                       (const SgdFlags*)s.flags, bad, s.part);
    hipLaunchKernelGGL(sgd_stream_kernel, dim3(L.GW), dim3(256), 0, st, U, M, n, t, (float)momentum, (const int*)s.frozen,
                       s.colmax, (const SgdFlags*)s.flags);
    hipLaunchKernelGGL(sgd_scatter_kernel, dim3(sblocks), dim3(256), 0, st, I, batch, n, t, (const float*)Gs, U, M, s.colmax,
                       (const SgdFlags*)s.flags, bad);
    hipLaunchKernelGGL(sgd_finalise_kernel, dim3(1), dim3(1024), 0, st, s, L.GB, t, 0, (const int*)bad);
    GP_HIP(ctx, hipGetLastError());
    ++it;
    if (it % POLL == 0 || it == max_iters) {
      const int rc2 = wait_seq(it + 1);
      if (rc2 < 0) return rc2;
    }
  }

  int stb = (int)((n * (int64_t)t + 255) / 256);
  if (stb > 8 * ctx->num_cu) stb = 8 * ctx->num_cu;
  hipLaunchKernelGGL(sgd_store_kernel, dim3(stb), dim3(256), 0, st, (const float*)U, n, t, (const int*)s.zero_rhs, dV, ldv);
  GP_HIP(ctx, hipGetLastError());
  GP_HIP(ctx, hipMemcpyAsync(hrel, s.relres, sizeof(float) * t, hipMemcpyDeviceToHost, st));
  GP_HIP(ctx, hipMemcpyAsync(hflags, s.flags, sizeof(SgdFlags), hipMemcpyDeviceToHost, st));
  GP_HIP(ctx, hipStreamSynchronize(st));
  if (h_iters) *h_iters = hflags->iters;
  if (h_kmv_count) *h_kmv_count = kmv_count;
  if (h_relres)
    for (int c = 0; c < t; ++c) h_relres[c] = hrel[c];
  if (hflags->bad == 2) return gp_fail(ctx, GP_ERR_ARG, "gp_sgd_solve: a mini-batch index is outside [0, n)");
  if (hflags->bad) return gp_fail(ctx, GP_ERR_BREAKDOWN, "gp_sgd_solve: non-finite residual estimate at step %d (learning rate too large?)", hflags->iters);
  return hflags->all_done ? GP_OK : GP_NOT_CONVERGED;
}
