// Marginal-likelihood gradient estimator, matrix-free (paper Section 2: the
// gradient equation; Section 2.1: trace replaced by the s-probe estimator and
// the solves v = H^{-1} b).  With
//   A_i = [ v_y,i / 2, -v_1,i / (2s), .., -v_s,i / (2s) ]   C_j = [ v_y,j, z_1,j, .., z_s,j ]
// the estimator is  g_k = sum_ij w_ij (dH/dtheta_k)_ij  with  w_ij = A_i . C_j.
// For both kernels dK_ij/d ell_k = a^2 psi_ij (xs_ik - xs_jk)^2 / ell_k with
//   psi = exp(-r^2/2) (SE),  psi = 3 exp(-sqrt(3) r) (Matern-3/2; r cancels, so
//   coincident points give 0 and not 0/0),
// and expanding the square turns the lengthscale gradients into row sums of one
// more matrix-free product G Q, G = w .* psi, Q = [xs, xs^2, 1]:
//   g_ell_k = a^2/ell_k sum_i ( xs_ik^2 (G 1)_i + (G xs^2)_ik - 2 xs_ik (G xs)_ik )
//   g_a     = 2 a sum_ij w_ij K_ij / a^2     (one extra column carried on the VALU)
//   g_sigma = 2 sigma sum_i w_ii
// The tile pass is the K V pass with a second MFMA chain for w in front of the
// elementwise stage.
#include "gpws_internal.h"

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr int GRAD_TBLOCK = 66;   // right-hand-side columns handled per tile pass (KT = 33 k-steps)

struct GradArgs {
  const float* XA;
  const float* XB;
  const float* CA;     // packed column-side C rows, [chunk][KT][64]
  const float* AB;     // packed row-side A rows
  const float* Q;      // n x ldq
  int64_t ldq;
  float* OUT;          // [JS][n][ldo]
  int64_t ldo;
  int64_t split_stride;
  int64_t n;
  int nchunks;
  int col0;            // first Q column of this pass
  int ncols;
  int vcol;            // output column for sum_j w_ij K_ij / a^2, or -1
  int JS;
  int cps;
};

template <int KIND, int KS, int KT, int NT>
__global__ __launch_bounds__(GP_THREADS) void grad_tile_kernel(GradArgs p) {
  constexpr int NC = 32 * NT;
  constexpr int XA_F = KS * 64;
  constexpr int CA_F = KT * 64;
  constexpr int XA_LD = (XA_F + GP_THREADS - 1) / GP_THREADS;
  constexpr int CA_LD = (CA_F + GP_THREADS - 1) / GP_THREADS;
  constexpr int CA_OFF = XA_LD * GP_THREADS;       // operand regions rounded up: unguarded staging
  constexpr int V_OFF = CA_OFF + CA_LD * GP_THREADS;
  constexpr int STAGE = V_OFF + 32 * NC;
  __shared__ __attribute__((aligned(16))) float lds[2][STAGE];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: lets the compiler branch on it
  const int h = lane >> 5;
  const int li = lane & 31;
  const int js = blockIdx.x % p.JS;
  const int rb = blockIdx.x / p.JS;
  const int sub0 = rb * GP_WAVES + wave;

  const int c_begin = js * p.cps;
  const int c_end = min(p.nchunks, c_begin + p.cps);

  float xb[KS], ab[KT];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) xb[ks] = p.XB[((int64_t)sub0 * KS + ks) * 64 + lane];
#pragma unroll
  for (int ks = 0; ks < KT; ++ks) ab[ks] = p.AB[((int64_t)sub0 * KT + ks) * 64 + lane];

  f32x16 acc[NT];
  float accv = 0.0f;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nt][r] = 0.0f;

  // staging: unconditional loads, rows clamped to n-1 (padding rows of XA make psi exactly 0),
  // columns clamped into the pass (their accumulator columns are never stored)
  float gxa[XA_LD], gca[CA_LD];
  f32x4 gv[NT];
  const int ld_jq = tid >> 5;
  const int ld_c = tid & 31;
  const int jmax = (int)(p.n - 1);
  int col_off[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) col_off[nt] = p.col0 + min(ld_c + 32 * nt, p.ncols - 1);

  auto load_chunk = [&](int ch) {
    const float* xa = p.XA + (int64_t)ch * XA_F;
    const float* ca = p.CA + (int64_t)ch * CA_F;
#pragma unroll
    for (int u = 0; u < XA_LD; ++u) gxa[u] = xa[tid + u * GP_THREADS];
#pragma unroll
    for (int u = 0; u < CA_LD; ++u) gca[u] = ca[tid + u * GP_THREADS];
    const int j0 = ch * 32 + 4 * ld_jq;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float* row = p.Q + (int64_t)min(j0 + q, jmax) * p.ldq;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) gv[nt][q] = row[col_off[nt]];
    }
  };
  auto store_chunk = [&](int st) {
    float* s = lds[st];
#pragma unroll
    for (int u = 0; u < XA_LD; ++u) s[tid + u * GP_THREADS] = gxa[u];
#pragma unroll
    for (int u = 0; u < CA_LD; ++u) s[CA_OFF + tid + u * GP_THREADS] = gca[u];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      *reinterpret_cast<f32x4*>(&s[V_OFF + (ld_jq * NC + ld_c + 32 * nt) * 4]) = gv[nt];
  };

  load_chunk(c_begin);
  store_chunk(0);
  __syncthreads();

  for (int ch = c_begin; ch < c_end; ++ch) {
    const int st = (ch - c_begin) & 1;
    if (ch + 1 < c_end) load_chunk(ch + 1);
    const float* s = lds[st];

    f32x16 S, W;
#pragma unroll
    for (int r = 0; r < 16; ++r) { S[r] = 0.0f; W[r] = 0.0f; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      S = __builtin_amdgcn_mfma_f32_32x32x2f32(s[ks * 64 + lane], xb[ks], S, 0, 0, 0);
#pragma unroll
    for (int ks = 0; ks < KT; ++ks)
      W = __builtin_amdgcn_mfma_f32_32x32x2f32(s[CA_OFF + ks * 64 + lane], ab[ks], W, 0, 0, 0);
    if (ch == sub0) {
      asm volatile("" ::: "memory");   // keeps this a real (wave-uniform) branch instead of selects on every chunk
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (8 * (r >> 2) + 4 * h + (r & 3) == li) S[r] = 0.0f;
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int jq = 2 * g + h;
      f32x4 vb[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        vb[nt] = *reinterpret_cast<const f32x4*>(&s[V_OFF + (jq * NC + li + 32 * nt) * 4]);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int r = 4 * g + q;
        float psi, kval;
        if (KIND == GP_SE_ARD) {
          psi = __builtin_amdgcn_exp2f(S[r]);
          kval = psi;
        } else {
          const float u = __builtin_amdgcn_sqrtf(fmaxf(S[r], 0.0f));
          const float e = __builtin_amdgcn_exp2f(-LOG2E * u);
          psi = 3.0f * e;
          kval = fmaf(u, e, e);
        }
        const float gval = W[r] * psi;
        accv = fmaf(W[r], kval, accv);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(gval, vb[nt][q], acc[nt], 0, 0, 0);
      }
    }
    if (ch + 1 < c_end) store_chunk(st ^ 1);
    __syncthreads();
  }

  float* out = p.OUT + (int64_t)js * p.split_stride;
  const int64_t ibase = (int64_t)sub0 * 32;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int c = li + 32 * nt;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t i = ibase + 8 * (r >> 2) + 4 * h + (r & 3);
      if (i < p.n && c < p.ncols) out[i * p.ldo + p.col0 + c] = acc[nt][r];
    }
  }
  if (p.vcol >= 0) {
    const float tot = accv + __shfl_xor(accv, 32);
    const int64_t i = ibase + li;
    if (h == 0 && i < p.n) out[i * p.ldo + p.vcol] = tot;
  }
}

// Q = [xs, xs^2, 1], n x (2d+1)
__global__ void grad_build_q_kernel(const float* __restrict__ Xs, int64_t n, int d, float* __restrict__ Q) {
  const int ldq = 2 * d + 1;
  const int64_t total = n * ldq;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int64_t i = e / ldq;
    const int c = (int)(e - i * ldq);
    float v = 1.0f;
    if (c < d) v = Xs[i * d + c];
    else if (c < 2 * d) { const float x = Xs[i * d + c - d]; v = x * x; }
    Q[e] = v;
  }
}

// packed operands of the w chain for right-hand-side columns [t0, t0 + tb)
__global__ void grad_pack_ac_kernel(const float* __restrict__ V, int64_t ldv, const float* __restrict__ B,
                                    int64_t ldb, int64_t n, int64_t n_pad, int t0, int tb, int KT, float half_w,
                                    float probe_w, float* __restrict__ CA, float* __restrict__ AB) {
  const int64_t total = n_pad * 2 * KT;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    // e = (chunk*KT + ks)*64 + lane
    const int lane = (int)(e & 63);
    const int64_t ck = e >> 6;
    const int ks = (int)(ck % KT);
    const int64_t chunk = ck / KT;
    const int64_t row = chunk * 32 + (lane & 31);
    const int m = 2 * ks + (lane >> 5);
    float c = 0.0f, a = 0.0f;
    if (row < n && m < tb) {
      const int col = t0 + m;
      const float v = V[row * ldv + col];
      if (col == 0) { c = v; a = half_w * v; }
      else { c = B[row * ldb + col]; a = probe_w * v; }
    }
    CA[e] = c;
    AB[e] = a;
  }
}

// per-workgroup fp64 partial sums of the d + 2 gradient components
__global__ __launch_bounds__(256) void grad_reduce_kernel(const float* __restrict__ OUT, int64_t split_stride,
                                                          int JS, int64_t ldo, const float* __restrict__ Xs,
                                                          int64_t n, int d, const float* __restrict__ V,
                                                          int64_t ldv, const float* __restrict__ B, int64_t ldb,
                                                          int t, float half_w, float probe_w, int first_block,
                                                          double* __restrict__ part /* [grid][d+2] */) {
  extern __shared__ double sh[];   // [256]
  const int nq = 2 * d + 2;
  // thread <-> (row, component): consecutive threads take consecutive components of a row;
  // components 0..d-1 are the lengthscales, d the amplitude
  const int ncomp = d + 1;
  double* mypart = part + (int64_t)blockIdx.x * (d + 2);
  for (int comp0 = 0; comp0 < ncomp; comp0 += 256) {
    const int comp = comp0 + (threadIdx.x % min(256, ncomp - comp0));
    const int lanes_per_row = min(256, ncomp - comp0);
    const int rows_per_step = 256 / lanes_per_row;
    const int rsub = threadIdx.x / lanes_per_row;
    double s = 0.0;
    if (rsub < rows_per_step) {
      for (int64_t i = (int64_t)blockIdx.x * rows_per_step + rsub; i < n; i += (int64_t)gridDim.x * rows_per_step) {
        if (comp < d) {
          float y = 0.f, t2 = 0.f, t1 = 0.f;
#pragma unroll 4
          for (int k = 0; k < JS; ++k) {
            const float* o = OUT + (int64_t)k * split_stride + i * ldo;
            y += o[comp]; t2 += o[d + comp]; t1 += o[2 * d];
          }
          const double x = (double)Xs[i * d + comp];
          s += x * x * (double)t1 + (double)t2 - 2.0 * x * (double)y;
        } else {
          float ga = 0.f;
#pragma unroll 4
          for (int k = 0; k < JS; ++k) ga += OUT[(int64_t)k * split_stride + i * ldo + nq - 1];
          s += (double)ga;
        }
      }
    }
    // fixed-order reduction over the rows handled by this workgroup
    __syncthreads();
    sh[threadIdx.x] = s;
    __syncthreads();
    if (rsub == 0 && threadIdx.x < lanes_per_row) {
      double tot = 0.0;
      for (int r = 0; r < rows_per_step; ++r) tot += sh[r * lanes_per_row + threadIdx.x];
      mypart[comp] = tot;
    }
  }
  // noise component: sum_i w_ii = sum_i A_i . C_i over all t columns, the workgroup's threads sharing
  // the elements of 8 rows at a time; fixed-order tree at the end
  double w = 0.0;
  if (first_block) {
    constexpr int RPS = 8;
    for (int64_t base = (int64_t)blockIdx.x * RPS; base < n; base += (int64_t)gridDim.x * RPS) {
      const int rows = (int)min((int64_t)RPS, n - base);
      const int cnt = rows * t;
      for (int e = threadIdx.x; e < cnt; e += 256) {
        const int r = e / t, c = e - r * t;
        const int64_t i = base + r;
        const double v = (double)V[i * ldv + c];
        w += c == 0 ? (double)half_w * v * v : (double)probe_w * v * (double)B[i * ldb + c];
      }
    }
  }
  __syncthreads();
  sh[threadIdx.x] = w;
  __syncthreads();
  for (int k = 128; k > 0; k >>= 1) {
    if ((int)threadIdx.x < k) sh[threadIdx.x] += sh[threadIdx.x + k];
    __syncthreads();
  }
  if (threadIdx.x == 0) mypart[d + 1] = sh[0];
}

// acc[comp] += sum over workgroup partials; one workgroup per component, fixed-order tree
__global__ __launch_bounds__(256) void grad_finalize_kernel(const double* __restrict__ part, int G, int ncomp,
                                                            double* __restrict__ acc) {
  __shared__ double sh[256];
  const int c = blockIdx.x;
  double s = 0.0;
  for (int g = threadIdx.x; g < G; g += 256) s += part[(int64_t)g * ncomp + c];
  sh[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) acc[c] += sh[0];
}

typedef void (*grad_fn)(GradArgs);

// two N-tiles need two LDS stages of (KS + KT)*64 + 2048 floats; the largest bucket only fits one
constexpr int grad_max_nt(int KS) { return KS >= 64 ? 1 : 2; }

template <int KIND, int KS>
grad_fn pick_kt_nt(int KT, int NT) {
  if constexpr (grad_max_nt(KS) >= 2) {
    if (NT == 2) return KT == 9 ? grad_tile_kernel<KIND, KS, 9, 2> : grad_tile_kernel<KIND, KS, 33, 2>;
  }
  return KT == 9 ? grad_tile_kernel<KIND, KS, 9, 1> : grad_tile_kernel<KIND, KS, 33, 1>;
}

template <int KIND>
grad_fn pick_grad(int KS, int KT, int NT) {
  switch (KS) {
    case 4: return pick_kt_nt<KIND, 4>(KT, NT);
    case 7: return pick_kt_nt<KIND, 7>(KT, NT);
    case 10: return pick_kt_nt<KIND, 10>(KT, NT);
    case 14: return pick_kt_nt<KIND, 14>(KT, NT);
    case 24: return pick_kt_nt<KIND, 24>(KT, NT);
    case 46: return pick_kt_nt<KIND, 46>(KT, NT);
    case 64: return pick_kt_nt<KIND, 64>(KT, NT);
  }
  return nullptr;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

int gp_grad_reduce_launch(gp_ctx* ctx, const float* OUT, int64_t split_stride, int JS, int nq, const float* dV,
                          int64_t ldv, const float* dB, int64_t ldb, int t, float half_w, float probe_w,
                          int first_block, double* part, int G, double* acc) {
  const int d = ctx->d;
  hipLaunchKernelGGL(grad_reduce_kernel, dim3(G), dim3(256), 256 * sizeof(double), ctx->stream, OUT, split_stride, JS,
                     (int64_t)nq, (const float*)ctx->dXs, ctx->n, d, dV, ldv, dB, ldb, t, half_w, probe_w, first_block,
                     part);
  hipLaunchKernelGGL(grad_finalize_kernel, dim3(d + 2), dim3(256), 0, ctx->stream, (const double*)part, G, d + 2, acc);
  GP_HIP(ctx, hipGetLastError());
  return GP_OK;
}

int gp_grad_run(gp_ctx* ctx, const float* dV, int64_t ldv, const float* dB, int64_t ldb, int t,
                double* h_grad) {
  if (ctx->path != GP_PATH_FP32) return gp_grad_run_f16(ctx, dV, ldv, dB, ldb, t, h_grad);
  const int d = ctx->d;
  const int64_t n = ctx->n;
  const int nq = 2 * d + 2;         // Q columns (2d+1) + the VALU column
  const int ldq = 2 * d + 1;
  const int s = t - 1;
  const float half_w = 0.5f;
  const float probe_w = s > 0 ? (float)(-0.5 / (double)s) : 0.0f;

  // plan: one 32-row sub-tile per wave, column range split until the chip is full
  const int64_t chunks = (n + 31) / 32;
  const int row_blocks = (int)((n + 127) / 128);
  int JS = 1;
  const int target = 2 * ctx->num_cu;
  if (row_blocks < target) {
    JS = (target + row_blocks - 1) / row_blocks;
    const int64_t max_js = chunks / 4 > 0 ? chunks / 4 : 1;
    if (JS > max_js) JS = (int)max_js;
    if (JS > 64) JS = 64;
  }
  const int cps = (int)((chunks + JS - 1) / JS);
  JS = (int)((chunks + cps - 1) / cps);

  const int KTmax = t <= 18 ? 9 : 33;
  // workgroups of the fp64 reduction: one step of 256 / (d + 2) rows each when n allows, so that
  // enough loads are in flight (the kernel is latency-bound at small n)
  int G;
  {
    const int per_step = 256 / (d + 2 < 256 ? d + 2 : 256);
    const int64_t want = (n + per_step - 1) / per_step;
    G = (int)(want < 8 * ctx->num_cu ? want : 8 * ctx->num_cu);
    if (G < 1) G = 1;
  }
  const size_t q_bytes = align_up((size_t)n * ldq * sizeof(float), 256);
  const size_t op_bytes = align_up(((size_t)(ctx->n_pad / 32) * KTmax * 64 + GP_PACK_SLACK) * sizeof(float), 256);
  const size_t out_bytes = align_up((size_t)JS * n * nq * sizeof(float), 256);
  const size_t part_bytes = align_up((size_t)G * (d + 2) * sizeof(double), 256);
  const size_t acc_bytes = align_up((size_t)(d + 2) * sizeof(double), 256);
  int rc = gp_ensure_scratch(ctx, q_bytes + 2 * op_bytes + out_bytes + part_bytes + acc_bytes);
  if (rc < 0) return rc;
  char* w = (char*)ctx->dScratch;
  float* Q = (float*)w; w += q_bytes;
  float* CA = (float*)w; w += op_bytes;
  float* AB = (float*)w; w += op_bytes;
  float* OUT = (float*)w; w += out_bytes;
  double* part = (double*)w; w += part_bytes;
  double* acc = (double*)w;
  hipStream_t st = ctx->stream;

  GP_HIP(ctx, hipMemsetAsync(acc, 0, acc_bytes, st));
  {
    const int64_t total = n * ldq;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 8 * ctx->num_cu) blocks = 8 * ctx->num_cu;
    hipLaunchKernelGGL(grad_build_q_kernel, dim3(blocks), dim3(256), 0, st, (const float*)ctx->dXs, n, d, Q);
    GP_HIP(ctx, hipGetLastError());
  }

  GradArgs a;
  a.XA = ctx->dXA;
  a.XB = ctx->dXB;
  a.CA = CA;
  a.AB = AB;
  a.Q = Q;
  a.ldq = ldq;
  a.OUT = OUT;
  a.ldo = nq;
  a.split_stride = n * (int64_t)nq;
  a.n = n;
  a.nchunks = (int)chunks;
  a.JS = JS;
  a.cps = cps;
  const dim3 grid(row_blocks * JS), block(GP_THREADS);

  for (int t0 = 0; t0 < t; t0 += GRAD_TBLOCK) {
    const int tb = t - t0 < GRAD_TBLOCK ? t - t0 : GRAD_TBLOCK;
    const int KT = tb <= 18 ? 9 : 33;
    {
      const int64_t total = ctx->n_pad * 2 * KT;
      int blocks = (int)((total + 255) / 256);
      if (blocks > 8 * ctx->num_cu) blocks = 8 * ctx->num_cu;
      hipLaunchKernelGGL(grad_pack_ac_kernel, dim3(blocks), dim3(256), 0, st, dV, ldv, dB, ldb, n, ctx->n_pad, t0, tb,
                         KT, half_w, probe_w, CA, AB);
      GP_HIP(ctx, hipGetLastError());
    }
    int vcol = nq - 1;
    for (int c = 0; c < ldq;) {
      const int rem = ldq - c;
      const int NT = (rem > 32 && grad_max_nt(ctx->KS) >= 2) ? 2 : 1;
      a.col0 = c;
      a.ncols = rem < 32 * NT ? rem : 32 * NT;
      a.vcol = vcol;
      vcol = -1;
      grad_fn fn = ctx->kernel == GP_SE_ARD ? pick_grad<GP_SE_ARD>(ctx->KS, KT, NT)
                                            : pick_grad<GP_MATERN32_ARD>(ctx->KS, KT, NT);
      if (!fn) return gp_fail(ctx, GP_ERR_ARG, "gp_mll_grad: no kernel for KS=%d", ctx->KS);
      const bool pr = gp_prof_begin(ctx, GP_PROF_GRAD_TILE);
      hipLaunchKernelGGL(fn, grid, block, 0, st, a);
      gp_prof_end(ctx, pr);
      GP_HIP(ctx, hipGetLastError());
      c += a.ncols;
    }
    rc = gp_grad_reduce_launch(ctx, OUT, a.split_stride, JS, nq, dV, ldv, dB, ldb, t, half_w, probe_w, t0 == 0 ? 1 : 0,
                               part, G, acc);
    if (rc < 0) return rc;
  }

  double* hacc = (double*)ctx->hPinned;
  GP_HIP(ctx, hipMemcpyAsync(hacc, acc, sizeof(double) * (d + 2), hipMemcpyDeviceToHost, st));
  GP_HIP(ctx, hipStreamSynchronize(st));
  const double a2 = ctx->a * ctx->a;
  for (int k = 0; k < d; ++k) h_grad[k] = a2 / ctx->ell[k] * hacc[k];
  h_grad[d] = 2.0 * ctx->a * hacc[d];
  h_grad[d + 1] = 2.0 * ctx->sigma * hacc[d + 1];
  return GP_OK;
}
