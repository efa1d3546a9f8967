// Matrix-free product OUT = K V (+ sigma^2 V) for ARD squared-exponential and
// Matern-3/2 kernels on gfx950: the product inside every solver iteration of
// the batched system of paper Section 2.1.  K is never stored.
//
// Per 32x32 tile of pairs (j, i), one wavefront does
//   1. S[j][i] = XA_j . XB_i          KS x v_mfma_f32_32x32x2_f32   (= g r^2_ij)
//   2. phi = exp2(S)                  (SE)   or (1+u) exp2(-log2e u), u = sqrt(max(S,0))  (Matern-3/2)
//   3. OUT_i += phi[i][j] V_j         16*NT x v_mfma_f32_32x32x2_f32
// The accumulator layout of step 1 (lane = i, register r <-> j) is exactly the
// A-operand layout step 3 needs once the V rows are fetched in the matching
// order, so phi never leaves registers.  One extra column (y, when t = 32q+1)
// is carried on the VALU so that t = 65 does not pay for a third MFMA N-tile.
#include "gpws_internal.h"

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

struct TileArgs {
  const float* XA;
  const float* XB;
  const float* V;
  int64_t ldv;
  float* OUT;
  int64_t ldo;
  int64_t split_stride;   // elements between consecutive split partials
  int64_t n;              // points on the column side (the context's n)
  int64_t nrows;          // rows of the output (n, or m for a rectangular product)
  int diag;               // square product: the pair (i, i) gets r^2 = 0 exactly
  int nchunks;            // ceil(n / 32)
  int col0;               // first column of V on the MFMA
  int ncols;              // MFMA columns in this pass (<= 32*NT)
  int vcol;               // column carried on the VALU, or -1
  int JS;
  int cps;                // chunks per split
  float a2;
  float sigma2;
  int add_noise;
};

constexpr float LOG2E = 1.4426950408889634f;

template <int KIND>
__device__ __forceinline__ float phi_of(float s) {
  if (KIND == GP_SE_ARD) {
    return __builtin_amdgcn_exp2f(s);             // s = -log2(e)/2 r^2
  } else {
    float u = __builtin_amdgcn_sqrtf(fmaxf(s, 0.0f));   // s = 3 r^2
    float e = __builtin_amdgcn_exp2f(-LOG2E * u);
    return fmaf(u, e, e);
  }
}

template <int KIND, int KS, int NT, int MI>
__global__ __launch_bounds__(GP_THREADS) void kmv_tile_kernel(TileArgs p) {
  constexpr int NC = 32 * NT;
  constexpr int XA_F = KS * 64;
  constexpr int XA_LD = (XA_F + GP_THREADS - 1) / GP_THREADS;
  constexpr int V_OFF = XA_LD * GP_THREADS;        // XA region rounded up so its staging needs no guard
  constexpr int VY_OFF = V_OFF + 32 * NC;
  constexpr int STAGE = VY_OFF + 32;
  __shared__ __attribute__((aligned(16))) float lds[2][STAGE];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: lets the compiler branch on it
  const int h = lane >> 5;
  const int li = lane & 31;
  const int js = blockIdx.x % p.JS;
  const int rb = blockIdx.x / p.JS;
  const int sub0 = (rb * GP_WAVES + wave) * MI;     // first 32-row sub-tile of this wave

  // The workgroup's column range [r_begin, r_end) is walked in segments [c_begin, c_end) of at most
  // GP_FLUSH_CHUNKS chunks; the accumulators are added into OUT after each segment (see flush below).
  const int r_begin = js * p.cps;
  const int r_end = min(p.nchunks, r_begin + p.cps);
  int c_begin = r_begin;
  int c_end = min(r_end, c_begin + GP_FLUSH_CHUNKS);

  // row-side operands stay in registers for the whole pass
  float xb[MI][KS];
#pragma unroll
  for (int m = 0; m < MI; ++m)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) xb[m][ks] = p.XB[((int64_t)(sub0 + m) * KS + ks) * 64 + lane];

  f32x16 acc[MI][NT];
  float accv[MI];
#pragma unroll
  for (int m = 0; m < MI; ++m) {
    accv[m] = 0.0f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[m][nt][r] = 0.0f;
  }

  // Staging of the next chunk.  Every load is unconditional: row indices are clamped to n-1 and
  // column indices into the pass's range.  Rows j >= n of XA carry a huge squared norm, so phi is
  // exactly 0 for them whatever V row was read; clamped columns land in accumulator columns that
  // are never stored.
  float gxa[XA_LD];
  f32x4 gv[NT];
  float gvy = 0.0f;
  const int ld_jq = tid >> 5;        // 0..7 : group of 4 consecutive rows j
  const int ld_c = tid & 31;
  const int jmax = (int)(p.n - 1);
  int col_off[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) col_off[nt] = p.col0 + min(ld_c + 32 * nt, p.ncols - 1);
  const int vy_off = p.vcol >= 0 ? p.vcol : 0;

  auto load_chunk = [&](int ch) {
    const float* xa = p.XA + (int64_t)ch * XA_F;
#pragma unroll
    for (int u = 0; u < XA_LD; ++u) gxa[u] = xa[tid + u * GP_THREADS];
    const int j0 = ch * 32 + 4 * ld_jq;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float* row = p.V + (int64_t)min(j0 + q, jmax) * p.ldv;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) gv[nt][q] = row[col_off[nt]];
    }
    gvy = p.V[(int64_t)min(ch * 32 + (tid & 31), jmax) * p.ldv + vy_off];
  };
  auto store_chunk = [&](int st) {
    float* s = lds[st];
#pragma unroll
    for (int u = 0; u < XA_LD; ++u) s[tid + u * GP_THREADS] = gxa[u];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      *reinterpret_cast<f32x4*>(&s[V_OFF + (ld_jq * NC + ld_c + 32 * nt) * 4]) = gv[nt];
    if (tid < 32) s[VY_OFF + tid] = gvy;
  };

  // Writes what the accumulators hold to OUT (first: stores a^2 acc plus the noise term once; later:
  // adds to what is there) and clears them.  Doing so after every segment keeps the chains
  // of fp32 partial sums short; the same threads read and write the same elements, in a fixed order.
  float* out = p.OUT + (int64_t)js * p.split_stride;
  auto flush = [&](bool first) {
    const bool noise = first && p.add_noise && js == 0;
    // an opaque zero keeps the address arithmetic of the flush inside it: hoisted out of the segment
    // loop it would hold dozens of registers across the main loop
    int zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(zero));
#pragma unroll
    for (int m = 0; m < MI; ++m) {
      const int64_t ibase = (int64_t)(sub0 + m) * 32 + zero;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int c = li + 32 * nt;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t i = ibase + 8 * (r >> 2) + 4 * h + (r & 3);
          if (i < p.nrows && c < p.ncols) {
            float v = p.a2 * acc[m][nt][r];
            if (noise) v = fmaf(p.sigma2, p.V[i * p.ldv + p.col0 + c], v);
            if (!first) v += out[i * p.ldo + p.col0 + c];
            out[i * p.ldo + p.col0 + c] = v;
          }
          acc[m][nt][r] = 0.0f;
        }
      }
      if (p.vcol >= 0) {
        const float tot = accv[m] + __shfl_xor(accv[m], 32);
        const int64_t i = ibase + li;
        if (h == 0 && i < p.nrows) {
          float v = p.a2 * tot;
          if (noise) v = fmaf(p.sigma2, p.V[i * p.ldv + p.vcol], v);
          if (!first) v += out[i * p.ldo + p.vcol];
          out[i * p.ldo + p.vcol] = v;
        }
        accv[m] = 0.0f;
      }
    }
  };
  bool first = true;

  for (;;) {
  // every split owns at least one chunk (the launcher sizes JS that way), so the prologue is
  // unconditional; its wait for the staged chunk also retires the xb loads above
  load_chunk(c_begin);
  store_chunk(0);
  __syncthreads();
  for (int ch = c_begin; ch < c_end; ++ch) {
    const int st = (ch - c_begin) & 1;
    if (ch + 1 < c_end) load_chunk(ch + 1);

    const float* s = lds[st];
    f32x16 S[MI];
#pragma unroll
    for (int m = 0; m < MI; ++m)
#pragma unroll
      for (int r = 0; r < 16; ++r) S[m][r] = 0.0f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const float xa = s[ks * 64 + lane];
#pragma unroll
      for (int m = 0; m < MI; ++m) S[m] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa, xb[m][ks], S[m], 0, 0, 0);
    }
    // the pair (i, i): r^2 is exactly zero
#pragma unroll
    for (int m = 0; m < MI; ++m) {
      if (p.diag && ch == sub0 + m) {
        // one chunk in thousands: an opaque statement keeps this a real (wave-uniform) branch instead of
        // sixteen selects executed on every chunk
        asm volatile("" ::: "memory");
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (8 * (r >> 2) + 4 * h + (r & 3) == li) S[m][r] = 0.0f;
      }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int jq = 2 * g + h;
      const f32x4 vy4 = *reinterpret_cast<const f32x4*>(&s[VY_OFF + 4 * jq]);
      f32x4 vb[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        vb[nt] = *reinterpret_cast<const f32x4*>(&s[V_OFF + (jq * NC + li + 32 * nt) * 4]);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int m = 0; m < MI; ++m) {
          const float ph = phi_of<KIND>(S[m][4 * g + q]);
          accv[m] = fmaf(ph, vy4[q], accv[m]);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            acc[m][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(ph, vb[nt][q], acc[m][nt], 0, 0, 0);
        }
      }
    }
    if (ch + 1 < c_end) store_chunk(st ^ 1);
    __syncthreads();
  }
  flush(first);
  first = false;
  if (c_end >= r_end) break;
  c_begin = c_end;
  c_end = min(r_end, c_begin + GP_FLUSH_CHUNKS);
  }
}

// OUT[i][c] = sum_js PART[js][i][c] for c in [c_lo, c_hi)
__global__ void kmv_reduce_kernel(const float* __restrict__ part, int64_t split_stride, int JS, int64_t n,
                                  int t, float* __restrict__ out, int64_t ldo) {
  const int64_t total = n * t;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int64_t i = e / t;
    const int c = (int)(e - i * t);
    float s = 0.0f;
    for (int k = 0; k < JS; ++k) s += part[(int64_t)k * split_stride + e];
    out[i * ldo + c] = s;
  }
}

typedef void (*tile_fn)(TileArgs);

template <int KIND, int KS>
tile_fn pick_nt_mi(int NT, int MI) {
  if (NT == 1) return MI == 1 ? kmv_tile_kernel<KIND, KS, 1, 1> : kmv_tile_kernel<KIND, KS, 1, 2>;
  return MI == 1 ? kmv_tile_kernel<KIND, KS, 2, 1> : kmv_tile_kernel<KIND, KS, 2, 2>;
}

template <int KIND>
tile_fn pick_ks(int KS, int NT, int MI) {
  switch (KS) {
    case 4: return pick_nt_mi<KIND, 4>(NT, MI);
    case 7: return pick_nt_mi<KIND, 7>(NT, MI);
    case 10: return pick_nt_mi<KIND, 10>(NT, MI);
    case 14: return pick_nt_mi<KIND, 14>(NT, MI);
    case 24: return pick_nt_mi<KIND, 24>(NT, MI);
    case 46: return pick_nt_mi<KIND, 46>(NT, MI);
    case 64: return pick_nt_mi<KIND, 64>(NT, MI);
  }
  return nullptr;
}

}  // namespace

int gp_ks_bucket(int d) {
  const int need = (d + 2 + 1) / 2;
  const int buckets[] = {4, 7, 10, 14, 24, 46, 64};
  for (int b : buckets)
    if (need <= b) return b;
  return -1;
}

KmvPlan gp_plan_kmv(const gp_ctx* ctx, int64_t rows, int64_t col_chunks) {
  KmvPlan pl;
  const int64_t chunks = col_chunks > 0 ? col_chunks : (ctx->n + 31) / 32;
  // two sub-tiles per wave once there are enough rows to fill the chip that way
  pl.MI = (ctx->KS <= 24 && rows >= 8192) ? 2 : 1;
  const int rows_per_wg = 32 * GP_WAVES * pl.MI;
  pl.row_blocks = (int)((rows + rows_per_wg - 1) / rows_per_wg);
  const int target = 2 * ctx->num_cu;
  int JS = 1;
  if (pl.row_blocks < target) {
    JS = (target + pl.row_blocks - 1) / pl.row_blocks;
    const int64_t max_js = chunks / 4 > 0 ? chunks / 4 : 1;   // keep at least 4 chunks per split
    if (JS > max_js) JS = (int)max_js;
    if (JS > 64) JS = 64;
  }
  pl.cps = (int)((chunks + JS - 1) / JS);
  pl.JS = (int)((chunks + pl.cps - 1) / pl.cps);
  return pl;
}

size_t gp_kmv_rect_scratch_bytes(const gp_ctx* ctx, int t, int64_t rows) {
  KmvPlan pl = gp_plan_kmv(ctx, rows);
  const size_t fp32_bytes = pl.JS <= 1 ? 0 : (size_t)pl.JS * (size_t)rows * (size_t)t * sizeof(float);
  const size_t f16_bytes = gp_kmv_f16_scratch_bytes(ctx, t, rows);
  return fp32_bytes > f16_bytes ? fp32_bytes : f16_bytes;
}

size_t gp_kmv_scratch_bytes(const gp_ctx* ctx, int t) { return gp_kmv_rect_scratch_bytes(ctx, t, ctx->n); }

// Scratch for a product over any column window of at most col_chunks chunks.  The number of column
// splits is not monotone in the window's length (65 chunks are cut into 13 ranges of 5, 64 chunks into
// 16 ranges of 4), so every length is planned.
size_t gp_kmv_window_scratch_bytes(const gp_ctx* ctx, int t, int col_chunks) {
  size_t need = 0;
  for (int c = 1; c <= col_chunks; ++c) {
    const KmvPlan pl = gp_plan_kmv(ctx, ctx->n, c);
    const size_t fp32_bytes = pl.JS <= 1 ? 0 : (size_t)pl.JS * (size_t)ctx->n * (size_t)t * sizeof(float);
    const size_t f16_bytes = gp_kmv_f16_scratch_bytes(ctx, t, ctx->n, c);
    if (fp32_bytes > need) need = fp32_bytes;
    if (f16_bytes > need) need = f16_bytes;
  }
  return need;
}

int gp_kmv_launch(gp_ctx* ctx, const float* dV, int64_t ldv, int t, float* dOut, int64_t ldo,
                  int add_noise, void* scratch, size_t scratch_bytes, const unsigned* colmax, const KmvRows* rows,
                  KmvDeferred* defer, const KmvWindow* win) {
  if (rows && add_noise) return gp_fail(ctx, GP_ERR_ARG, "rectangular product with a noise term");
  const int64_t all_chunks = (ctx->n + 31) / 32;
  if (win && (add_noise || rows || win->chunk0 < 0 || win->nchunks < 1 || (int64_t)win->chunk0 + win->nchunks > all_chunks))
    return gp_fail(ctx, GP_ERR_ARG, "gp_kmv: bad column window");
  if ((rows ? rows->path : ctx->path) != GP_PATH_FP32)
    return gp_kmv_launch_f16(ctx, dV, ldv, t, dOut, ldo, add_noise, scratch, scratch_bytes, colmax, rows, defer, win);
  const int64_t nrows = rows ? rows->m : ctx->n;
  const KmvPlan pl = gp_plan_kmv(ctx, nrows, win ? win->nchunks : 0);
  const bool split = pl.JS > 1;
  if (split && scratch_bytes < (size_t)pl.JS * (size_t)nrows * (size_t)t * sizeof(float))
    return gp_fail(ctx, GP_ERR_WORKSPACE, "gp_kmv: scratch too small for %d column splits", pl.JS);

  TileArgs a;
  a.XA = ctx->dXA;
  a.XB = rows ? rows->XB : ctx->dXB;
  a.V = dV;
  a.ldv = ldv;
  a.OUT = split ? (float*)scratch : dOut;
  a.ldo = split ? t : ldo;
  a.split_stride = split ? nrows * (int64_t)t : 0;
  a.n = ctx->n;
  a.nrows = nrows;
  a.diag = rows ? 0 : 1;
  a.nchunks = (int)all_chunks;
  if (win) {   // the kernel sees the window as a point set of its own, starting at chunk 0
    const int64_t first = (int64_t)win->chunk0 * 32;
    const int64_t stop = first + (int64_t)win->nchunks * 32;
    a.XA = ctx->dXA + (int64_t)win->chunk0 * ctx->KS * 64;
    a.V = dV + first * ldv;
    a.n = (stop < ctx->n ? stop : ctx->n) - first;
    a.nchunks = win->nchunks;
    a.diag = 0;
  }
  a.JS = pl.JS;
  a.cps = pl.cps;
  a.a2 = (float)(ctx->a * ctx->a);
  a.sigma2 = (float)(ctx->sigma * ctx->sigma);
  a.add_noise = add_noise;

  // column passes: optional VALU column (when t = 32q + 1, q >= 1), then MFMA groups of <= 64
  int vcol = (t > 1 && t % 32 == 1) ? 0 : -1;
  int c = vcol >= 0 ? 1 : 0;
  const dim3 grid(pl.row_blocks * pl.JS), block(GP_THREADS);
  while (c < t) {
    const int rem = t - c;
    const int NT = rem > 32 ? 2 : 1;
    a.col0 = c;
    a.ncols = rem < 32 * NT ? rem : 32 * NT;
    a.vcol = vcol;
    vcol = -1;   // carried by the first pass only
    tile_fn fn = ctx->kernel == GP_SE_ARD ? pick_ks<GP_SE_ARD>(ctx->KS, NT, pl.MI)
                                          : pick_ks<GP_MATERN32_ARD>(ctx->KS, NT, pl.MI);
    if (!fn) return gp_fail(ctx, GP_ERR_ARG, "gp_kmv: no kernel for KS=%d", ctx->KS);
    const bool prof = gp_prof_begin(ctx, GP_PROF_TILE);
    hipLaunchKernelGGL(fn, grid, block, 0, ctx->stream, a);
    GP_HIP(ctx, hipGetLastError());
    gp_prof_end(ctx, prof);
    c += a.ncols;
  }
  if (defer) {
    defer->part = (const float*)scratch;
    defer->stride = a.split_stride;
    defer->JS = pl.JS;
  }
  if (split && !defer) {
    const int64_t total = nrows * (int64_t)t;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 4 * ctx->num_cu) blocks = 4 * ctx->num_cu;
    hipLaunchKernelGGL(kmv_reduce_kernel, dim3(blocks), dim3(256), 0, ctx->stream, (const float*)scratch,
                       a.split_stride, pl.JS, nrows, t, dOut, ldo);
    GP_HIP(ctx, hipGetLastError());
  }
  return GP_OK;
}
