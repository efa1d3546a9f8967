// O(n d) preparation done at gp_create / gp_set_theta: column means of X and
// the packed, pre-scaled operand arrays the tile kernels read (layout in
// gpws_internal.h).  Distances are translation invariant, so centring only
// shrinks |xs|^2 and with it the rounding of the dot-form r^2.
#include <cstring>

#include "gpws_internal.h"

namespace {

// one workgroup per input dimension; fp64 accumulation
__global__ void column_mean_kernel(const float* __restrict__ X, int64_t n, int d, double* __restrict__ mean) {
  const int k = blockIdx.x;
  double s = 0.0;
  for (int64_t i = threadIdx.x; i < n; i += blockDim.x) s += (double)X[i * d + k];
  __shared__ double red[256];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) mean[k] = red[0] / (double)n;
}

// one workgroup per input dimension: max_i |x_ik - mean_k| (max is order-independent, so exact and reproducible)
__global__ void column_absdev_kernel(const float* __restrict__ X, int64_t n, int d, const double* __restrict__ mean,
                                     double* __restrict__ out) {
  const int k = blockIdx.x;
  const double mu = mean[k];
  double m = 0.0;
  for (int64_t i = threadIdx.x; i < n; i += blockDim.x) {
    const double v = fabs((double)X[i * d + k] - mu);
    m = (v > m || v != v) ? v : m;      // a NaN input propagates
  }
  __shared__ double red[256];
  red[threadIdx.x] = m;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) {
      const double o = red[threadIdx.x + w];
      if (o > red[threadIdx.x] || o != o) red[threadIdx.x] = o;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) out[k] = red[0];
}

// one thread per row: scaled centred row, its squared norm, and both packed operands
__global__ void pack_kernel(const float* __restrict__ X, int64_t n, int64_t n_pad, int d, int KS,
                            const double* __restrict__ mean, const double* __restrict__ theta /* 1/ell (d) */,
                            float gamma, float* __restrict__ XA, float* __restrict__ XB,
                            float* __restrict__ Xs, float* __restrict__ norm, unsigned* __restrict__ max_norm) {
  const int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= n_pad) return;
  const int64_t chunk = row >> 5;
  const int li = (int)(row & 31);
  float* xa = XA + chunk * KS * 64 + li;
  float* xb = XB + chunk * KS * 64 + li;
  const bool live = row < n;
  double nrm = 0.0;
  for (int k = 0; k < d; ++k) {
    float xs = 0.0f;
    if (live) {
      xs = (float)(((double)X[row * d + k] - mean[k]) * theta[k]);
      Xs[row * d + k] = xs;
      nrm += (double)xs * (double)xs;
    }
    const int off = (k >> 1) * 64 + (k & 1) * 32;
    xa[off] = xs;
    xb[off] = -2.0f * gamma * xs;
  }
  const float nf = (float)nrm;
  norm[row] = nf;
  if (live) atomicMax(max_norm, __float_as_uint(nf));     // non-negative floats order like unsigned ints
  for (int k = d; k < 2 * KS; ++k) {
    const int off = (k >> 1) * 64 + (k & 1) * 32;
    float va = 0.0f, vb = 0.0f;
    if (!live && k == d) va = GP_PAD_NORM;     // padding rows: r^2 is huge, the kernel value exactly 0
    if (live && k == d) { va = nf; vb = gamma; }
    if (live && k == d + 1) { va = 1.0f; vb = gamma * nf; }
    xa[off] = va;
    xb[off] = vb;
  }
}

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// x = hi + mid + lo with hi, mid truncated to 11 significant bits (exact in fp16), lo rounded
__device__ __forceinline__ void split3(float x, float& hi, float& mid, float& lo) {
  hi = __uint_as_float(__float_as_uint(x) & 0xFFFFE000u);
  const float r1 = x - hi;
  mid = __uint_as_float(__float_as_uint(r1) & 0xFFFFE000u);
  lo = r1 - mid;
}

// split-fp16 operands of the matrix-core path; one thread per (chunk, kh, lane)
__global__ void pack_f16_kernel(const float* __restrict__ Xs, const float* __restrict__ norm, int64_t n,
                                int64_t n_pad, int d, int KH, int is_se, float gamma, u32x4* __restrict__ A0,
                                u32x4* __restrict__ A1, u32x4* __restrict__ A2, u32x4* __restrict__ B0,
                                u32x4* __restrict__ B1, u32x4* __restrict__ B2) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (n_pad / 32) * KH * 64;
  if (gid >= total) return;
  const int lane = (int)(gid & 63);
  const int kh = (int)((gid >> 6) % KH);
  const int64_t chunk = (gid >> 6) / KH;
  const int64_t row = chunk * 32 + (lane & 31);
  const bool live = row < n;
  const float nf = norm[row];
  u32x4 a[3], b[3];
#pragma unroll
  for (int e2 = 0; e2 < 4; ++e2) {
    float pa[3][2], pb[3][2];
#pragma unroll
    for (int z = 0; z < 2; ++z) {
      const int k = 16 * kh + 8 * (lane >> 5) + 2 * e2 + z;
      float va = 0.0f, vb = 0.0f;
      if (live) {
        if (k < d) { const float xs = Xs[row * d + k]; va = xs; vb = -2.0f * gamma * xs; }
        else if (k == d) { va = nf; vb = gamma; }
        else if (k == d + 1) { va = 1.0f; vb = gamma * nf; }
        else if (k == d + 2 && is_se) { va = 1.0f; vb = 15.0f; }   // phi is carried as 2^15 phi
      } else if (k == d) {
        va = GP_PAD_NORM_H;
      }
      split3(va, pa[0][z], pa[1][z], pa[2][z]);
      split3(vb, pb[0][z], pb[1][z], pb[2][z]);
    }
#pragma unroll
    for (int pc = 0; pc < 3; ++pc) {
      a[pc][e2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(pa[pc][0], pa[pc][1]));
      b[pc][e2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(pb[pc][0], pb[pc][1]));
    }
  }
  A0[gid] = a[0]; A1[gid] = a[1]; A2[gid] = a[2];
  B0[gid] = b[0]; B1[gid] = b[1]; B2[gid] = b[2];
}

}  // namespace

int gp_launch_column_means(gp_ctx* ctx) {
  hipLaunchKernelGGL(column_mean_kernel, dim3(ctx->d), dim3(256), 0, ctx->stream, ctx->dX, ctx->n, ctx->d,
                     ctx->dMean);
  GP_HIP(ctx, hipGetLastError());
  // per-dimension spread, kept on the host: sum_k (xabs_k / ell_k)^2 bounds every scaled squared norm, which
  // lets gp_set_theta choose the product path without reading anything back in the common case
  double* dabs = ctx->dRed;
  hipLaunchKernelGGL(column_absdev_kernel, dim3(ctx->d), dim3(256), 0, ctx->stream, ctx->dX, ctx->n, ctx->d,
                     (const double*)ctx->dMean, dabs);
  GP_HIP(ctx, hipGetLastError());
  double* h = (double*)ctx->hPinned;
  GP_HIP(ctx, hipMemcpyAsync(h, dabs, sizeof(double) * ctx->d, hipMemcpyDeviceToHost, ctx->stream));
  GP_HIP(ctx, hipStreamSynchronize(ctx->stream));
  for (int k = 0; k < ctx->d; ++k) ctx->xabs[k] = h[k];
  return GP_OK;
}

int gp_launch_pack(gp_ctx* ctx) {
  const float gamma = ctx->kernel == GP_SE_ARD ? (float)(-0.5 * 1.4426950408889634) : 3.0f;
  const int blocks = (int)((ctx->n_pad + 255) / 256);
  hipLaunchKernelGGL(pack_kernel, dim3(blocks), dim3(256), 0, ctx->stream, ctx->dX, ctx->n, ctx->n_pad, ctx->d,
                     ctx->KS, (const double*)ctx->dMean, (const double*)ctx->dTheta, gamma, ctx->dXA, ctx->dXB,
                     ctx->dXs, ctx->dNorm, ctx->dMaxNorm);
  GP_HIP(ctx, hipGetLastError());
  const int64_t units = (ctx->n_pad / 32) * ctx->KH * 64;
  hipLaunchKernelGGL(pack_f16_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, ctx->stream,
                     (const float*)ctx->dXs, (const float*)ctx->dNorm, ctx->n, ctx->n_pad, ctx->d, ctx->KH,
                     ctx->kernel == GP_SE_ARD ? 1 : 0, gamma, (u32x4*)ctx->dXAh[0], (u32x4*)ctx->dXAh[1],
                     (u32x4*)ctx->dXAh[2], (u32x4*)ctx->dXBh[0], (u32x4*)ctx->dXBh[1], (u32x4*)ctx->dXBh[2]);
  GP_HIP(ctx, hipGetLastError());
  return GP_OK;
}

namespace {
inline size_t up256(size_t v) { return (v + 255) / 256 * 256; }

struct RowBufs {
  size_t off_xa, off_xb, off_xs, off_norm, off_max, off_a[3], off_b[3], total;
};
RowBufs row_bufs(const gp_ctx* ctx, int64_t m) {
  RowBufs L;
  const int64_t m_pad = (m + GP_ROW_ALIGN - 1) / GP_ROW_ALIGN * GP_ROW_ALIGN;
  const size_t p32 = up256(((size_t)(m_pad / 32) * ctx->KS * 64 + GP_PACK_SLACK) * sizeof(float));
  const size_t p16 = up256((size_t)(m_pad / 32) * ctx->KH * 64 * 16);
  size_t o = 0;
  L.off_xa = o; o += p32;
  L.off_xb = o; o += p32;
  L.off_xs = o; o += up256((size_t)m * ctx->d * sizeof(float));
  L.off_norm = o; o += up256((size_t)m_pad * sizeof(float));
  L.off_max = o; o += 256;
  for (int pc = 0; pc < 3; ++pc) { L.off_a[pc] = o; o += p16; }
  for (int pc = 0; pc < 3; ++pc) { L.off_b[pc] = o; o += p16; }
  L.total = o;
  return L;
}
}  // namespace

size_t gp_pack_rows_bytes(const gp_ctx* ctx, int64_t m) { return row_bufs(ctx, m).total; }

int gp_pack_rows(gp_ctx* ctx, const float* dXstar, int64_t m, void* buf, KmvRows* rows) {
  const RowBufs L = row_bufs(ctx, m);
  char* w = (char*)buf;
  const int64_t m_pad = (m + GP_ROW_ALIGN - 1) / GP_ROW_ALIGN * GP_ROW_ALIGN;
  const float gamma = ctx->kernel == GP_SE_ARD ? (float)(-0.5 * 1.4426950408889634) : 3.0f;
  unsigned* dmax = (unsigned*)(w + L.off_max);
  GP_HIP(ctx, hipMemsetAsync(dmax, 0, sizeof(unsigned), ctx->stream));
  hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((m_pad + 255) / 256)), dim3(256), 0, ctx->stream, dXstar, m, m_pad,
                     ctx->d, ctx->KS, (const double*)ctx->dMean, (const double*)ctx->dTheta, gamma,
                     (float*)(w + L.off_xa), (float*)(w + L.off_xb), (float*)(w + L.off_xs), (float*)(w + L.off_norm), dmax);
  GP_HIP(ctx, hipGetLastError());
  const int64_t units = (m_pad / 32) * ctx->KH * 64;
  hipLaunchKernelGGL(pack_f16_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, ctx->stream,
                     (const float*)(w + L.off_xs), (const float*)(w + L.off_norm), m, m_pad, ctx->d, ctx->KH,
                     ctx->kernel == GP_SE_ARD ? 1 : 0, gamma, (u32x4*)(w + L.off_a[0]), (u32x4*)(w + L.off_a[1]),
                     (u32x4*)(w + L.off_a[2]), (u32x4*)(w + L.off_b[0]), (u32x4*)(w + L.off_b[1]), (u32x4*)(w + L.off_b[2]));
  GP_HIP(ctx, hipGetLastError());
  // the product path must cover the scaled norms of both point sets
  unsigned* hmax = (unsigned*)((char*)ctx->hPinned + GP_PIN_NORM);
  GP_HIP(ctx, hipMemcpyAsync(hmax, dmax, sizeof(unsigned), hipMemcpyDeviceToHost, ctx->stream));
  GP_HIP(ctx, hipStreamSynchronize(ctx->stream));
  float mx;
  memcpy(&mx, hmax, sizeof(float));
  if (ctx->max_norm > mx) mx = ctx->max_norm;
  int path = mx <= GP_NORM_X2_MAX ? GP_PATH_F16X2 : (mx <= GP_NORM_X3_MAX ? GP_PATH_F16X3 : GP_PATH_FP32);
  if (ctx->path_forced >= 0 && !(ctx->path_forced != GP_PATH_FP32 && mx > GP_NORM_X3_MAX)) path = ctx->path_forced;
  if (!ctx->f16_ok) path = GP_PATH_FP32;
  rows->m = m;
  rows->XB = (const float*)(w + L.off_xb);
  for (int pc = 0; pc < 3; ++pc) rows->XBh[pc] = w + L.off_b[pc];
  rows->path = path;
  return GP_OK;
}
