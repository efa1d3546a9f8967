// O(n d) preparation done at gp_create / gp_set_theta: column means of X and
// the packed, pre-scaled operand arrays the tile kernels read (layout in
// gpws_internal.h).  Distances are translation invariant, so centring only
// shrinks |xs|^2 and with it the rounding of the dot-form r^2.
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

// one thread per row: scaled centred row, its squared norm, and both packed operands
__global__ void pack_kernel(const float* __restrict__ X, int64_t n, int64_t n_pad, int d, int KS,
                            const double* __restrict__ mean, const double* __restrict__ theta /* 1/ell (d) */,
                            float gamma, float* __restrict__ XA, float* __restrict__ XB,
                            float* __restrict__ Xs) {
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

}  // namespace

int gp_launch_column_means(gp_ctx* ctx) {
  hipLaunchKernelGGL(column_mean_kernel, dim3(ctx->d), dim3(256), 0, ctx->stream, ctx->dX, ctx->n, ctx->d,
                     ctx->dMean);
  GP_HIP(ctx, hipGetLastError());
  return GP_OK;
}

int gp_launch_pack(gp_ctx* ctx) {
  const float gamma = ctx->kernel == GP_SE_ARD ? (float)(-0.5 * 1.4426950408889634) : 3.0f;
  const int blocks = (int)((ctx->n_pad + 255) / 256);
  hipLaunchKernelGGL(pack_kernel, dim3(blocks), dim3(256), 0, ctx->stream, ctx->dX, ctx->n, ctx->n_pad, ctx->d,
                     ctx->KS, (const double*)ctx->dMean, (const double*)ctx->dTheta, gamma, ctx->dXA, ctx->dXB,
                     ctx->dXs);
  GP_HIP(ctx, hipGetLastError());
  return GP_OK;
}
