// Column-wise streaming over row-major n x t blocks with 256-thread workgroups: shared by the
// alternating-projections and stochastic-gradient solver kernels.
#ifndef GPWS_COL_STREAMS_H
#define GPWS_COL_STREAMS_H

#include <hip/hip_runtime.h>

namespace {

// Column c of thread groups: tw = min(t, 256) columns side by side, 256 / tw rows side by side.
struct ColMap {
  int tw, lanes, cl, rl;
};
__device__ __forceinline__ ColMap col_map(int t) {
  ColMap m;
  m.tw = t < 256 ? t : 256;
  m.lanes = 256 / m.tw;
  m.cl = threadIdx.x % m.tw;
  m.rl = threadIdx.x / m.tw;
  return m;
}

// sum the per-row-lane values of every column in a fixed order and store them as doubles
__device__ __forceinline__ void store_column_sums(const ColMap& m, bool valid, float v, int cg, int t, float* red,
                                                  double* __restrict__ out) {
  if (m.rl < m.lanes) red[m.rl * m.tw + m.cl] = valid ? v : 0.0f;
  __syncthreads();
  if ((int)threadIdx.x < m.tw && cg + (int)threadIdx.x < t) {
    double s = 0.0;
    for (int l = 0; l < m.lanes; ++l) s += (double)red[l * m.tw + threadIdx.x];
    out[cg + threadIdx.x] = s;
  }
  __syncthreads();
}

}  // namespace

#endif
