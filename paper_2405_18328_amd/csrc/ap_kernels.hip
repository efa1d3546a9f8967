// Alternating projections as the linear system solver (Section 2.1 lists it beside conjugate
// gradients, citing Wu et al., 2024; Appendix B fixes the block size 2000 and the stopping rule).
//
// The n indices are cut into consecutive blocks of `block` indices.  One step: pick the block I whose
// residual rows are largest (summed over the columns still being updated), solve H[I,I] d = R[I,:]
// exactly, V[I,:] += d, R -= H[:,I] d.  R stays B - H V throughout.
//
// How the step is laid out for this chip:
//   - set-up (once per solve, i.e. once per theta): every H[I,I] is built, factorised (Cholesky, fp64,
//     64 x 64 tiles, many blocks side by side in one launch), and turned into its explicit inverse
//     (triangular inverse, then L^-T L^-1), stored in fp32.  The block solve of every later step is
//     then one dense product H[I,I]^-1 R[I,:] on the fp32 matrix cores spread over the chip instead of
//     two triangular solves that a few workgroups would have to walk through row tile by row tile;
//   - H[:,I] d is the matrix-free tile pass restricted to the block's columns (KmvWindow);
//   - one streaming kernel applies the update and leaves per-slice squared residual norms, one small
//     kernel turns those into the stopping test and the next block, and posts both to pinned host
//     memory for the host loop (as the CG loop does).
// All floating-point reductions have a fixed order; the atomics are integer maxima (column maxima) and
// one integer ticket counter (which workgroup of the finalise kernel finishes last).
#include <math.h>
#include <stdint.h>

#include "gpws_internal.h"
#include "col_streams.h"

namespace {

constexpr int TS = 64;              // tile edge of the factorisation kernels
constexpr int AP_BATCH = 64;        // blocks factorised side by side (3 x 32 MiB of fp64 scratch each at block 2000)

typedef double fac_t;

struct ApFlags {
  int all_done;
  int breakdown;
  int iters;
  int sel;          // block chosen for the next step
  int seq;          // host mirror only: finalise steps posted so far (written last)
  int pad[3];
};

struct ApDev {
  ApFlags* flags;
  ApFlags* post;    // pinned host memory
  double* bn2;      // [t]
  float* tol;       // [t]
  float* relres;    // [t]
  int* frozen;      // [t]
  int* zero_rhs;    // [t]
  unsigned* colmax; // [t] bit patterns of max |d| per column for the split-fp16 product
  double* norms;    // [nb][S][t] squared residual norms per block slice
  double* normsB;   // [nb][S][t] the same for B (init only)
  double* bnorm;    // [nb][t] squared residual norms per block (finalise kernel's scratch)
  double* bnormB;   // [nb][t] the same for B (init only)
  unsigned* ticket; // workgroups of the finalise kernel that are through with their block sums
};

// ---- 64 x 64 tile products on the fp64 matrix cores ---------------------------------------------
// out[r][c] += sum_m A(r, m) B(m, c) over slabs of KD contraction indices staged in LDS.  A workgroup is
// 4 waves; wave w owns rows 16 w .. 16 w + 15 of the output tile and all 64 columns, as four
// 16 x 16 blocks of v_mfma_f64_16x16x4_f64 (A operand: lane l holds A[l % 16][l / 16]; B operand:
// B[l / 16][l % 16]; result register v of lane l: D[4 v + l / 16][l % 16]).
//
// An operand slab is kept in LDS the way it lies in memory, so that it is fetched with 16-byte loads
// and stored with 16-byte LDS writes, never transposed on the way:
//   - "k-major": memory rows are contraction indices, slab element (m, x) at base[m * ld + x], x = the
//     operand's row (A) or column (B) inside the tile; LDS word m * 64 + (x ^ 16 (m & 1));
//   - "x-major": memory rows are the operand's own rows/columns, element (x, m) at base[x * ld + m];
//     LDS word x * KD + (m ^ 2 (x & 15)).
// The exclusive-ors make the matrix instructions' operand reads (16 values of x for each of 4
// consecutive m per wave) hit every LDS bank once, without padding.
typedef double d4 __attribute__((ext_vector_type(4)));
typedef double d2 __attribute__((ext_vector_type(2)));

constexpr int KD = 32;   // contraction depth held in LDS at a time: two 32 x 64 operand slabs = 32 KB per
                         // workgroup, so that four workgroups share a compute unit and their loads, LDS
                         // traffic and matrix-core work overlap

struct alignas(16) Tile {
  fac_t v[KD * TS];
};

struct Acc {
  d4 b[4];   // column block cb: rows 16 w + 4 v + l / 16, column 16 cb + l % 16
};

// One 64 x 64 operand tile in memory (see above); `xmajor` is fixed per call site (template argument
// of tile_chain), `base` and `ld` are not.  Slab h of a tile = contraction indices 32 h .. 32 h + 31.
struct Operand {
  const fac_t* base;
  int64_t ld;
};

struct SlabRegs {
  d2 v[4];
};
// all 4 loads of a thread are issued before anything waits on them
template <bool XMAJOR>
__device__ __forceinline__ void fetch_slab(SlabRegs& g, const Operand& o, int h) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int e = threadIdx.x + 256 * q;            // pair of doubles e of the slab
    const fac_t* src = XMAJOR ? o.base + (int64_t)(e / (KD / 2)) * o.ld + KD * h + 2 * (e % (KD / 2))
                              : o.base + (int64_t)(KD * h + e / (TS / 2)) * o.ld + 2 * (e % (TS / 2));
    g.v[q] = *reinterpret_cast<const d2*>(src);
  }
}
template <bool XMAJOR>
__device__ __forceinline__ void stash_slab(Tile& T, const SlabRegs& g) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int e = threadIdx.x + 256 * q;
    int word;
    if (XMAJOR) {
      const int x = e / (KD / 2), m = 2 * (e % (KD / 2));
      word = x * KD + (m ^ (2 * (x & 15)));
    } else {
      const int m = e / (TS / 2), x = 2 * (e % (TS / 2));
      word = m * TS + (x ^ (16 * (m & 1)));
    }
    *reinterpret_cast<d2*>(&T.v[word]) = g.v[q];     // the exclusive-ors are even: a pair stays a pair
  }
}
// operand value (x, m) of a staged slab
template <bool XMAJOR>
__device__ __forceinline__ fac_t slab_at(const Tile& T, int x, int m) {
  return XMAJOR ? T.v[x * KD + (m ^ (2 * (x & 15)))] : T.v[m * TS + (x ^ (16 * (m & 1)))];
}

__device__ __forceinline__ void clear_acc(Acc& acc) {
#pragma unroll
  for (int cb = 0; cb < 4; ++cb) acc.b[cb] = d4{0.0, 0.0, 0.0, 0.0};
}

template <bool AX, bool BX>
__device__ __forceinline__ void mac_slab(const Tile& TA, const Tile& TB, Acc& acc) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int lo = lane & 15, hi = lane >> 4;
#pragma unroll 4
  for (int m0 = 0; m0 < KD; m0 += 4) {
    const fac_t a = slab_at<AX>(TA, 16 * w + lo, m0 + hi);
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
      acc.b[cb] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, slab_at<BX>(TB, 16 * cb + lo, m0 + hi), acc.b[cb], 0, 0, 0);
  }
}

// acc += sum over the tiles m = m_lo .. m_hi of A_m B_m, where opA(m) / opB(m) name the two 64 x 64
// operand tiles of step m (AX / BX: x-major in memory).  The next slab's loads are in flight while the
// matrix cores work on the current one.
template <bool AX, bool BX, typename FA, typename FB>
__device__ __forceinline__ void tile_chain(Tile& TA, Tile& TB, Acc& acc, int m_lo, int m_hi, FA opA, FB opB) {
  if (m_lo > m_hi) return;
  const int steps = 2 * (m_hi - m_lo + 1);
  SlabRegs ga, gb;
  Operand oa = opA(m_lo), ob = opB(m_lo);
  fetch_slab<AX>(ga, oa, 0);
  fetch_slab<BX>(gb, ob, 0);
  for (int q = 0; q < steps; ++q) {
    stash_slab<AX>(TA, ga);
    stash_slab<BX>(TB, gb);
    __syncthreads();
    if (q + 1 < steps) {
      const int m = m_lo + (q + 1) / 2;
      oa = opA(m);
      ob = opB(m);
      fetch_slab<AX>(ga, oa, (q + 1) & 1);
      fetch_slab<BX>(gb, ob, (q + 1) & 1);
    }
    mac_slab<AX, BX>(TA, TB, acc);
    __syncthreads();
  }
}

// row and column (inside the 64 x 64 tile) of element v of column block cb held by this thread
__device__ __forceinline__ int acc_row(int v) { return 16 * (threadIdx.x >> 6) + 4 * v + ((threadIdx.x & 63) >> 4); }
__device__ __forceinline__ int acc_col(int cb) { return 16 * cb + (threadIdx.x & 15); }

// ---- set-up: H[I,I], Cholesky, inverse ------------------------------------------------------------
// A[z] (BP x BP, row-major, fp64) = H[I,I] for block blk0 + z, identity on the padding rows/columns.
// One workgroup per 64 x 64 tile on or below the diagonal (the mirror image is written too); the 2 x 64
// input rows are staged in LDS, differences (exact), scaling and the kernel function in fp64.
__global__ __launch_bounds__(256) void ap_build_kernel(const float* __restrict__ X, int d, int64_t n,
                                                       const double* __restrict__ theta, int kind, int block, int BP,
                                                       int blk0, fac_t* __restrict__ A) {
  extern __shared__ float xs[];            // [2][64][d + 1] input rows of the tile's row and column ranges
  if (blockIdx.x > blockIdx.y) return;
  const int ti = blockIdx.y, tj = blockIdx.x;
  const int64_t j0 = (int64_t)(blk0 + blockIdx.z) * block;
  const int64_t left = n - j0;
  const int bs = (int)(left < block ? left : block);
  const int ldx = d + 1;
  for (int e = threadIdx.x; e < 2 * TS * d; e += 256) {
    const int side = e / (TS * d), q = e % (TS * d);
    const int r = q / d, kk = q % d;
    const int row = (side == 0 ? ti : tj) * TS + r;
    xs[(side * TS + r) * ldx + kk] = row < bs ? X[(j0 + row) * d + kk] : 0.0f;
  }
  __syncthreads();
  const double a = theta[d], sg = theta[d + 1];
  fac_t* Ab = A + (int64_t)blockIdx.z * BP * BP;
  for (int e = threadIdx.x; e < TS * TS; e += 256) {
    const int r = e / TS, c = e % TS;
    const int i = ti * TS + r, j = tj * TS + c;
    fac_t v;
    if (i < bs && j < bs) {
      const float* xi = xs + r * ldx;
      const float* xj = xs + (TS + c) * ldx;
      double r2 = 0.0;
      for (int kk = 0; kk < d; ++kk) {
        const double df = ((double)xi[kk] - (double)xj[kk]) * theta[kk];   // exact difference; theta[kk] = 1 / ell_kk
        r2 = fma(df, df, r2);
      }
      if (kind == GP_SE_ARD) {
        v = a * a * exp(-0.5 * r2);
      } else {
        const double u = sqrt(3.0 * r2);
        v = a * a * (1.0 + u) * exp(-u);
      }
      if (i == j) v += sg * sg;
    } else {
      v = (i == j) ? 1.0 : 0.0;
    }
    Ab[(int64_t)i * BP + j] = v;
    Ab[(int64_t)j * BP + i] = v;
  }
}

// value of v in lane `src` (wave-uniform), for a double
__device__ __forceinline__ double lane_bcast(double v, int src) {
  const unsigned long long u = __builtin_bit_cast(unsigned long long, v);
  const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)u, src);
  const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(u >> 32), src);
  return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}

// 16 x 16 block product on the matrix cores with both operands row-major in LDS (row stride TS + 1):
// acc += P[0..15][0..15] Q[0..15][0..15], P and Q pointing at the blocks' first elements.
__device__ __forceinline__ d4 block16_mac(const fac_t* P, const fac_t* Q, d4 acc) {
  const int lane = threadIdx.x & 63, lo = lane & 15, hi = lane >> 4;
#pragma unroll
  for (int s4 = 0; s4 < 16; s4 += 4)
    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(P[lo * (TS + 1) + s4 + hi], Q[(s4 + hi) * (TS + 1) + lo], acc, 0, 0, 0);
  return acc;
}
// the same with the second operand transposed: acc += P Q^T
__device__ __forceinline__ d4 block16_mac_nt(const fac_t* P, const fac_t* Q, d4 acc) {
  const int lane = threadIdx.x & 63, lo = lane & 15, hi = lane >> 4;
#pragma unroll
  for (int s4 = 0; s4 < 16; s4 += 4)
    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(P[lo * (TS + 1) + s4 + hi], Q[lo * (TS + 1) + s4 + hi], acc, 0, 0, 0);
  return acc;
}

// diagonal tile k of every block in the batch: L_kk in place (upper part zeroed); its inverse goes to
// DI and to the diagonal tile of X (the matrix that becomes L^-1).  One workgroup of four waves per
// tile, the tile in LDS, worked in panels of 16 columns:
//   - a panel is factorised by wave 0 with lane = row and the row's 16 panel entries in registers: the
//     64 dependent column steps of the tile (pivot, reciprocal square root, scale, rank-1 update of the
//     panel's remaining columns) touch no memory, the other rows' entries come by lane broadcast;
//   - the rest of the tile is then updated with the panel (rank 16) on the matrix cores by all waves.
// The inverse is built the same way: the four 16 x 16 diagonal blocks by forward substitution in
// registers (lane = column, one block per wave), the blocks below them by merging pairs,
// X21 = -X22 (L21 X11), on the matrix cores.
__global__ __launch_bounds__(256) void ap_chol_diag_kernel(fac_t* __restrict__ A, int BP, int k,
                                                           fac_t* __restrict__ DI, fac_t* __restrict__ X,
                                                           int* __restrict__ breakdown) {
  constexpr int LD = TS + 1;
  constexpr int PW = 16;                 // panel width
  __shared__ fac_t T[TS * LD];           // the tile, then L (lower part)
  __shared__ fac_t Xi[TS * LD];          // L^-1
  __shared__ fac_t Tm[32 * LD];          // L21 X11 of the pair being merged
  __shared__ fac_t rdiag[TS];            // 1 / L[c][c]
  const int64_t tile_off = (int64_t)blockIdx.x * BP * BP + (int64_t)k * TS * BP + k * TS;
  fac_t* Ab = A + tile_off;
  fac_t* Xb = X + tile_off;
  fac_t* DIb = DI + (int64_t)blockIdx.x * BP * TS + (int64_t)k * TS * TS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = lane & 15, hi = lane >> 4;
  {
    fac_t g[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int e = tid + 256 * q;
      g[q] = Ab[(int64_t)(e / TS) * BP + (e % TS)];
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int e = tid + 256 * q;
      T[(e / TS) * LD + (e % TS)] = g[q];
      Xi[(e / TS) * LD + (e % TS)] = 0.0;
    }
  }
  __syncthreads();
  bool any_bad = false;
  for (int p0 = 0; p0 < TS; p0 += PW) {
    if (wave == 0) {
      fac_t x[PW];
#pragma unroll
      for (int q = 0; q < PW; ++q) x[q] = T[lane * LD + p0 + q];
#pragma unroll
      for (int c = 0; c < PW; ++c) {
        const fac_t piv0 = lane_bcast(x[c], p0 + c);
        const bool bad = !(piv0 > 0.0) || !(piv0 < 1.0e300);   // also catches NaN
        any_bad = any_bad || bad;
        const fac_t piv = bad ? 1.0 : piv0;
        // 1 / sqrt(piv) from the single-precision estimate and three Newton steps (each squares the
        // relative error: 2^-22, 2^-43, below 2^-53); this chain is the critical path of a column step
        fac_t rinv = (fac_t)__builtin_amdgcn_rsqf((float)piv);
#pragma unroll
        for (int it = 0; it < 3; ++it) rinv = rinv * fma(-0.5 * piv, rinv * rinv, 1.5);
        const fac_t lc = lane > p0 + c ? x[c] * rinv : (lane == p0 + c ? piv * rinv : 0.0);   // column p0 + c of L
        x[c] = lc;
        if (lane == p0 + c) rdiag[p0 + c] = rinv;
#pragma unroll
        for (int j = c + 1; j < PW; ++j) x[j] = fma(-lc, lane_bcast(lc, p0 + j), x[j]);   // meaningful for rows >= p0 + j
      }
      if (lane >= p0) {
#pragma unroll
        for (int q = 0; q < PW; ++q) T[lane * LD + p0 + q] = x[q];
      }
    }
    __syncthreads();
    // trailing blocks (bi >= bj > panel): T_bi,bj -= L_bi,p L_bj,p^T
    const int pb = p0 / PW, nbk = TS / PW;
    int idx = 0;
    for (int bi = pb + 1; bi < nbk; ++bi)
      for (int bj = pb + 1; bj <= bi; ++bj, ++idx) {
        if ((idx & 3) != wave) continue;
        d4 acc = block16_mac_nt(&T[(PW * bi) * LD + p0], &T[(PW * bj) * LD + p0], d4{0.0, 0.0, 0.0, 0.0});
#pragma unroll
        for (int v = 0; v < 4; ++v) T[(PW * bi + 4 * v + hi) * LD + PW * bj + lo] -= acc[v];
      }
    __syncthreads();
  }
  if (any_bad && tid == 0) *breakdown = 1;
  // inverse of the four diagonal 16 x 16 blocks: wave w takes block w, lane j < 16 its column j,
  // x_i = (delta_ij - sum_{m < i} L[i][m] x_m) / L[i][i]
  if (lo == lane) {   // lanes 0..15
    const int o = PW * wave;
    fac_t x[PW];
#pragma unroll
    for (int i = 0; i < PW; ++i) {
      fac_t s0 = lane == i ? 1.0 : 0.0;
#pragma unroll
      for (int m = 0; m < i; ++m) s0 = fma(-T[(o + i) * LD + o + m], x[m], s0);
      x[i] = s0 * rdiag[o + i];
    }
#pragma unroll
    for (int i = 0; i < PW; ++i) Xi[(o + i) * LD + o + lane] = x[i];
  }
  __syncthreads();
  // merge pairs of blocks: level 1 = (0,1) and (2,3), 16 x 16 each; level 2 = the 32 x 32 block below
  // the first two block columns.  Tm = L21 X11, then X21 = -X22 Tm.
  {
    // level 1: waves 0 and 1 take one pair each
    if (wave < 2) {
      const int o1 = 2 * PW * wave, o2 = o1 + PW;
      const d4 t = block16_mac(&T[o2 * LD + o1], &Xi[o1 * LD + o1], d4{0.0, 0.0, 0.0, 0.0});
#pragma unroll
      for (int v = 0; v < 4; ++v) Tm[(PW * wave + 4 * v + hi) * LD + lo] = t[v];
    }
    __syncthreads();
    if (wave < 2) {
      const int o1 = 2 * PW * wave, o2 = o1 + PW;
      const d4 r = block16_mac(&Xi[o2 * LD + o2], &Tm[(PW * wave) * LD], d4{0.0, 0.0, 0.0, 0.0});
#pragma unroll
      for (int v = 0; v < 4; ++v) Xi[(o2 + 4 * v + hi) * LD + o1 + lo] = -r[v];
    }
    __syncthreads();
    // level 2: four 16 x 16 output blocks (bi, bj), one per wave; halves are 2 blocks wide
    const int bi = wave >> 1, bj = wave & 1;
    {
      d4 t = d4{0.0, 0.0, 0.0, 0.0};
      for (int m = bj; m < 2; ++m)     // X11 is lower triangular: block (m, bj) is zero for m < bj
        t = block16_mac(&T[(32 + PW * bi) * LD + PW * m], &Xi[(PW * m) * LD + PW * bj], t);
#pragma unroll
      for (int v = 0; v < 4; ++v) Tm[(PW * bi + 4 * v + hi) * LD + PW * bj + lo] = t[v];
    }
    __syncthreads();
    {
      d4 r = d4{0.0, 0.0, 0.0, 0.0};
      for (int m = 0; m <= bi; ++m)    // X22 is lower triangular
        r = block16_mac(&Xi[(32 + PW * bi) * LD + 32 + PW * m], &Tm[(PW * m) * LD + PW * bj], r);
#pragma unroll
      for (int v = 0; v < 4; ++v) Xi[(32 + PW * bi + 4 * v + hi) * LD + PW * bj + lo] = -r[v];
    }
    __syncthreads();
  }
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int e = tid + 256 * q;
    const int i = e / TS, j = e % TS;
    Ab[(int64_t)i * BP + j] = j <= i ? T[i * LD + j] : 0.0;
    const fac_t v = Xi[i * LD + j];
    DIb[i * TS + j] = v;
    Xb[(int64_t)i * BP + j] = v;
  }
}

// panel below the diagonal tile: L_ik = A_ik L_kk^-T, row tile i = k + 1 + blockIdx.x
__global__ __launch_bounds__(256) void ap_chol_panel_kernel(fac_t* __restrict__ A, int BP, int k,
                                                            const fac_t* __restrict__ DI) {
  __shared__ Tile TA, TB;
  const int it = k + 1 + blockIdx.x;
  fac_t* Aik = A + (int64_t)blockIdx.y * BP * BP + (int64_t)it * TS * BP + k * TS;
  const fac_t* DIb = DI + (int64_t)blockIdx.y * BP * TS + (int64_t)k * TS * TS;
  Acc acc;
  clear_acc(acc);
  const int64_t ldA = BP;
  tile_chain<true, true>(TA, TB, acc, 0, 0,
                         [=](int) { return Operand{Aik, ldA}; },      // A_ik(r, m)
                         [=](int) { return Operand{DIb, TS}; });      // L_kk^-1(c, m)
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int v = 0; v < 4; ++v) Aik[(int64_t)acc_row(v) * BP + acc_col(cb)] = acc.b[cb][v];
}

// trailing update A_IJ -= sum_{m = k0}^{k0 + klen - 1} L_Im L_Jm^T for the tiles I >= J, J = j0 + blockIdx.x
// (blockIdx.x < gridDim.x), I = j0 + blockIdx.y.  The factorisation works in rounds of CHOL_ROUND tile
// columns: inside a round the earlier columns are applied to the next column alone (one tile column),
// and once the round is factorised all its columns are applied to the rest of the matrix together,
// which reads and writes the trailing matrix once per round instead of once per column -- that traffic,
// not the arithmetic, is what bounds the update.
constexpr int CHOL_ROUND = 2;   // 4 measured no better: the one-column updates inside a round are few workgroups with longer chains
__global__ __launch_bounds__(256) void ap_chol_update_kernel(fac_t* __restrict__ A, int BP, int k0, int klen, int j0) {
  __shared__ Tile TA, TB;
  if (blockIdx.x > blockIdx.y) return;
  const int I = j0 + blockIdx.y, J = j0 + blockIdx.x;
  fac_t* Ab = A + (int64_t)blockIdx.z * BP * BP;
  Acc acc;
  clear_acc(acc);
  const fac_t* LI = Ab + (int64_t)I * TS * BP;
  const fac_t* LJ = Ab + (int64_t)J * TS * BP;
  const int64_t ldA = BP;
  tile_chain<true, true>(TA, TB, acc, k0, k0 + klen - 1,
                         [=](int m) { return Operand{LI + m * TS, ldA}; },       // L_Im(r, q)
                         [=](int m) { return Operand{LJ + m * TS, ldA}; });      // L_Jm(c, q)
  fac_t* Aij = Ab + (int64_t)I * TS * BP + J * TS;
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int v = 0; v < 4; ++v) Aij[(int64_t)acc_row(v) * BP + acc_col(cb)] -= acc.b[cb][v];
}

// Workgroup numbering of X^T X, the kernel with the longest tile-product chains: the output tiles are
// grouped into super-blocks of SB x SB tiles, and the workgroups of a super-block follow each other on
// one XCD (workgroup w of a launch runs on XCD w % XCDS), so that the operand tiles they share are
// fetched into that XCD's L2 once.  Numbered row by row over the whole grid, every XCD pulled all of X
// through its own L2 several times, and the kernel waited for memory 70 % of the time (1.25 ms against
// 0.62 ms for nine blocks of 2048).  The triangular inverse's merges gained nothing from the same
// numbering (fewer, shorter chains per launch) and keep the plain grid.
constexpr int XCDS = 8;
constexpr int SB = 8;         // super-block edge of X^T X (90 super-blocks for nine blocks of 2048: 11 or 12 per XCD)
struct SbIndex {
  int sb;        // super-block
  int di, dj;    // tile inside it
};
__device__ __forceinline__ SbIndex sb_decode(int edge) {      // edge = tiles per super-block edge
  const int per = edge * edge;
  const int slot = blockIdx.x / XCDS;
  const int within = slot % per;
  return SbIndex{(slot / per) * XCDS + (int)(blockIdx.x % XCDS), within / edge, within % edge};
}
inline int sb_grid(int superblocks, int edge) { return XCDS * ((superblocks + XCDS - 1) / XCDS) * edge * edge; }

// X = L^-1 by merging diagonal blocks pairwise, level by level (s = 1, 2, 4, .. tiles): for the pair
// [[L11, 0], [L21, L22]] whose halves X11 = L11^-1 and X22 = L22^-1 are complete,
//   X21 = -X22 (L21 X11).
// Every level is two launches, each a set of independent tile products whose chains are at most s
// tiles long.  Pair p of a level covers tiles [2 s p, 2 s p + s) and [2 s p + s, min(2 s p + 2 s, nt)).
// step 0: T = L21 X11, tile (ti, tj) = sum_{m = tj}^{s - 1} L21(ti, m) X11(m, tj)   (X11 is lower triangular)
// step 1: X21 = -X22 T, tile (ti, tj) = -sum_{m = 0}^{ti} X22(ti, m) T(m, tj)       (X22 is lower triangular)
// Grid (s, s, pairs * batch).
__global__ __launch_bounds__(256) void ap_trinv_merge_kernel(const fac_t* __restrict__ A, fac_t* X, fac_t* T, int BP,
                                                             int s, int pairs, int step) {
  __shared__ Tile TA, TB;
  const int nt = BP / TS;
  const int pr = blockIdx.z % pairs, z = blockIdx.z / pairs;
  const int o1 = 2 * s * pr, o2 = o1 + s;
  const int s2 = nt - o2 < s ? nt - o2 : s;         // tiles in the second half (may be short or empty)
  // workgroups are dispatched x first, then y: the slow index is the one the chain length depends on,
  // longest chains first (step 0: s - tj products, step 1: ti + 1), so that the launch does not end
  // on a few long chains that started last
  const int ti = step == 0 ? blockIdx.x : s - 1 - (int)blockIdx.y;
  const int tj = step == 0 ? blockIdx.y : blockIdx.x;
  if (ti >= s2) return;
  const int64_t zo = (int64_t)z * BP * BP;
  const fac_t* P;      // left factor, tile (ti, m) at P + (ti * TS * BP + m * TS)
  const fac_t* Q;      // right factor, tile (m, tj)
  int mlo, mhi;
  if (step == 0) {
    P = A + zo + (int64_t)o2 * TS * BP + o1 * TS;
    Q = X + zo + (int64_t)o1 * TS * BP + o1 * TS;
    mlo = tj;
    mhi = s - 1;
  } else {
    P = X + zo + (int64_t)o2 * TS * BP + o2 * TS;
    Q = T + zo + (int64_t)o2 * TS * BP + o1 * TS;
    mlo = 0;
    mhi = ti;
  }
  Acc acc;
  clear_acc(acc);
  {
    const fac_t* Pt = P + (int64_t)ti * TS * BP;
    const fac_t* Qt = Q + (int64_t)tj * TS;
    const int64_t ld = BP;
    tile_chain<true, false>(TA, TB, acc, mlo, mhi,
                            [=](int m) { return Operand{Pt + (int64_t)m * TS, ld}; },          // P(r, q): the source column is the contraction index
                            [=](int m) { return Operand{Qt + (int64_t)m * TS * ld, ld}; });    // Q(q, c)
  }
  fac_t* out = (step == 0 ? T : X) + zo + (int64_t)(o2 + ti) * TS * BP + (o1 + tj) * TS;
  const fac_t sign = step == 0 ? 1.0 : -1.0;
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int v = 0; v < 4; ++v) out[(int64_t)acc_row(v) * BP + acc_col(cb)] = sign * acc.b[cb][v];
}

// H[I,I]^-1 = X^T X, tiles (ti >= tj) and their mirror images, rounded to fp32.  The inverse is stored in
// panels of 16 rows and, inside a panel, in groups of 4 contraction indices: element (r, c) at
// ((r / 16) (BP / 4) + c / 4) 64 + (r % 16) 4 + c % 4.  What one wave of the block solve reads for its
// row tile and 16 consecutive contraction indices (lane = (row, 4 of them), 16 bytes each) is then one
// contiguous kilobyte, and the next 16 indices are the next kilobyte.
__device__ __forceinline__ int64_t hinv_at(int r, int c, int BP) {
  return ((int64_t)(r >> 4) * (BP >> 2) + (c >> 2)) * 64 + (r & 15) * 4 + (c & 3);
}
__device__ __forceinline__ constexpr int hinv_step() { return 64; }   // floats between c and c + 4 at fixed r
// Workgroups are numbered by super-block (see sb_decode) and walk the contraction index downwards from
// the same starting tile row, so that the 2 SB tile columns of X a super-block shares stay in its
// XCD's L2 while they are in use.
__host__ __device__ inline int lauum_superblocks(int nt) {
  const int ns = (nt + SB - 1) / SB;
  return ns * (ns + 1) / 2;
}
__global__ __launch_bounds__(256) void ap_lauum_kernel(const fac_t* __restrict__ W, int BP, int cnt,
                                                       float* __restrict__ Hinv) {
  __shared__ Tile TA, TB;
  const int nt = BP / TS;
  const int nsb = lauum_superblocks(nt);
  const SbIndex w = sb_decode(SB);
  if (w.sb >= cnt * nsb) return;
  const int z = w.sb / nsb, p = w.sb % nsb;
  int I = 0;
  while ((I + 1) * (I + 2) / 2 <= p) ++I;                             // p = I (I + 1) / 2 + J, J <= I
  const int J = p - I * (I + 1) / 2;
  const int ti = SB * I + w.di, tj = SB * J + w.dj;
  if (ti >= nt || tj > ti) return;
  const fac_t* Wb = W + (int64_t)z * BP * BP;
  Acc acc;
  clear_acc(acc);
  {
    const fac_t* Wi = Wb + (int64_t)ti * TS;
    const fac_t* Wj = Wb + (int64_t)tj * TS;
    const int64_t ld = BP;
    const int top = nt - 1 + ti;                                      // step m of the chain reads tile row top - m
    tile_chain<false, false>(TA, TB, acc, ti, nt - 1,
                             [=](int m) { return Operand{Wi + (int64_t)(top - m) * TS * ld, ld}; },    // X_m,ti(q, r)
                             [=](int m) { return Operand{Wj + (int64_t)(top - m) * TS * ld, ld}; });   // X_m,tj(q, c)
  }
  float* Hb = Hinv + (int64_t)z * BP * BP;
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int r = ti * TS + acc_row(v), c = tj * TS + acc_col(cb);
      const float val = (float)acc.b[cb][v];
      Hb[hinv_at(r, c, BP)] = val;
      Hb[hinv_at(c, r, BP)] = val;
    }
}

// ---- the iteration -------------------------------------------------------------------------------
// workgroup blockIdx.x = k S + s owns slice s (of S) of block k
__device__ __forceinline__ void slice_rows(int64_t n, int block, int S, int64_t* r0, int64_t* r1) {
  const int64_t k = blockIdx.x / S;
  const int s = blockIdx.x % S;
  const int64_t b0 = k * block;
  const int64_t b1 = b0 + block < n ? b0 + block : n;
  const int64_t per = (b1 - b0 + S - 1) / S;
  *r0 = b0 + s * per;
  const int64_t e = *r0 + per;
  *r1 = e < b1 ? e : b1;
}

// V <- X0 (or 0), R <- B - HX0 (HX0 given when X0 is), D <- 0, squared norms of B and R per block slice.
// Grid: nb * S workgroups, workgroup (k, s) owns slice s of block k.
__global__ __launch_bounds__(256) void ap_init_kernel(const float* __restrict__ B, int64_t ldb,
                                                      const float* __restrict__ X0, int64_t ldx,
                                                      const float* __restrict__ HX0, int64_t n, int t, int block, int S,
                                                      float* __restrict__ V, float* __restrict__ R,
                                                      float* __restrict__ D, double* __restrict__ norms,
                                                      double* __restrict__ normsB) {
  __shared__ float red[256];
  int64_t r0, r1;
  slice_rows(n, block, S, &r0, &r1);
  const ColMap m = col_map(t);
  for (int cg = 0; cg < t; cg += m.tw) {
    const int c = cg + m.cl;
    const bool valid = c < t && m.rl < m.lanes;
    float accb = 0.0f, accr = 0.0f;
    if (valid) {
      for (int64_t i = r0 + m.rl; i < r1; i += m.lanes) {
        const int64_t e = i * t + c;
        const float b = B[i * ldb + c];
        const float x = X0 ? X0[i * ldx + c] : 0.0f;
        const float r = X0 ? b - HX0[e] : b;
        V[e] = x;
        R[e] = r;
        D[e] = 0.0f;
        accb = fmaf(b, b, accb);
        accr = fmaf(r, r, accr);
      }
    }
    store_column_sums(m, valid, accb, cg, t, red, normsB + (int64_t)blockIdx.x * t);
    store_column_sums(m, valid, accr, cg, t, red, norms + (int64_t)blockIdx.x * t);
  }
}

// d = H[I,I]^-1 R[I,:], columns no longer updated set to 0, written to rows j0 .. j0 + bs - 1 of D, and
// the columns' largest |d| to colmax (zero on entry).  One workgroup per 16 rows and 64 columns of d, on
// the fp32 matrix cores (v_mfma_f32_16x16x4_f32: A operand lane l holds A[l % 16][l / 16], B operand
// B[l / 16][l % 16], result register v of lane l is D[4 (l / 16) + v][l % 16]).
//   - Every operand load is 16 bytes per lane (the memory pipeline of a compute unit spends the same
//     time on a 4-byte-per-lane load).  A: the inverse is symmetric and stored so that lane l's four
//     floats are Hinv[row0 + l % 16][m0 + 4 (l / 16) + j], j = 0..3 (see hinv_at).  B: lane l loads
//     R[m][4 (l % 16) .. + 3] for the four m = m0 + 4 (l / 16) + j.  Matrix instruction (j, i) then
//     contracts over the indices {m0 + 4 h + j} and produces the 16 columns {4 c + i}: the 64 columns
//     of the workgroup are four interleaved tiles.  One A load and four B loads feed 16 instructions.
//   - The contraction index is cut into SOLVE_WAVES ranges, one per wave, whose partial tiles are
//     added in a fixed order through LDS; nothing is exchanged between workgroups.
//   - Loads are unconditional (indices clamped, values replaced by zero when used), so a wave keeps
//     two batches in flight and waits only for the older one.  Reading four floats at the end of a
//     row of R runs into the next row (never past the array D that follows R in the workspace).
typedef float f4 __attribute__((ext_vector_type(4)));
constexpr int SOLVE_WAVES = 8;

// NTL consecutive floats at a 4-byte-aligned address
template <int NTL> struct RowVec;
template <> struct RowVec<4> { typedef float type __attribute__((ext_vector_type(4), aligned(4))); };
template <> struct RowVec<2> { typedef float type __attribute__((ext_vector_type(2), aligned(4))); };

// NTL = interleaved column tiles per workgroup: 4 (64 columns, 16-byte loads of R) or 2 (32 columns,
// 8-byte loads; twice as many workgroups, for products whose 16-row tiles alone do not fill the chip)
// The block is the one the last finalise step chose (flags->sel, read here on the device), so the host
// can queue this kernel right behind that step without waiting to learn the choice; it does nothing once
// the solve is over.  The grid covers a full block; workgroups past a short last block leave at once.
template <int NTL>
__global__ __launch_bounds__(64 * SOLVE_WAVES) void ap_block_solve_kernel(const float* __restrict__ Hinv_all, int BP,
                                                                         int block, int64_t n,
                                                                         const float* __restrict__ R, int t,
                                                                         const ApFlags* __restrict__ flags,
                                                                         const int* __restrict__ frozen,
                                                                         float* __restrict__ D,
                                                                         unsigned* __restrict__ colmax) {
  typedef typename RowVec<NTL>::type rowvec;
  constexpr int CW = 16 * NTL;                         // columns of a workgroup
  constexpr int SOLVE_G = 2;                           // groups of 16 contraction indices per batch of loads
  __shared__ f4 red[SOLVE_WAVES][NTL][64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lo = lane & 15, hi = lane >> 4;
  const int row0 = 16 * blockIdx.x;
  const int done = flags->all_done, k = flags->sel;
  if (done) return;
  const int64_t j0 = (int64_t)k * block;
  const int bs = (int)(n - j0 < block ? n - j0 : block);
  if (row0 >= bs) return;
  const float* Hinv = Hinv_all + (int64_t)k * BP * BP;
  const int cbase = CW * blockIdx.y + NTL * lo;        // this lane's B columns: cbase + i
  bool cok[NTL], live[NTL];
  bool any_live = false;
#pragma unroll
  for (int i = 0; i < NTL; ++i) {
    cok[i] = cbase + i < t;
    live[i] = frozen[cok[i] ? cbase + i : 0] == 0;     // unconditional loads, all in flight together
  }
#pragma unroll
  for (int i = 0; i < NTL; ++i) {
    live[i] = live[i] && cok[i];
    any_live = any_live || live[i];
  }
  if (!__any(any_live)) {                              // every column of the workgroup has converged
    if (wave == 0) {
#pragma unroll
      for (int i = 0; i < NTL; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int c = cbase + i;                     // tile i, lane column lo
          if (c < t && row0 + 4 * hi + v < bs) D[(j0 + row0 + 4 * hi + v) * t + c] = 0.0f;
        }
    }
    return;
  }
  // tiles whose columns all lie past t are skipped (wave-uniform): tile i holds the columns
  // CW cg + NTL c + i, present iff i < t - CW cg
  int ntile = t - CW * (int)blockIdx.y;
  ntile = ntile >= NTL ? NTL : ntile;
  const int kw = ((bs + SOLVE_WAVES - 1) / SOLVE_WAVES + 15) & ~15;   // contraction indices per wave, a multiple of 16
  const int mb = wave * kw;
  const int me = mb + kw < bs ? mb + kw : bs;
  const float* ap = Hinv + hinv_at(row0 + lo, 4 * hi, BP);            // + hinv_step() floats per 4 contraction indices
  const int bcol = cok[0] ? cbase : 0;
  const float* bp = R + j0 * t + bcol;
  f4 acc[NTL];
#pragma unroll
  for (int i = 0; i < NTL; ++i) acc[i] = f4{0.0f, 0.0f, 0.0f, 0.0f};
  if (mb < me) {
    struct Batch {
      f4 a[SOLVE_G];
      rowvec b[SOLVE_G][4];
    };
    Batch b0, b1;
    const int mlast = me - 1;
    auto fetch = [&](Batch& q, int ms) {
#pragma unroll
      for (int g = 0; g < SOLVE_G; ++g) {
        const int m0 = ms + 16 * g;                    // group of 16 contraction indices
        const int mq = m0 < me ? m0 : (mlast & ~15);   // a group that starts inside the range (its tail is masked)
        q.a[g] = *reinterpret_cast<const f4*>(ap + hinv_step() * (mq >> 2));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int m = mq + 4 * hi + j;
          const int mc = m < me ? m : mlast;
          q.b[g][j] = *reinterpret_cast<const rowvec*>(bp + (int64_t)mc * t);
        }
      }
    };
    auto mac = [&](const Batch& q, int ms) {
#pragma unroll
      for (int g = 0; g < SOLVE_G; ++g) {
        const int m0 = ms + 16 * g;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool ok = m0 + 4 * hi + j < me;
          const float av = ok ? q.a[g][j] : 0.0f;
#pragma unroll
          for (int i = 0; i < NTL; ++i) {
            if (i < ntile)
              acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, (ok && cok[i]) ? q.b[g][j][i] : 0.0f, acc[i], 0, 0, 0);
          }
        }
      }
    };
    fetch(b0, mb);
    for (int ms = mb; ms < me; ms += 32 * SOLVE_G) {
      fetch(b1, ms + 16 * SOLVE_G);
      mac(b0, ms);
      fetch(b0, ms + 32 * SOLVE_G);
      mac(b1, ms + 16 * SOLVE_G);
    }
  }
#pragma unroll
  for (int i = 0; i < NTL; ++i) red[wave][i][lane] = acc[i];
  __syncthreads();
  if (wave >= NTL || wave >= ntile) return;
  // wave i finishes tile i: columns CW cg + NTL c + i for lane column c = lo
  const int i = wave;
  f4 sum = red[0][i][lane];
#pragma unroll
  for (int w = 1; w < SOLVE_WAVES; ++w) sum += red[w][i][lane];
  const int c = CW * blockIdx.y + NTL * lo + i;
  const bool c_ok = c < t;
  const bool c_live = c_ok && !frozen[c_ok ? c : 0];
  float big = 0.0f;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const float val = c_live ? sum[v] : 0.0f;
    if (c_ok && row0 + 4 * hi + v < bs) {
      D[(j0 + row0 + 4 * hi + v) * t + c] = val;
      big = fmaxf(big, fabsf(val));
    }
  }
  big = fmaxf(big, __shfl_xor(big, 16, 64));
  big = fmaxf(big, __shfl_xor(big, 32, 64));
  if (hi == 0 && big > 0.0f) atomicMax(&colmax[c], __float_as_uint(big));
}

// R -= H[:,I] d (the product's result, column-split partials summed here when JS > 1, plus sigma^2 d
// on the block's own rows), V[I,:] += d, D[I,:] <- 0, squared residual norms per block slice.  A
// workgroup streams its slice (whole rows, contiguous in memory) as a flat array; the squares go to
// LDS, where one thread per column adds them up row by row.  All loads of a pass (UPD_U elements per
// thread, every array) are unconditional and issued before the first use, so a workgroup waits for
// memory once per pass; a slice lies inside one block, so "own rows" is a property of the workgroup.
constexpr int UPD_E = 4096;   // elements of a slice between two column-sum passes
constexpr int UPD_U = 8;

template <int JSC, bool OWN>   // JSC: number of partial images (0: JS of them, any number)
__device__ __forceinline__ void ap_update_pass(float* __restrict__ R, float* __restrict__ V, float* __restrict__ D,
                                               const float* __restrict__ src, int64_t stride, int JS, int64_t base,
                                               int E, int f0, float sigma2, float* sq) {
  const int tid = threadIdx.x;
  int64_t e[UPD_U];
  float hp[JSC > 0 ? JSC : 1][UPD_U], rv[UPD_U], dl[UPD_U], vv[UPD_U];
#pragma unroll
  for (int u = 0; u < UPD_U; ++u) {
    const int f = f0 + tid + 256 * u;
    e[u] = base + (f < E ? f : E - 1);
  }
  if (JSC > 0) {
#pragma unroll
    for (int q = 0; q < JSC; ++q)
#pragma unroll
      for (int u = 0; u < UPD_U; ++u) hp[q][u] = src[(int64_t)q * stride + e[u]];
  } else {
#pragma unroll
    for (int u = 0; u < UPD_U; ++u) hp[0][u] = 0.0f;
    for (int q = 0; q < JS; ++q)
#pragma unroll
      for (int u = 0; u < UPD_U; ++u) hp[0][u] += src[(int64_t)q * stride + e[u]];
  }
#pragma unroll
  for (int u = 0; u < UPD_U; ++u) {
    rv[u] = R[e[u]];
    if (OWN) {
      dl[u] = D[e[u]];
      vv[u] = V[e[u]];
    }
  }
#pragma unroll
  for (int u = 0; u < UPD_U; ++u) {
    const int f = f0 + tid + 256 * u;
    float h = hp[0][u];
    if (JSC > 1) {
      h = 0.0f;
#pragma unroll
      for (int q = 0; q < JSC; ++q) h += hp[q][u];      // same order as the running sum of the general case
    }
    if (OWN) h = fmaf(sigma2, dl[u], h);
    const float r = rv[u] - h;
    if (f < E) {
      if (OWN) {
        V[e[u]] = vv[u] + dl[u];
        D[e[u]] = 0.0f;
      }
      R[e[u]] = r;
      sq[f] = r * r;
    }
  }
}

template <int JSC>
__global__ __launch_bounds__(256) void ap_update_kernel(float* __restrict__ R, float* __restrict__ V,
                                                        float* __restrict__ D, const float* __restrict__ src,
                                                        int64_t stride, int JS, int64_t n, int t, int block, int S,
                                                        int ksel, float sigma2, double* __restrict__ norms) {
  __shared__ float sq[UPD_E];
  int64_t r0, r1;
  slice_rows(n, block, S, &r0, &r1);
  const bool own = (int)(blockIdx.x / S) == ksel;
  const int tid = threadIdx.x;
  constexpr int CG = (GP_MAX_T + 255) / 256;
  double cs[CG];
#pragma unroll
  for (int g = 0; g < CG; ++g) cs[g] = 0.0;
  const int rows_sub = UPD_E / t;
  for (int64_t rs = r0; rs < r1; rs += rows_sub) {
    const int nrow = (int)(rs + rows_sub < r1 ? rows_sub : r1 - rs);
    const int E = nrow * t;
    for (int f0 = 0; f0 < E; f0 += 256 * UPD_U) {
      if (own) ap_update_pass<JSC, true>(R, V, D, src, stride, JS, rs * t, E, f0, sigma2, sq);
      else ap_update_pass<JSC, false>(R, V, D, src, stride, JS, rs * t, E, f0, sigma2, sq);
    }
    __syncthreads();
#pragma unroll
    for (int g = 0; g < CG; ++g) {
      const int c = tid + 256 * g;
      if (c < t)
        for (int row = 0; row < nrow; ++row) cs[g] += (double)sq[row * t + c];
    }
    __syncthreads();
  }
#pragma unroll
  for (int g = 0; g < CG; ++g) {
    const int c = tid + 256 * g;
    if (c < t) norms[(int64_t)blockIdx.x * t + c] = cs[g];
  }
}

// Stopping test per column, choice of the next block, post to the host.  Workgroups of 1024.
// First every workgroup turns the slice partials of its blocks (k = blockIdx.x, blockIdx.x + gridDim.x,
// ..) into per-block squared norms bnorm[k][c]: min(S, 1024 / t) threads per column take every so-many-th
// slice each, and their sums are combined in a fixed order through LDS.  One workgroup alone would have
// to pull all nb S t partials through a single compute unit.  The workgroup that arrives last at the
// ticket counter (release fence before the ticket, acquire fence after it; nobody waits for anybody)
// then sums the blocks per column, applies the stopping rule and picks the next block.
__device__ void ap_block_sums(const double* __restrict__ src, double* __restrict__ bnorm, int nb, int S, int t,
                              double* spart) {
  const int tid = threadIdx.x;
  int CH = 1024 / t;                       // t <= 1024
  if (CH > S) CH = S;
  const int ch = tid / t, c = tid - ch * t;
  for (int k = blockIdx.x; k < nb; k += gridDim.x) {
    if (ch < CH) {
      const double* sp = src + (int64_t)k * S * t + c;
      double v = 0.0;
#pragma unroll 4
      for (int q = ch; q < S; q += CH) v += sp[(int64_t)q * t];
      spart[ch * t + c] = v;
    }
    __syncthreads();
    if (tid < t) {
      double v = 0.0;
      for (int h = 0; h < CH; ++h) v += spart[h * t + tid];
      bnorm[(int64_t)k * t + tid] = v;
    }
    __syncthreads();
  }
}

// per-column totals over the blocks, in 1024 / t segments combined in a fixed order
__device__ void ap_column_totals(const double* bnorm, int nb, int t, double* spart, double* scol) {
  const int tid = threadIdx.x;
  const int nseg = 1024 / t;
  const int per = (nb + nseg - 1) / nseg;
  const int seg = tid / t, c = tid - seg * t;
  if (seg < nseg) {
    double v = 0.0;
    const int k1 = (seg + 1) * per < nb ? (seg + 1) * per : nb;
#pragma unroll 4
    for (int k = seg * per; k < k1; ++k) v += bnorm[(int64_t)k * t + c];
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

__global__ __launch_bounds__(1024) void ap_finalise_kernel(ApDev s, int nb, int S, int t, int init,
                                                           const int* __restrict__ fac_breakdown) {
  __shared__ double sscore[1024];
  __shared__ double scol[GP_MAX_T];
  __shared__ int sidx[1024];
  __shared__ int sfrozen[GP_MAX_T];
  __shared__ int s_any, s_bad, s_last;
  const int tid = threadIdx.x;
  if (init) ap_block_sums(s.normsB, s.bnormB, nb, S, t, sscore);
  ap_block_sums(s.norms, s.bnorm, nb, S, t, sscore);
  __threadfence();
  __syncthreads();
  if (tid == 0) s_last = atomicAdd(s.ticket, 1u) == gridDim.x - 1 ? 1 : 0;
  __syncthreads();
  if (!s_last) return;
  __threadfence();
  if (tid == 0) {
    *s.ticket = 0u;
    s_any = 0;
    s_bad = *fac_breakdown ? 1 : 0;
  }
  if (init) {
    ap_column_totals(s.bnormB, nb, t, sscore, scol);
    if (tid < t) {
      s.bn2[tid] = scol[tid];
      s.zero_rhs[tid] = (scol[tid] == 0.0) ? 1 : 0;
    }
    __syncthreads();
  }
  ap_column_totals(s.bnorm, nb, t, sscore, scol);
  if (tid < t) {
    const int c = tid;
    const double bn2 = s.bn2[c];          // written by this same thread when init
    const int zero = s.zero_rhs[c];
    int fr = init ? zero : s.frozen[c];
    if (init && zero) s.relres[c] = 0.0f;
    if (!fr) {
      const double rel = sqrt(scol[c] / bn2);
      if (!(rel == rel) || rel > 3.0e38) atomicOr(&s_bad, 1);
      s.relres[c] = (float)rel;
      if ((float)rel < s.tol[c]) fr = 1;
    }
    s.frozen[c] = fr;
    sfrozen[c] = fr;
    if (!fr) atomicOr(&s_any, 1);
    s.colmax[c] = 0u;
  }
  __syncthreads();
  // block with the largest residual over the live columns, lowest index on a tie: wave w scores the
  // blocks w, w + 16, ..: lanes take the columns 64 apart, then a butterfly sum (fixed order)
  double best = -1.0;
  int bi = 0x7fffffff;
  {
    const int lane = tid & 63, w = tid >> 6;
    for (int k = w; k < nb; k += 16) {
      double sc = 0.0;
      for (int c = lane; c < t; c += 64)
        if (!sfrozen[c]) sc += s.bnorm[(int64_t)k * t + c];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) sc += __shfl_xor(sc, off, 64);
      if (sc > best) {
        best = sc;
        bi = k;
      }
    }
  }
  sscore[tid] = best;
  sidx[tid] = bi;
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if (tid < off) {
      const double o = sscore[tid + off];
      const int oi = sidx[tid + off];
      if (o > sscore[tid] || (o == sscore[tid] && oi < sidx[tid])) {
        sscore[tid] = o;
        sidx[tid] = oi;
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    ApFlags f = *s.flags;
    if (!init) f.iters += 1;
    if (s_bad) f.breakdown = 1;
    f.all_done = (!s_any || f.breakdown) ? 1 : 0;
    f.sel = sidx[0] < nb ? sidx[0] : 0;
    *s.flags = f;
    s.post->all_done = f.all_done;
    s.post->breakdown = f.breakdown;
    s.post->iters = f.iters;
    s.post->sel = f.sel;
    __threadfence_system();
    s.post->seq = f.iters + 1;
    __threadfence_system();
  }
}

__global__ __launch_bounds__(256) void ap_store_kernel(const float* __restrict__ V, int64_t n, int t,
                                                       const int* __restrict__ zero_rhs, float* __restrict__ out,
                                                       int64_t ldo) {
  const int64_t total = n * t;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
    const int64_t i = e / t;
    const int c = (int)(e - i * t);
    out[i * ldo + c] = zero_rhs[c] ? 0.0f : V[e];
  }
}

// ---- host ------------------------------------------------------------------------------------------
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct ApLayout {
  int nb, BP, batch, win_chunks, S;
  size_t off_hinv, off_A, off_W, off_T, off_DI, off_V, off_R, off_D, off_HP, off_norms, off_normsB, off_bnorm, off_bnormB, off_state, off_kmv, total;
  size_t kmv_bytes;
};

ApLayout ap_layout(const gp_ctx* ctx, int t, int block) {
  ApLayout L;
  L.nb = (int)((ctx->n + block - 1) / block);
  L.BP = (block + TS - 1) / TS * TS;
  L.batch = L.nb < AP_BATCH ? L.nb : AP_BATCH;
  L.win_chunks = (block + 31) / 32 + 1;   // a block that starts inside a chunk touches one more
  const int64_t all_chunks = (ctx->n + 31) / 32;
  if (L.win_chunks > all_chunks) L.win_chunks = (int)all_chunks;
  const size_t bp2 = (size_t)L.BP * L.BP;
  const size_t arr = align_up((size_t)ctx->n * t * sizeof(float), 256);
  // row slices per block in the streaming kernels: enough workgroups to fill the chip when blocks are few
  L.S = (2 * ctx->num_cu + L.nb - 1) / L.nb;
  if (L.S > 256) L.S = 256;
  if (L.S < 1) L.S = 1;
  const size_t nrm = align_up((size_t)L.nb * L.S * t * sizeof(double), 256);
  size_t o = 0;
  L.off_hinv = o; o += align_up((size_t)L.nb * bp2 * sizeof(float), 256);
  L.off_A = o; o += align_up((size_t)L.batch * bp2 * sizeof(fac_t), 256);
  L.off_W = o; o += align_up((size_t)L.batch * bp2 * sizeof(fac_t), 256);
  L.off_T = o; o += align_up((size_t)L.batch * bp2 * sizeof(fac_t), 256);
  L.off_DI = o; o += align_up((size_t)L.batch * L.BP * TS * sizeof(fac_t), 256);
  L.off_V = o; o += arr;
  L.off_R = o; o += arr;
  L.off_D = o; o += arr;
  L.off_HP = o; o += arr;
  L.off_norms = o; o += nrm;
  L.off_normsB = o; o += nrm;
  L.off_bnorm = o; o += align_up((size_t)L.nb * t * sizeof(double), 256);
  L.off_bnormB = o; o += align_up((size_t)L.nb * t * sizeof(double), 256);
  L.off_state = o; o += align_up(sizeof(ApFlags) + 64 + (size_t)t * (sizeof(double) + 2 * sizeof(float) + 3 * sizeof(int)) + 256, 256);
  L.off_kmv = o;
  size_t kb = gp_kmv_scratch_bytes(ctx, t);
  const size_t wb = gp_kmv_window_scratch_bytes(ctx, t, L.win_chunks);
  if (wb > kb) kb = wb;
  L.kmv_bytes = align_up(kb, 256);
  o += L.kmv_bytes;
  L.total = o;
  return L;
}

}  // namespace

size_t gp_ap_workspace_bytes_impl(const gp_ctx* ctx, int t, int block) { return ap_layout(ctx, t, block).total; }

int gp_ap_run(gp_ctx* ctx, const float* dB, int64_t ldb, const float* dX0, float* dV, int64_t ldv, int t,
              const float* h_tol, int block, int max_iters, void* dWork, size_t work_bytes, int* h_iters,
              int* h_kmv_count, float* h_relres, int* h_picks) {
  const ApLayout L = ap_layout(ctx, t, block);
  if (work_bytes < L.total) return gp_fail(ctx, GP_ERR_WORKSPACE, "gp_ap_solve: workspace %zu < %zu bytes", work_bytes, L.total);
  if ((uintptr_t)dWork % 256) return gp_fail(ctx, GP_ERR_WORKSPACE, "gp_ap_solve: workspace not 256-byte aligned");
  hipStream_t st = ctx->stream;
  const int64_t n = ctx->n;
  char* w = (char*)dWork;
  float* Hinv = (float*)(w + L.off_hinv);
  fac_t* A = (fac_t*)(w + L.off_A);
  fac_t* W = (fac_t*)(w + L.off_W);
  fac_t* TT = (fac_t*)(w + L.off_T);
  fac_t* DI = (fac_t*)(w + L.off_DI);
  float* V = (float*)(w + L.off_V);
  float* R = (float*)(w + L.off_R);
  float* D = (float*)(w + L.off_D);
  float* HP = (float*)(w + L.off_HP);
  ApDev s;
  int* fac_breakdown;
  {
    char* q = w + L.off_state;
    s.flags = (ApFlags*)q; q += sizeof(ApFlags);
    fac_breakdown = (int*)q; q += 32;
    s.ticket = (unsigned*)q; q += 32;
    s.bn2 = (double*)q; q += sizeof(double) * t;
    s.tol = (float*)q; q += sizeof(float) * t;
    s.relres = (float*)q; q += sizeof(float) * t;
    s.frozen = (int*)q; q += sizeof(int) * t;
    s.zero_rhs = (int*)q; q += sizeof(int) * t;
    s.colmax = (unsigned*)q; q += sizeof(unsigned) * t;
  }
  s.norms = (double*)(w + L.off_norms);
  s.normsB = (double*)(w + L.off_normsB);
  s.bnorm = (double*)(w + L.off_bnorm);
  s.bnormB = (double*)(w + L.off_bnormB);
  void* kmv_scratch = w + L.off_kmv;

  const size_t need_pinned = sizeof(ApFlags) + sizeof(float) * t * 2;
  if (ctx->pinned_bytes < GP_PIN_POST + sizeof(ApFlags) || need_pinned > GP_PIN_THETA)
    return gp_fail(ctx, GP_ERR_ARG, "gp_ap_solve: t too large for the pinned staging block");
  ApFlags* hflags = (ApFlags*)((char*)ctx->hPinned + GP_PIN_SOLVER);
  float* htol = (float*)((char*)ctx->hPinned + GP_PIN_SOLVER + sizeof(ApFlags));
  float* hrel = htol + t;
  GP_HIP(ctx, hipStreamSynchronize(st));   // the pinned block may still be in use by an earlier call
  for (int c = 0; c < t; ++c) htol[c] = h_tol[c];
  GP_HIP(ctx, hipMemsetAsync(w + L.off_state, 0, L.off_kmv - L.off_state, st));
  GP_HIP(ctx, hipMemcpyAsync(s.tol, htol, sizeof(float) * t, hipMemcpyHostToDevice, st));

  ApFlags* hpost = (ApFlags*)((char*)ctx->hPinned + GP_PIN_POST);
  s.post = (ApFlags*)((char*)ctx->dPinned + GP_PIN_POST);
  hpost->seq = 0;
  auto wait_seq = [&](int want) -> int {
    volatile ApFlags* h = hpost;
    for (unsigned spins = 1;; ++spins) {
      if (h->seq >= want) break;
      if ((spins & 4095u) == 0) {
        const hipError_t q = hipStreamQuery(st);
        if (q == hipSuccess) {          // nothing left to run: the post must be there by now
          if (h->seq >= want) break;
          return gp_fail(ctx, GP_ERR_HIP, "gp_ap_solve: the solver kernels did not report their state");
        }
        if (q != hipErrorNotReady) return gp_fail(ctx, GP_ERR_HIP, "gp_ap_solve: %s", hipGetErrorString(q));
      }
    }
    __atomic_thread_fence(__ATOMIC_ACQUIRE);
    return GP_OK;
  };

  // ---- set-up: the inverse of every diagonal block, AP_BATCH blocks per round of launches
  const int BP = L.BP, nt = BP / TS;
  for (int blk0 = 0; blk0 < L.nb; blk0 += L.batch) {
    const int cnt = L.nb - blk0 < L.batch ? L.nb - blk0 : L.batch;
    hipLaunchKernelGGL(ap_build_kernel, dim3(nt, nt, cnt), dim3(256), 2 * TS * (ctx->d + 1) * sizeof(float), st, ctx->dX,
                       ctx->d, n, (const double*)ctx->dTheta, ctx->kernel, block, BP, blk0, A);
    for (int k0 = 0; k0 < nt; k0 += CHOL_ROUND) {
      const int k1 = k0 + CHOL_ROUND < nt ? k0 + CHOL_ROUND : nt;
      for (int c = k0; c < k1; ++c) {
        // the round's earlier columns applied to column c (tiles (I, c), I >= c)
        if (c > k0) hipLaunchKernelGGL(ap_chol_update_kernel, dim3(1, nt - c, cnt), dim3(256), 0, st, A, BP, k0, c - k0, c);
        hipLaunchKernelGGL(ap_chol_diag_kernel, dim3(cnt), dim3(256), 0, st, A, BP, c, DI, W, fac_breakdown);
        if (nt - c - 1 > 0)
          hipLaunchKernelGGL(ap_chol_panel_kernel, dim3(nt - c - 1, cnt), dim3(256), 0, st, A, BP, c, (const fac_t*)DI);
      }
      // the whole round applied to everything past it
      const int rest = nt - k1;
      if (rest > 0) hipLaunchKernelGGL(ap_chol_update_kernel, dim3(rest, rest, cnt), dim3(256), 0, st, A, BP, k0, k1 - k0, k1);
    }
    for (int sz = 1; sz < nt; sz *= 2) {
      const int pairs = (nt + 2 * sz - 1) / (2 * sz);
      for (int step = 0; step < 2; ++step)
        hipLaunchKernelGGL(ap_trinv_merge_kernel, dim3(sz, sz, pairs * cnt), dim3(256), 0, st, (const fac_t*)A, W, TT, BP, sz,
                           pairs, step);
    }
    {
      const int sbs = cnt * lauum_superblocks(nt);
      hipLaunchKernelGGL(ap_lauum_kernel, dim3(sb_grid(sbs, SB)), dim3(256), 0, st,
                         (const fac_t*)W, BP, cnt, Hinv + (size_t)blk0 * BP * BP);
    }
    GP_HIP(ctx, hipGetLastError());
  }

  // ---- initial residual
  int kmv_count = 0;
  if (dX0) {
    const int rc = gp_kmv_launch(ctx, dX0, ldv, t, HP, t, 1, kmv_scratch, L.kmv_bytes, nullptr);
    if (rc < 0) return rc;
    ++kmv_count;
  }
  const dim3 sgrid(L.nb * L.S), sblock(256);
  const int fgrid = L.nb < 64 ? L.nb : 64;     // workgroups of the finalise kernel
  hipLaunchKernelGGL(ap_init_kernel, sgrid, sblock, 0, st, dB, ldb, dX0, ldv, (const float*)HP, n, t, block, L.S, V, R, D,
                     s.norms, s.normsB);
  hipLaunchKernelGGL(ap_finalise_kernel, dim3(fgrid), dim3(1024), 0, st, s, L.nb, L.S, t, 1, (const int*)fac_breakdown);
  GP_HIP(ctx, hipGetLastError());
  {
    const int rc = wait_seq(1);
    if (rc < 0) return rc;
  }

  const float sigma2 = (float)(ctx->sigma * ctx->sigma);
  // The block solve of a step takes the block choice from the device, so it is queued behind the
  // previous step's finalise kernel before the host has seen that step's outcome: the host's poll and its
  // next launches then run while the block solve does.
  auto launch_solve = [&]() {
    const int full = (int)(n < block ? n : block);
    const int rt = (full + 15) / 16;
    // 64 columns per workgroup read R with 16-byte loads; 32 columns double the workgroups when those
    // would not reach one per compute unit (a block of 2000 has 125 row tiles)
    if (rt * ((t + 63) / 64) >= ctx->num_cu)
      hipLaunchKernelGGL(ap_block_solve_kernel<4>, dim3(rt, (t + 63) / 64), dim3(64 * SOLVE_WAVES), 0, st,
                         (const float*)Hinv, BP, block, n, (const float*)R, t, (const ApFlags*)s.flags,
                         (const int*)s.frozen, D, s.colmax);
    else
      hipLaunchKernelGGL(ap_block_solve_kernel<2>, dim3(rt, (t + 31) / 32), dim3(64 * SOLVE_WAVES), 0, st,
                         (const float*)Hinv, BP, block, n, (const float*)R, t, (const ApFlags*)s.flags,
                         (const int*)s.frozen, D, s.colmax);
  };
  int it = 0;
  if (!hpost->all_done && max_iters > 0) launch_solve();
  while (!hpost->all_done && it < max_iters) {
    const int k = hpost->sel;
    if (k < 0 || k >= L.nb) return gp_fail(ctx, GP_ERR_HIP, "gp_ap_solve: block choice %d out of range", k);
    if (h_picks) h_picks[it] = k;
    const int64_t j0 = (int64_t)k * block;
    const int64_t j1 = j0 + block < n ? j0 + block : n;
    KmvWindow win;
    win.chunk0 = (int)(j0 / 32);
    win.nchunks = (int)((j1 + 31) / 32) - win.chunk0;
    KmvDeferred df = {nullptr, 0, 1};
    const int rc = gp_kmv_launch(ctx, D, t, t, HP, t, 0, kmv_scratch, L.kmv_bytes, s.colmax, nullptr, &df, &win);
    if (rc < 0) return rc;
    {
      const float* src = df.JS > 1 ? df.part : (const float*)HP;
      auto upd = df.JS == 1 ? ap_update_kernel<1> : df.JS == 2 ? ap_update_kernel<2> : df.JS == 3 ? ap_update_kernel<3>
                 : df.JS == 4 ? ap_update_kernel<4> : ap_update_kernel<0>;
      hipLaunchKernelGGL(upd, sgrid, sblock, 0, st, R, V, D, src, df.stride, df.JS, n, t, block, L.S, k, sigma2, s.norms);
    }
    hipLaunchKernelGGL(ap_finalise_kernel, dim3(fgrid), dim3(1024), 0, st, s, L.nb, L.S, t, 0, (const int*)fac_breakdown);
    if (it + 1 < max_iters) launch_solve();      // the next step's, should there be one
    GP_HIP(ctx, hipGetLastError());
    const int rc2 = wait_seq(it + 2);
    if (rc2 < 0) return rc2;
    ++it;
  }

  int sblocks = (int)((n * (int64_t)t + 255) / 256);
  if (sblocks > 8 * ctx->num_cu) sblocks = 8 * ctx->num_cu;
  hipLaunchKernelGGL(ap_store_kernel, dim3(sblocks), dim3(256), 0, st, (const float*)V, n, t, (const int*)s.zero_rhs, dV, ldv);
  GP_HIP(ctx, hipGetLastError());
  GP_HIP(ctx, hipMemcpyAsync(hrel, s.relres, sizeof(float) * t, hipMemcpyDeviceToHost, st));
  GP_HIP(ctx, hipMemcpyAsync(hflags, s.flags, sizeof(ApFlags), hipMemcpyDeviceToHost, st));
  GP_HIP(ctx, hipStreamSynchronize(st));
  if (h_iters) *h_iters = hflags->iters;
  if (h_kmv_count) *h_kmv_count = kmv_count;
  if (h_relres)
    for (int c = 0; c < t; ++c) h_relres[c] = hrel[c];
  if (hflags->breakdown)
    return gp_fail(ctx, GP_ERR_BREAKDOWN, "gp_ap_solve: a diagonal block is not positive definite in fp64, or a non-finite residual (step %d)", hflags->iters);
  return hflags->all_done ? GP_OK : GP_NOT_CONVERGED;
}
