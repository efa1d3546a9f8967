// Marginal-likelihood gradient estimator (paper Section 2 gradient equation with the Section 2.1
// trace estimator), split-fp16 matrix-core tile pass.  Same mathematics as the fp32 pass:
//   g_k = sum_ij w_ij (dH/dtheta_k)_ij,  w_ij = A_i . C_j,  G = w .* psi,  row sums of G Q with
//   Q = [xs, xs^2, 1], plus one vector-ALU column sum_j w_ij K_ij / a^2 for the amplitude.
// All three contractions of a 32x32 tile of pairs run on v_mfma_f32_32x32x16_f16 with operands split
// into two fp16 pieces (three products per fp32 product, fp32 accumulation):
//   1. S[j][i]  = XA_j . XB_i        the distance chain of the K V pass (same packed operands)
//   2. W'[j][i] = C'_j . A'_i        C' = C scaled per column to max in [2^6, 2^7), A' carries the
//                                    inverse column scales and a global power of two alpha chosen so
//                                    that |W' psi| < 2^15 (from sum_c max|A_c| max|C_c| >= |w_ij|)
//   3. OUT_i   += G'[i][j] Q'_j      G' = W' psi split on the VALU, Q' = 2^qshift Q pre-split
// The epilogue removes alpha and 2^qshift.  K and w are never stored.
#include <cstdlib>

#include "gpws_internal.h"

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr int C_TOP = 7;                    // max |C'_c| in [2^6, 2^7)
constexpr int W_TOP = 13;                   // alpha sum_c max|A_c| max|C_c| <= 2^13, so |W' psi| <= 3 2^13 < 2^15
constexpr int GRAD_TBLOCK_H = 80;           // right-hand-side columns per tile pass (5 k-steps of 16)

struct GradArgsH {
  const u32x4* XA[3];     // column-side distance pieces [(chunk*KH + kh)*64 + lane]
  const u32x4* XB[3];     // row-side distance pieces
  const u32x4* CA;        // C' images, column side: [((chunk*2 + part)*KT + kt)*64 + lane]
  const u32x4* AB;        // A' images, row side, same indexing by sub-tile
  const u32x4* QP;        // Q' images of this column pass: [(((chunk*2 + mh)*NT + nt)*2 + part)*64 + lane]
  const int* scales;      // [0] = exponent of alpha
  float* OUT;             // [JS][n][ldo]
  int64_t ldo;
  int64_t split_stride;
  int64_t n;
  int nchunks;
  int col0, ncols;        // Q columns of this pass
  int vcol;               // output column of sum_j w_ij K_ij / a^2, or -1
  int JS, cps;
  int qshift;             // Q' = 2^qshift Q
  int slot_kh, slot_h, slot_e;   // where the row-side operand carries the SE exponent shift, or -1
};

__device__ __forceinline__ f16x8 as_f16x8(u32x4 v) { return __builtin_bit_cast(f16x8, v); }

// x - (float)half H of pk, one v_fma_mix_f32 (source 0 read as the fp16 half, sources 1 and 2 as fp32)
template <int H>
__device__ __forceinline__ float minus_half(unsigned pk, float x) {
  float r;
  if (H == 0) asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(pk), "v"(x));
  else asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(pk), "v"(x));
  return r;
}

template <int KIND, int KH, int XP, int KT, int NT>
__global__ __launch_bounds__(256) void grad_tile_f16_kernel(GradArgsH p) {
  constexpr int W = 4;
  constexpr int XA_G = XP * KH;          // groups of 64 16-byte units per stage
  constexpr int C_G = 2 * KT;
  constexpr int Q_G = 4 * NT;
  constexpr int G = XA_G + C_G + Q_G;
  constexpr int C_OFF = XA_G * 64;
  constexpr int Q_OFF = (XA_G + C_G) * 64;
  constexpr int STAGE = G * 64;
  constexpr int NS = G > 24 ? 2 : 3;     // LDS ring: chunks up to ch + NS - 1 in flight while ch is consumed
  constexpr int DEPTH = NS - 1;
  constexpr int LPW = (G + W - 1) / W;   // group loads per wave per chunk
  static_assert((DEPTH - 1) * LPW < 64, "vmcnt cannot express the pipeline depth");
  __shared__ u32x4 lds[NS][STAGE];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: lets the compiler branch on it
  const int h = lane >> 5;
  const int li = lane & 31;
  const int js = blockIdx.x % p.JS;
  const int rb = blockIdx.x / p.JS;
  const int sub0 = rb * W + wave;
  // The workgroup's column range [r_begin, r_end) is walked in segments [c_begin, c_end) of at most
  // GP_FLUSH_CHUNKS chunks; the accumulators are added into OUT after each segment (see flush below).
  const int r_begin = js * p.cps;
  const int r_end = min(p.nchunks, r_begin + p.cps);
  int c_begin = r_begin;
  int c_end = min(r_end, c_begin + GP_FLUSH_CHUNKS);

  // row-side operands stay in registers for the whole pass
  f16x8 xb[XP][KH], abh[KT], abl[KT];
#pragma unroll
  for (int pc = 0; pc < XP; ++pc)
#pragma unroll
    for (int kh = 0; kh < KH; ++kh) xb[pc][kh] = as_f16x8(p.XB[pc][((int64_t)sub0 * KH + kh) * 64 + lane]);
  if (KIND == GP_SE_ARD) {
    // the K V pass carries phi as 2^15 phi through one extra operand component; psi is used unshifted here
#pragma unroll
    for (int kh = 0; kh < KH; ++kh)
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (kh == p.slot_kh && e == p.slot_e && h == p.slot_h) xb[0][kh][e] = (_Float16)0.0f;
  }
#pragma unroll
  for (int kt = 0; kt < KT; ++kt) {
    abh[kt] = as_f16x8(p.AB[((int64_t)(sub0 * 2 + 0) * KT + kt) * 64 + lane]);
    abl[kt] = as_f16x8(p.AB[((int64_t)(sub0 * 2 + 1) * KT + kt) * 64 + lane]);
  }

  f32x16 acc[NT];
  float accv = 0.0f;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nt][r] = 0.0f;

  // global -> LDS staging without registers (global_load_lds_dwordx4), DEPTH chunks ahead; every wave
  // issues LPW loads per chunk (surplus slots repeat the last group) so one vmcnt value per wave tells
  // when its share of a chunk has landed, and the barrier that follows publishes the whole chunk.
  const u32x4* g_src[LPW];
  int g_stride[LPW];
  unsigned g_lds[LPW];
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) void*)&lds[0][0];
#pragma unroll
  for (int x = 0; x < LPW; ++x) {
    const int g = min(wave + W * x, G - 1);
    if (g < XA_G) {
      g_src[x] = p.XA[g / KH] + (g % KH) * 64 + lane;
      g_stride[x] = KH * 64;
    } else if (g < XA_G + C_G) {
      g_src[x] = p.CA + (g - XA_G) * 64 + lane;
      g_stride[x] = C_G * 64;
    } else {
      g_src[x] = p.QP + (g - XA_G - C_G) * 64 + lane;
      g_stride[x] = Q_G * 64;
    }
    g_lds[x] = __builtin_amdgcn_readfirstlane(lds_base + 16u * (unsigned)(g * 64));
  }
  // inline assembly keeps the ordering explicit (s_waitcnt vmcnt(N) + barrier) instead of the
  // compiler's conservative drain of all LDS-DMA loads at every barrier; m0 is restored
  auto dma16 = [](const u32x4* src, unsigned lds_addr) {
    // m0 carries the LDS address of the load; it is declared clobbered, so the compiler keeps nothing in it
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(lds_addr) : "memory", "m0");
  };
  auto issue_chunk = [&](int ch_target) {
    const int ch = min(ch_target, c_end - 1);           // past the end: harmless reload of the last chunk
    const unsigned stage_off = (unsigned)((ch_target - c_begin) % NS) * (unsigned)(STAGE * 16);
#pragma unroll
    for (int x = 0; x < LPW; ++x) dma16(g_src[x] + (int64_t)ch * g_stride[x], __builtin_amdgcn_readfirstlane(g_lds[x] + stage_off));
  };
  constexpr int WAIT_N = (DEPTH - 1) * LPW;   // all but the newest DEPTH - 1 chunks have landed

  // Writes the accumulators to OUT (first: stores; later: adds to what is there) without alpha and
  // 2^qshift, and clears them.  Doing so after every segment keeps the chains of fp32 partial sums
  // short; the same threads read and write the same elements, in a fixed order.
  // The weights of odd row sub-tiles are packed with their sign flipped (grad_pack_ac_f16_kernel) and the
  // flip is undone here: what is left of the one-sided rounding described at the weight chain below
  // then enters the sums over rows with alternating sign instead of adding up.
  const int alpha_exp = p.scales[0];
  const float row_sign = (sub0 & 1) ? -1.0f : 1.0f;
  const float oscale = row_sign * ldexpf(1.0f, -alpha_exp - p.qshift);
  const float vscale = row_sign * ldexpf(1.0f, -alpha_exp);
  float* out = p.OUT + (int64_t)js * p.split_stride;
  auto flush = [&](bool first) {
    // an opaque zero keeps the address arithmetic of the flush inside it: hoisted out of the segment
    // loop it would hold dozens of registers across the main loop
    int zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(zero));
    const int64_t ibase = (int64_t)sub0 * 32 + zero;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int c = li + 32 * nt;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t i = ibase + 8 * (r >> 2) + 4 * h + (r & 3);
        if (i < p.n && c < p.ncols) {
          float v = oscale * acc[nt][r];
          if (!first) v += out[i * p.ldo + p.col0 + c];
          out[i * p.ldo + p.col0 + c] = v;
        }
        acc[nt][r] = 0.0f;
      }
    }
    if (p.vcol >= 0) {
      const float tot = accv + __shfl_xor(accv, 32);
      const int64_t i = ibase + li;
      if (h == 0 && i < p.n) {
        float v = vscale * tot;
        if (!first) v += out[i * p.ldo + p.vcol];
        out[i * p.ldo + p.vcol] = v;
      }
      accv = 0.0f;
    }
  };
  bool first = true;

  for (;;) {
#pragma unroll
  for (int d0 = 0; d0 < DEPTH; ++d0) issue_chunk(c_begin + d0);
  for (int ch = c_begin; ch < c_end; ++ch) {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(WAIT_N) : "memory");
    __syncthreads();              // chunk ch is complete in LDS; every wave is done with chunk ch - 1
    issue_chunk(ch + DEPTH);      // refills the stage chunk ch - 1 occupied
    const u32x4* s = lds[(ch - c_begin) % NS];

    f32x16 S, Wc;
#pragma unroll
    for (int r = 0; r < 16; ++r) { S[r] = 0.0f; Wc[r] = 0.0f; }
#pragma unroll
    for (int kh = 0; kh < KH; ++kh) {
      f16x8 xa[XP];
#pragma unroll
      for (int pc = 0; pc < XP; ++pc) xa[pc] = as_f16x8(s[(pc * KH + kh) * 64 + lane]);
      // smallest terms first
      if constexpr (XP == 3) {
        S = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[1], xb[1][kh], S, 0, 0, 0);
        S = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[2], xb[0][kh], S, 0, 0, 0);
        S = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[0], xb[XP - 1][kh], S, 0, 0, 0);
      }
      S = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[1], xb[0][kh], S, 0, 0, 0);
      S = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[0], xb[1][kh], S, 0, 0, 0);
      S = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[0], xb[0][kh], S, 0, 0, 0);
    }
    // Per k-step the hi*hi products first, on purpose.  This matrix instruction rounds to nearest when
    // its accumulator input is the largest addend, but an accumulator input smaller than the products is
    // cut off below half a unit in the last place of the result toward minus infinity (measured on
    // MI355X).  Small cross terms summed first and the hi*hi products added on top of them would give
    // every w_ij a bias of about -2^-25 |w_ij| of one sign, which the sum over all pairs does not average
    // out while the terms themselves cancel (V nearly orthogonal to K's large eigenvectors, as after a solve).
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      const f16x8 ch_ = as_f16x8(s[C_OFF + (0 * KT + kt) * 64 + lane]);
      const f16x8 cl_ = as_f16x8(s[C_OFF + (1 * KT + kt) * 64 + lane]);
      Wc = __builtin_amdgcn_mfma_f32_32x32x16_f16(ch_, abh[kt], Wc, 0, 0, 0);
      Wc = __builtin_amdgcn_mfma_f32_32x32x16_f16(ch_, abl[kt], Wc, 0, 0, 0);
      Wc = __builtin_amdgcn_mfma_f32_32x32x16_f16(cl_, abh[kt], Wc, 0, 0, 0);
    }
    if (ch == sub0) {   // the pair (i, i): r^2 = 0 exactly
      asm volatile("" ::: "memory");   // keeps this a real (wave-uniform) branch instead of selects on every chunk
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (8 * (r >> 2) + 4 * h + (r & 3) == li) S[r] = 0.0f;
    }

#pragma unroll
    for (int mh = 0; mh < 2; ++mh) {
      u32x4 gh, gl;
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        float g[2];
#pragma unroll
        for (int z = 0; z < 2; ++z) {
          const int r = 8 * mh + 2 * e2 + z;
          float psi, kval;
          if (KIND == GP_SE_ARD) {
            psi = __builtin_amdgcn_exp2f(S[r]);                 // S = -log2(e)/2 r^2
            kval = psi;
          } else {
            // S = 3 r^2; rounding-level negatives are mirrored (free source modifier), (i, i) is exactly 0
            const float u = __builtin_amdgcn_sqrtf(__builtin_fabsf(S[r]));
            const float e = __builtin_amdgcn_exp2f(-LOG2E * u);
            psi = 3.0f * e;
            kval = fmaf(u, e, e);
          }
          g[z] = Wc[r] * psi;
          accv = fmaf(Wc[r], kval, accv);
        }
        // hi = g truncated to fp16, lo = g - hi read from the packed halves by the mixed-precision FMA
        gh[e2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(g[0], g[1]));
        gl[e2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(minus_half<0>(gh[e2], g[0]), minus_half<1>(gh[e2], g[1])));
      }
      const f16x8 ah = as_f16x8(gh), al = as_f16x8(gl);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const f16x8 bh = as_f16x8(s[Q_OFF + ((mh * NT + nt) * 2 + 0) * 64 + lane]);
        const f16x8 bl = as_f16x8(s[Q_OFF + ((mh * NT + nt) * 2 + 1) * 64 + lane]);
        acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bh, acc[nt], 0, 0, 0);
        acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bl, acc[nt], 0, 0, 0);
        acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, acc[nt], 0, 0, 0);
      }
    }
  }
  // no LDS write may be in flight, and no wave still reading, when the ring is refilled or released
  asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
  __syncthreads();
  flush(first);
  first = false;
  if (c_end >= r_end) break;
  c_begin = c_end;
  c_end = min(r_end, c_begin + GP_FLUSH_CHUNKS);
  }
}

// exponent e with m = f 2^e, f in [0.5, 1); dflt for m = 0
__device__ __forceinline__ int exponent_of(float m, int dflt) {
  if (!(m > 0.0f)) return dflt;
  int e;
  (void)frexpf(m, &e);
  return e < -100 ? -100 : (e > 100 ? 100 : e);
}

// scales of one block of right-hand-side columns [t0, t0 + tb): scales[0] = exponent of alpha,
// scales[1 + m] = exponent e_m with max |C_m| in [2^(e_m - 1), 2^e_m).  One workgroup, fixed-order sum.
__global__ __launch_bounds__(128) void grad_scales_kernel(const unsigned* __restrict__ cmV, const unsigned* __restrict__ cmB,
                                                          int t0, int tb, float half_w, float probe_w,
                                                          int* __restrict__ scales) {
  __shared__ float bound[128];
  const int m = threadIdx.x;
  float b = 0.0f;
  if (m < tb) {
    const int col = t0 + m;
    const float maxV = __uint_as_float(cmV[col]);
    const float maxC = col == 0 ? maxV : __uint_as_float(cmB[col]);
    const float maxA = fabsf(col == 0 ? half_w : probe_w) * maxV;
    scales[1 + m] = exponent_of(maxC, C_TOP);
    b = maxA * maxC;
  }
  bound[m] = b;
  __syncthreads();
  if (m == 0) {
    float wb = 0.0f;
    for (int k = 0; k < tb; ++k) wb += bound[k];
    // |w_ij| <= wb <= 2^e, so alpha = 2^(W_TOP - e) keeps alpha |w_ij| <= 2^W_TOP
    scales[0] = (wb > 0.0f && wb < 3.0e38f) ? W_TOP - exponent_of(wb, W_TOP) : 0;
  }
}

__device__ __forceinline__ void split2(float v, float& hi, float& lo) {
  // hi is what fp16 truncation really stores (also for subnormal results), lo the exact remainder
  const auto pk = __builtin_amdgcn_cvt_pkrtz(v, 0.0f);
  hi = (float)pk[0];
  lo = v - hi;
}

// C' (column side) and A' (row side) images of columns [t0, t0 + tb); one thread per (chunk, kt, lane)
__global__ __launch_bounds__(256) void grad_pack_ac_f16_kernel(const float* __restrict__ V, int64_t ldv,
                                                               const float* __restrict__ B, int64_t ldb, int64_t n,
                                                               int64_t nchunks_pad, int t0, int tb, int KT, float half_w,
                                                               float probe_w, const int* __restrict__ scales,
                                                               u32x4* __restrict__ CA, u32x4* __restrict__ AB) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gid >= nchunks_pad * KT * 64) return;
  const int lane = (int)(gid & 63);
  const int kt = (int)((gid >> 6) % KT);
  const int64_t chunk = (gid >> 6) / KT;
  const int64_t row = chunk * 32 + (lane & 31);
  const int alpha_exp = scales[0];
  u32x4 ch, cl, ah, al;
#pragma unroll
  for (int e2 = 0; e2 < 4; ++e2) {
    float c_hi[2], c_lo[2], a_hi[2], a_lo[2];
#pragma unroll
    for (int z = 0; z < 2; ++z) {
      const int m = 16 * kt + 8 * (lane >> 5) + 2 * e2 + z;
      float c = 0.0f, a = 0.0f;
      if (row < n && m < tb) {
        const int col = t0 + m;
        const int ec = scales[1 + m];
        const float v = V[row * ldv + col];
        const float cv = col == 0 ? v : B[row * ldb + col];
        c = ldexpf(cv, C_TOP - ec);
        a = ldexpf((col == 0 ? half_w : probe_w) * v, alpha_exp + ec - C_TOP);
        if (chunk & 1) a = -a;   // undone by the tile kernel's epilogue (row_sign)
      }
      split2(c, c_hi[z], c_lo[z]);
      split2(a, a_hi[z], a_lo[z]);
    }
    ch[e2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(c_hi[0], c_hi[1]));
    cl[e2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(c_lo[0], c_lo[1]));
    ah[e2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(a_hi[0], a_hi[1]));
    al[e2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(a_lo[0], a_lo[1]));
  }
  const int64_t u_hi = ((chunk * 2 + 0) * KT + kt) * 64 + lane;
  const int64_t u_lo = ((chunk * 2 + 1) * KT + kt) * 64 + lane;
  CA[u_hi] = ch; CA[u_lo] = cl;
  AB[u_hi] = ah; AB[u_lo] = al;
}

// Q' images of Q columns [col0, col0 + ncols), Q = [xs (d), xs^2 (d), 1]; one thread per (chunk, mh, nt, lane).
// Element e of lane l is row 32 chunk + 16 mh + 8 (e/4) + 4 (l/32) + e%4 (the register order of the
// accumulator layout that G' comes in), column col0 + 32 nt + l%32.
__global__ __launch_bounds__(256) void grad_pack_q_f16_kernel(const float* __restrict__ Xs, int64_t n, int d,
                                                              int nchunks, int NT, int col0, int ncols, int qshift,
                                                              u32x4* __restrict__ QP) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gid >= (int64_t)nchunks * 2 * NT * 64) return;
  const int lane = (int)(gid & 63);
  int64_t q = gid >> 6;
  const int nt = (int)(q % NT); q /= NT;
  const int mh = (int)(q & 1);
  const int64_t chunk = q >> 1;
  const int hh = lane >> 5;
  const int cc = 32 * nt + (lane & 31);
  const int col = col0 + cc;
  const bool cok = cc < ncols;
  u32x4 hi, lo;
#pragma unroll
  for (int e2 = 0; e2 < 4; ++e2) {
    float fh[2], fl[2];
#pragma unroll
    for (int z = 0; z < 2; ++z) {
      const int e = 2 * e2 + z;
      const int64_t j = chunk * 32 + 16 * mh + 8 * (e >> 2) + 4 * hh + (e & 3);
      float v = 0.0f;
      if (cok && j < n) {
        if (col < d) v = Xs[j * d + col];
        else if (col < 2 * d) { const float x = Xs[j * d + col - d]; v = x * x; }
        else v = 1.0f;
        v = ldexpf(v, qshift);
      }
      split2(v, fh[z], fl[z]);
    }
    hi[e2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(fh[0], fh[1]));
    lo[e2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(fl[0], fl[1]));
  }
  u32x4* dst = QP + ((chunk * 2 + mh) * NT + nt) * 2 * 64;
  dst[lane] = hi;
  dst[64 + lane] = lo;
}

typedef void (*gradh_fn)(GradArgsH);

template <int KIND, int KH, int XP>
gradh_fn pick_kt_nt(int KT, int NT) {
  if (KT == 2) return NT == 1 ? grad_tile_f16_kernel<KIND, KH, XP, 2, 1> : grad_tile_f16_kernel<KIND, KH, XP, 2, 2>;
  return NT == 1 ? grad_tile_f16_kernel<KIND, KH, XP, 5, 1> : grad_tile_f16_kernel<KIND, KH, XP, 5, 2>;
}

template <int KIND, int XP>
gradh_fn pick_kh(int KH, int KT, int NT) {
  switch (KH) {
    case 1: return pick_kt_nt<KIND, 1, XP>(KT, NT);
    case 2: return pick_kt_nt<KIND, 2, XP>(KT, NT);
    case 3: return pick_kt_nt<KIND, 3, XP>(KT, NT);
    case 4: return pick_kt_nt<KIND, 4, XP>(KT, NT);
    case 6: return pick_kt_nt<KIND, 6, XP>(KT, NT);
    case 8: return pick_kt_nt<KIND, 8, XP>(KT, NT);
  }
  return nullptr;
}

gradh_fn pick_gradh(int kind, int KH, int XP, int KT, int NT) {
  if (kind == GP_SE_ARD) return XP == 2 ? pick_kh<GP_SE_ARD, 2>(KH, KT, NT) : pick_kh<GP_SE_ARD, 3>(KH, KT, NT);
  return XP == 2 ? pick_kh<GP_MATERN32_ARD, 2>(KH, KT, NT) : pick_kh<GP_MATERN32_ARD, 3>(KH, KT, NT);
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

int gp_grad_run_f16(gp_ctx* ctx, const float* dV, int64_t ldv, const float* dB, int64_t ldb, int t,
                    double* h_grad) {
  const int d = ctx->d;
  const int64_t n = ctx->n;
  const int nq = 2 * d + 2;         // Q columns (2d+1) + the vector-ALU column
  const int ldq = 2 * d + 1;
  const int s = t - 1;
  const float half_w = 0.5f;
  const float probe_w = s > 0 ? (float)(-0.5 / (double)s) : 0.0f;

  // plan: one 32-row sub-tile per wave; the column range is split over workgroups until the chip is
  // full (the kernel itself flushes its accumulators at intervals, so long column ranges need no split)
  const int64_t chunks = (n + 31) / 32;
  const int64_t chunks_pad = ctx->n_pad / 32;
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
  const int KTmax = t <= 32 ? 2 : 5;
  // workgroups of the fp64 reduction: one step of 256 / (d + 2) rows each when n allows, so that
  // enough loads are in flight (the kernel is latency-bound at small n)
  int G;
  {
    const int per_step = 256 / (d + 2 < 256 ? d + 2 : 256);
    const int64_t want = (n + per_step - 1) / per_step;
    G = (int)(want < 8 * ctx->num_cu ? want : 8 * ctx->num_cu);
    if (G < 1) G = 1;
  }
  const size_t op_bytes = align_up((size_t)chunks_pad * 2 * KTmax * 64 * 16, 256);
  const size_t q_bytes = align_up((size_t)chunks * 2 * 2 * 2 * 64 * 16, 256);
  const size_t out_bytes = align_up((size_t)JS * n * nq * sizeof(float), 256);
  const size_t part_bytes = align_up((size_t)G * (d + 2) * sizeof(double), 256);
  const size_t acc_bytes = align_up((size_t)(d + 2) * sizeof(double), 256);
  const size_t cm_bytes = align_up((size_t)t * sizeof(unsigned), 256);
  const size_t sc_bytes = align_up((size_t)(1 + GRAD_TBLOCK_H) * sizeof(int), 256);
  int rc = gp_ensure_scratch(ctx, 2 * op_bytes + q_bytes + out_bytes + part_bytes + acc_bytes + 2 * cm_bytes + sc_bytes);
  if (rc < 0) return rc;
  char* w = (char*)ctx->dScratch;
  u32x4* CA = (u32x4*)w; w += op_bytes;
  u32x4* AB = (u32x4*)w; w += op_bytes;
  u32x4* QP = (u32x4*)w; w += q_bytes;
  float* OUT = (float*)w; w += out_bytes;
  double* part = (double*)w; w += part_bytes;
  double* acc = (double*)w; w += acc_bytes;
  unsigned* cmV = (unsigned*)w; w += cm_bytes;
  unsigned* cmB = (unsigned*)w; w += cm_bytes;
  int* scales = (int*)w;
  hipStream_t st = ctx->stream;

  GP_HIP(ctx, hipMemsetAsync(acc, 0, acc_bytes + 2 * cm_bytes, st));   // acc, cmV, cmB lie back to back
  rc = gp_launch_colmax(ctx, dV, ldv, t, cmV, dB, ldb, cmB, true);
  if (rc < 0) return rc;

  // Q' = 2^qshift Q with max |Q| = max(1, max_i |xs_i|^2) kept below 2^15
  int qshift = 8;
  {
    int e = 0;
    (void)frexpf(ctx->max_norm > 1.0f ? ctx->max_norm : 1.0f, &e);   // max <= 2^e
    if (14 - e < qshift) qshift = 14 - e;
    if (qshift < 0) qshift = 0;
  }

  GradArgsH a;
  for (int pc = 0; pc < 3; ++pc) {
    a.XA[pc] = (const u32x4*)ctx->dXAh[pc];
    a.XB[pc] = (const u32x4*)ctx->dXBh[pc];
  }
  a.CA = CA;
  a.AB = AB;
  a.QP = QP;
  a.scales = scales;
  a.OUT = OUT;
  a.ldo = nq;
  a.split_stride = n * (int64_t)nq;
  a.n = n;
  a.nchunks = (int)chunks;
  a.JS = JS;
  a.cps = cps;
  a.qshift = qshift;
  a.slot_kh = a.slot_h = a.slot_e = -1;
  if (ctx->kernel == GP_SE_ARD) {
    const int k = d + 2;
    a.slot_kh = k / 16;
    a.slot_h = (k % 16) / 8;
    a.slot_e = k % 8;
  }
  const dim3 grid(row_blocks * JS), block(256);

  for (int t0 = 0; t0 < t; t0 += GRAD_TBLOCK_H) {
    const int tb = t - t0 < GRAD_TBLOCK_H ? t - t0 : GRAD_TBLOCK_H;
    const int KT = tb <= 32 ? 2 : 5;
    hipLaunchKernelGGL(grad_scales_kernel, dim3(1), dim3(128), 0, st, (const unsigned*)cmV, (const unsigned*)cmB, t0, tb,
                       half_w, probe_w, scales);
    GP_HIP(ctx, hipGetLastError());
    {
      const int64_t units = chunks_pad * KT * 64;
      hipLaunchKernelGGL(grad_pack_ac_f16_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, st, dV, ldv, dB, ldb,
                         n, chunks_pad, t0, tb, KT, half_w, probe_w, (const int*)scales, CA, AB);
      GP_HIP(ctx, hipGetLastError());
    }
    int vcol = nq - 1;
    for (int c = 0; c < ldq;) {
      const int rem = ldq - c;
      const int NT = rem > 32 ? 2 : 1;
      a.col0 = c;
      a.ncols = rem < 32 * NT ? rem : 32 * NT;
      a.vcol = vcol;
      vcol = -1;
      {
        const int64_t units = chunks * 2 * NT * 64;
        hipLaunchKernelGGL(grad_pack_q_f16_kernel, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, st,
                           (const float*)ctx->dXs, n, d, (int)chunks, NT, a.col0, a.ncols, qshift, QP);
        GP_HIP(ctx, hipGetLastError());
      }
      gradh_fn fn = pick_gradh(ctx->kernel, ctx->KH, ctx->XP, KT, NT);
      if (!fn) return gp_fail(ctx, GP_ERR_ARG, "gp_mll_grad: no fp16 kernel for KH=%d", ctx->KH);
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
