// Matrix-free product OUT = K V (+ sigma^2 V), split-fp16 matrix-core path.
//
// On gfx950 the fp32 MFMA shares the SIMD's FMA lanes with the VALU (measured: VALU work adds to
// fp32-MFMA time instead of hiding under it), while the fp16 MFMA runs on the matrix cores at 16x the
// rate and overlaps with VALU work.  This path therefore evaluates both contractions of the tile pass
// with v_mfma_f32_32x32x16_f16 on operands split into fp16 pieces, fp32 accumulation:
//   x = hi + mid (+ lo), each piece an 11-bit fp16 mantissa, hi and mid obtained by truncation, so
//   a.b ~ ah.bh + ah.bm + am.bh (+ ah.bl + al.bh + am.bm): relative error 2^-22 (2^-33), i.e. fp32-class.
// The VALU keeps what needs fp32: the kernel function (exp2 / sqrt) and the split of phi.
//
// Per 32x32 tile of pairs (j, i), one wavefront:
//   1. S[j][i] = XA_j . XB_i     3 (or 6) MFMAs per 16 components      (= g r^2_ij [+ 15 for SE])
//   2. phi' = 2^15 phi(S)        VALU; hi = phi' truncated to fp16, lo = phi' - hi; packed to fp16 pairs
//   3. OUT_i += phi'[i][j] V'_j  2 k-steps x NT x 3 MFMAs; V' = V scaled per column by a power of two
//                                so that max |V'_c| is in [2^13, 2^14), pre-split and pre-packed
// The accumulator layout of step 1 (lane = i, register r <-> j = 8(r/4) + 4(lane/32) + r%4) gives each lane
// eight consecutive registers per k-step that are exactly its eight A-operand elements, provided the
// V' rows are packed in that order; phi never leaves registers, K is never stored.
#include <cstdlib>

#include "gpws_internal.h"

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr unsigned HI_MASK = 0xFFFFE000u;       // keeps sign, exponent and the top 10 mantissa bits
constexpr int PHI_SHIFT = 15;                   // phi' = 2^15 phi <= 32768 stays inside fp16's range
constexpr int V_TOP = 14;                       // max |V'_c| in [2^13, 2^14)

// exponent e with max = f 2^e, f in [0.5, 1); 14 for an all-zero column (scale 1)
__device__ __forceinline__ int column_exponent(unsigned max_bits) {
  const float m = __uint_as_float(max_bits);
  if (!(m > 0.0f)) return V_TOP;
  int e;
  (void)frexpf(m, &e);
  return e < -60 ? -60 : e;
}

struct TileArgsH {
  const u32x4* XA[3];     // column-side pieces, 16-byte units [(chunk*KH + kh)*64 + lane]
  const u32x4* XB[3];     // row-side pieces
  const u32x4* VP;        // packed V' images of this pass, [chunk][mh][nt][part][lane]
  const float* VY;        // [n_pad] the VALU column, unscaled (zeros when unused)
  const float* V;         // the caller's V (noise term in the epilogue)
  int64_t ldv;
  const unsigned* colmax; // [t] bit patterns of max_i |V_ic|
  float* OUT;
  int64_t ldo;
  int64_t split_stride;
  int64_t n;               // rows of the output (the context's n, or m for a rectangular product)
  int diag;                // square product: the pair (i, i) gets r^2 = 0 exactly
  int nchunks;             // column chunks (always the context's points)
  int col0, ncols, vcol;
  int JS, cps;             // column-range splits inside this launch, chunks per split
  float a2, sigma2;
  int add_noise;
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

// W wavefronts per workgroup: every workgroup streams all of V' and XA through its LDS, so the
// L2-to-LDS traffic of a launch is inversely proportional to the rows a workgroup owns (32 MI W).
template <int KIND, int KH, int XP, int NT, int MI, int W>
__global__ __launch_bounds__(64 * W) __attribute__((amdgpu_waves_per_eu(2, 2))) void kmv_tile_f16_kernel(TileArgsH p) {
  // One pipeline stage in LDS, in 16-byte units: G groups of 64 units (one wave-wide 16-byte load
  // each): XP*KH groups of XA pieces, then 4*NT groups of V' images; then one 8-unit y slot per wave.
  constexpr int XA_G = XP * KH;
  constexpr int V_G = 4 * NT;
  constexpr int G = XA_G + V_G;
  constexpr int V_OFF = XA_G * 64;
  constexpr int V_U = V_G * 64;
  constexpr int VY_OFF = G * 64;
  constexpr int STAGE = VY_OFF + 8 * W;
  constexpr int NS = G > 12 ? 3 : 4;               // stages: chunks up to ch + NS - 1 are in flight while ch is consumed
  constexpr int DEPTH = NS - 1;
  constexpr int LPW = (G + W - 1) / W;             // group loads per wave per chunk
  constexpr int LPC = LPW + 1;                     // + the y slot
  static_assert((DEPTH - 1) * LPC < 64, "vmcnt cannot express the pipeline depth");
  __shared__ u32x4 lds[NS][STAGE];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: lets the compiler branch on it
  const int h = lane >> 5;
  const int li = lane & 31;
  const int js = blockIdx.x % p.JS;
  const int rb = blockIdx.x / p.JS;
  const int sub0 = (rb * W + wave) * MI;
  // The workgroup's column range [r_begin, r_end) is walked in segments [c_begin, c_end) of at most
  // GP_FLUSH_CHUNKS chunks; the accumulators are added into OUT after each segment (see flush below).
  const int r_begin = js * p.cps;
  const int r_end = min(p.nchunks, r_begin + p.cps);
  int c_begin = r_begin;
  int c_end = min(r_end, c_begin + GP_FLUSH_CHUNKS);

  // row-side operands: registers for the whole pass
  f16x8 xb[MI][XP][KH];
#pragma unroll
  for (int m = 0; m < MI; ++m)
#pragma unroll
    for (int pc = 0; pc < XP; ++pc)
#pragma unroll
      for (int kh = 0; kh < KH; ++kh)
        xb[m][pc][kh] = as_f16x8(p.XB[pc][((int64_t)(sub0 + m) * KH + kh) * 64 + lane]);

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

  // Staging goes global -> LDS directly (global_load_lds_dwordx4: lane L of a wave lands at the
  // wave's LDS base + 16 L), NS - 1 chunks ahead of the chunk being consumed, so no registers are held
  // and the L2/HBM latency is spread over several chunks of work.  Every wave issues the same number of
  // loads per chunk (its groups wave, wave + W, ..; surplus slots repeat the last group, which rewrites
  // identical bytes), so one vmcnt value tells each wave when its part of a chunk has landed; the
  // barrier that follows makes the whole chunk visible.
  const u32x4* g_src[LPW];
  int g_stride[LPW], g_off[LPW];
#pragma unroll
  for (int x = 0; x < LPW; ++x) {
    const int g = min(wave + W * x, G - 1);
    if (g < XA_G) {
      g_src[x] = p.XA[g / KH] + (g % KH) * 64 + lane;
      g_stride[x] = KH * 64;
    } else {
      g_src[x] = p.VP + (g - XA_G) * 64 + lane;
      g_stride[x] = V_U;
    }
    g_off[x] = g * 64;
  }
  // The loads are issued through inline assembly on purpose: the compiler's wait-count pass treats an
  // LDS-DMA load as aliasing every later LDS read and would drain all chunks in flight (vmcnt(0)) at
  // each barrier.  Here the ordering is explicit instead: s_waitcnt vmcnt(WAIT_N), then the barrier.
  const bool vy_lane = lane < 8;
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) void*)&lds[0][0];
  unsigned g_lds[LPW];
#pragma unroll
  for (int x = 0; x < LPW; ++x) g_lds[x] = __builtin_amdgcn_readfirstlane(lds_base + 16u * (unsigned)g_off[x]);
  const unsigned vy_lds = __builtin_amdgcn_readfirstlane(lds_base + 16u * (unsigned)(VY_OFF + 8 * wave));
  auto dma16 = [](const u32x4* src, unsigned lds_addr) {
    // m0 carries the LDS address of the load; it is declared clobbered, so the compiler keeps nothing in it
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(lds_addr) : "memory", "m0");
  };
  auto issue_chunk = [&](int ch_target) {
    const int ch = min(ch_target, c_end - 1);           // past the end: harmless reload of the last chunk
    const unsigned stage_off = (unsigned)((ch_target - c_begin) % NS) * (unsigned)(STAGE * 16);
#pragma unroll
    for (int x = 0; x < LPW; ++x) dma16(g_src[x] + (int64_t)ch * g_stride[x], __builtin_amdgcn_readfirstlane(g_lds[x] + stage_off));
    if (vy_lane) dma16(reinterpret_cast<const u32x4*>(p.VY + (int64_t)ch * 32) + lane, __builtin_amdgcn_readfirstlane(vy_lds + stage_off));
  };
  // vmcnt <= (DEPTH-1)*LPC: everything but the newest DEPTH-1 chunks has landed (loads retire in order)
  constexpr int WAIT_N = (DEPTH - 1) * LPC;

  // distance chain of one chunk: S[j][i] = XA_j . XB_i, with the pair (i, i) forced to r^2 = 0
  auto distance = [&](int ch, f32x16 (&S)[MI]) {
    const u32x4* s = lds[(ch - c_begin) % NS];
#pragma unroll
    for (int m = 0; m < MI; ++m)
#pragma unroll
      for (int r = 0; r < 16; ++r) S[m][r] = 0.0f;
#pragma unroll
    for (int kh = 0; kh < KH; ++kh) {
      f16x8 xa[XP];
#pragma unroll
      for (int pc = 0; pc < XP; ++pc) xa[pc] = as_f16x8(s[(pc * KH + kh) * 64 + lane]);
#pragma unroll
      for (int m = 0; m < MI; ++m) {
        // smallest terms first
        if constexpr (XP == 3) {
          S[m] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[1], xb[m][1][kh], S[m], 0, 0, 0);
          S[m] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[2], xb[m][0][kh], S[m], 0, 0, 0);
          S[m] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[0], xb[m][XP - 1][kh], S[m], 0, 0, 0);
        }
        S[m] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[1], xb[m][0][kh], S[m], 0, 0, 0);
        S[m] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[0], xb[m][1][kh], S[m], 0, 0, 0);
        S[m] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[0], xb[m][0][kh], S[m], 0, 0, 0);
      }
    }
#pragma unroll
    for (int m = 0; m < MI; ++m) {
      if (p.diag && ch == sub0 + m) {
        // one chunk in thousands: an opaque statement keeps this a real (wave-uniform) branch instead of
        // sixteen selects executed on every chunk
        asm volatile("" ::: "memory");
        const float s0 = KIND == GP_SE_ARD ? (float)PHI_SHIFT : 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (8 * (r >> 2) + 4 * h + (r & 3) == li) S[m][r] = s0;
      }
    }
  };

  // ---- main loop ---------------------------------------------------------------------------------
  // A chunk is worked through in NG = 2 MI groups of 8 values per lane (group g = (mh, m): the k-step
  // mh of sub-tile m).  Two software pipelines keep the matrix core and the VALU busy together:
  //   * the distance chain runs one chunk ahead (S of chunk ch + 1 while chunk ch is consumed);
  //   * the phi/split stage runs one group ahead of the contraction, and the two are emitted as
  //     bundles "one MFMA, then the VALU work of one value pair".  The matrix pipe accepts an MFMA only
  //     when it is free; a wave that reaches its next MFMA early stalls there with its VALU work
  //     undone, so MFMAs are spaced by at least their own duration of VALU instructions.
  constexpr int NG = 2 * MI;
  constexpr int MPG = 3 * NT;        // contraction MFMAs per group

  // phi and its split for values 2 e2, 2 e2 + 1 of group (mh, m); vy = the lane's y values for that mh
  auto phi_pair = [&](const f32x16& Sv, int mh, int e2, const f32x4 (&vy)[2], float& av, unsigned& oh, unsigned& ol) {
    float f[2];
#pragma unroll
    for (int z = 0; z < 2; ++z) {
      const int e = 2 * e2 + z;
      const float sv = Sv[8 * mh + e];
      if (KIND == GP_SE_ARD) {
        f[z] = __builtin_amdgcn_exp2f(sv);                 // sv = -log2(e)/2 r^2 + 15
      } else {
        // sv = 3 r^2; a rounding-level negative value is mirrored instead of clamped (|.| is a free
        // source modifier), the pair (i, i) was set to exactly 0 above
        const float u = __builtin_amdgcn_sqrtf(__builtin_fabsf(sv));
        const float ex = __builtin_amdgcn_exp2f(fmaf(u, -LOG2E, (float)PHI_SHIFT));
        f[z] = fmaf(u, ex, ex);
      }
      av = fmaf(f[z], vy[e >> 2][e & 3], av);
    }
    // hi = f truncated to fp16 (both values in one conversion), lo = f - hi taken straight from the
    // packed halves by the mixed-precision FMA, so the split costs two instructions per value
    oh = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(f[0], f[1]));
    ol = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(minus_half<0>(oh, f[0]), minus_half<1>(oh, f[1])));
  };
  auto load_vy = [&](const u32x4* s, int mh, f32x4 (&vy)[2]) {
#pragma unroll
    for (int g2 = 0; g2 < 2; ++g2) vy[g2] = __builtin_bit_cast(f32x4, s[VY_OFF + 8 * wave + 2 * (2 * mh + g2) + h]);
  };

  f32x16 S0[MI], S1[MI];             // S of the chunk being consumed / of the next chunk, roles alternate
  unsigned ph[4], pl[4];             // packed A operands of the group about to be contracted
  f32x4 vy0[2];                      // y values of k-step 0 of the chunk being consumed
  // fills the pipelines at the start of a segment: DEPTH chunks in flight, S and the first phi group of
  // the first chunk ready
  auto segment_prologue = [&]() {
#pragma unroll
    for (int d0 = 0; d0 < DEPTH; ++d0) issue_chunk(c_begin + d0);
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(WAIT_N) : "memory");
    __syncthreads();
    distance(c_begin, S0);
    load_vy(lds[0], 0, vy0);
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) phi_pair(S0[0], 0, e2, vy0, accv[0], ph[e2], pl[e2]);
  };

  // one chunk: S = its distances (ready), Sn = receives the next chunk's
  auto chunk_body = [&](int ch, f32x16 (&S)[MI], f32x16 (&Sn)[MI]) {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(WAIT_N - LPC) : "memory");
    __syncthreads();            // chunks <= ch + 1 are complete in LDS; every wave is done with chunk ch - 1
    issue_chunk(ch + DEPTH);    // refills the stage chunk ch - 1 occupied
    const u32x4* s = lds[(ch - c_begin) % NS];
    const u32x4* s_next = lds[(ch + 1 - c_begin) % NS];
    // every LDS operand of the chunk is fetched here, ahead of the distance chain, so that no MFMA or
    // VALU instruction further down waits on LDS latency
    f16x8 bh[2][NT], bl[2][NT];
#pragma unroll
    for (int mh = 0; mh < 2; ++mh)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        bh[mh][nt] = as_f16x8(s[V_OFF + ((mh * NT + nt) * 2 + 0) * 64 + lane]);
        bl[mh][nt] = as_f16x8(s[V_OFF + ((mh * NT + nt) * 2 + 1) * 64 + lane]);
      }
    f32x4 vy1[2], vy0n[2];
    load_vy(s, 1, vy1);
    load_vy(s_next, 0, vy0n);
    {   // past the last chunk the look-ahead group must not reach the y accumulator
      const float keep = ch + 1 < c_end ? 1.0f : 0.0f;
      vy0n[0] *= keep;
      vy0n[1] *= keep;
    }
    distance(ch + 1, Sn);       // past the last chunk this reads a harmless reload of it

#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int mh = g / MI, m = g % MI;
      // the group whose phi stage rides along: g + 1 of this chunk, or group 0 of the next chunk
      const bool wrap = g + 1 == NG;
      const int gn = wrap ? 0 : g + 1;
      const int mhn = gn / MI, mn = gn % MI;
      const f32x4 (&vyn)[2] = wrap ? vy0n : (mhn == 0 ? vy0 : vy1);
      const f16x8 ah = as_f16x8(u32x4{ph[0], ph[1], ph[2], ph[3]}), al = as_f16x8(u32x4{pl[0], pl[1], pl[2], pl[3]});
      unsigned nh[4], nl[4];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int k = 0; k < MPG; ++k) {
        const int nt = k / 3, term = k % 3;      // smallest terms first: lo*hi, hi*lo, hi*hi
        acc[m][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(term == 0 ? al : ah, term == 1 ? bl[mh][nt] : bh[mh][nt],
                                                            acc[m][nt], 0, 0, 0);
        // the 4 value pairs of the next group, spread over the MPG bundles
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2)
          if ((e2 * MPG) / 4 == k) phi_pair(wrap ? Sn[mn] : S[mn], mhn, e2, vyn, accv[mn], nh[e2], nl[e2]);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        ph[e2] = nh[e2];
        pl[e2] = nl[e2];
      }
    }
    vy0[0] = vy0n[0];
    vy0[1] = vy0n[1];
  };

  // Writes what the accumulators hold to OUT (first: stores, adds the noise term once; later: adds to
  // what is there) and clears them.  Undoes the power-of-two scalings and multiplies by a^2.
  float* out = p.OUT + (int64_t)js * p.split_stride;
  float oscale[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int c = min(li + 32 * nt, p.ncols - 1);
    oscale[nt] = p.a2 * ldexpf(1.0f, column_exponent(p.colmax[p.col0 + c]) - V_TOP - PHI_SHIFT);
  }
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
          if (i < p.n && c < p.ncols) {
            float v = oscale[nt] * acc[m][nt][r];
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
        if (h == 0 && i < p.n) {
          float v = p.a2 * ldexpf(1.0f, -PHI_SHIFT) * tot;
          if (noise) v = fmaf(p.sigma2, p.V[i * p.ldv + p.vcol], v);
          if (!first) v += out[i * p.ldo + p.vcol];
          out[i * p.ldo + p.vcol] = v;
        }
        accv[m] = 0.0f;
      }
    }
  };

  // Rounding error of an fp32 accumulator grows with the length of its chain of partial sums, so the
  // accumulators are added into OUT after every segment (the running sum then sees one addition per
  // segment).  The same threads read and write the same elements: no race, fixed order.
  bool first = true;
  for (;;) {
    segment_prologue();
    for (int ch = c_begin; ch < c_end; ch += 2) {
      chunk_body(ch, S0, S1);
      if (ch + 1 < c_end) chunk_body(ch + 1, S1, S0);
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

// ---- per-call operand preparation -------------------------------------------------------------
// colmax[c] = max_i |V_ic| as a bit pattern (non-negative floats order like unsigned ints)
// blockIdx.y = 1 does the same for a second matrix of the same shape.
__global__ __launch_bounds__(256) void colmax_kernel(const float* __restrict__ V, int64_t ldv,
                                                     const float* __restrict__ V2, int64_t ldv2, int64_t n, int t,
                                                     unsigned* __restrict__ colmax, unsigned* __restrict__ colmax2) {
  if (blockIdx.y) {
    V = V2;
    ldv = ldv2;
    colmax = colmax2;
  }
  // a thread keeps one column (per group of 256 columns) and walks rows: consecutive threads read
  // consecutive columns of a row, the running maximum stays in a register
  extern __shared__ unsigned smax[];   // [t]
  for (int c = threadIdx.x; c < t; c += 256) smax[c] = 0u;
  __syncthreads();
  const int64_t rows_per_block = (n + gridDim.x - 1) / gridDim.x;
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
  const int64_t r1 = min(n, r0 + rows_per_block);
  const int tw = t < 256 ? t : 256;        // columns handled side by side
  const int lanes = 256 / tw;              // rows handled side by side
  const int cl = threadIdx.x % tw, rl = threadIdx.x / tw;
  if (rl < lanes) {
    for (int c = cl; c < t; c += tw) {
      float m0 = 0.0f, m1 = 0.0f, m2 = 0.0f, m3 = 0.0f;
      int64_t i = r0 + rl;
      for (; i + 3 * lanes < r1; i += 4 * lanes) {
        m0 = fmaxf(m0, fabsf(V[i * ldv + c]));
        m1 = fmaxf(m1, fabsf(V[(i + lanes) * ldv + c]));
        m2 = fmaxf(m2, fabsf(V[(i + 2 * lanes) * ldv + c]));
        m3 = fmaxf(m3, fabsf(V[(i + 3 * lanes) * ldv + c]));
      }
      for (; i < r1; i += lanes) m0 = fmaxf(m0, fabsf(V[i * ldv + c]));
      m0 = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
      atomicMax(&smax[c], __float_as_uint(m0));
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < t; c += 256)
    if (smax[c]) atomicMax(&colmax[c], smax[c]);
}

// zeroes t words of one or two arrays (a kernel, not a memset command: memset nodes recorded into a
// captured graph have misbehaved on replay, and gp_kmv_static must be capturable)
__global__ __launch_bounds__(256) void clear_words_kernel(unsigned* __restrict__ a, unsigned* __restrict__ b, int t) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c < t) {
    a[c] = 0u;
    if (b) b[c] = 0u;
  }
}

// V' images of one column pass: unit u = ((chunk*2 + mh)*NT + nt)*2 + part, lane l: element e is
// V'[32 chunk + 16 mh + 8 (e/4) + 4 (l/32) + e%4][col0 + 32 nt + l%32]; rows >= n and columns past the pass are zero.
__global__ __launch_bounds__(256) void pack_v_kernel(const float* __restrict__ V, int64_t ldv, int64_t n, int nchunks,
                                                     int NT, int col0, int ncols, int vcol,
                                                     const unsigned* __restrict__ colmax, u32x4* __restrict__ VP,
                                                     float* __restrict__ VY) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = (int64_t)nchunks * 2 * NT * 64;
  if (gid < total) {
    const int lane = (int)(gid & 63);
    int64_t q = gid >> 6;
    const int nt = (int)(q % NT); q /= NT;
    const int mh = (int)(q & 1);
    const int64_t chunk = q >> 1;
    const int hh = lane >> 5;
    const int cc = 32 * nt + (lane & 31);
    const bool cok = cc < ncols;
    const int col = col0 + (cok ? cc : 0);
    const float scale = ldexpf(1.0f, V_TOP - column_exponent(colmax[col]));
    u32x4 hi, lo;
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      float fh[2], fl[2];
#pragma unroll
      for (int z = 0; z < 2; ++z) {
        const int e = 2 * e2 + z;
        const int64_t j = chunk * 32 + 16 * mh + 8 * (e >> 2) + 4 * hh + (e & 3);
        const float v = (cok && j < n) ? V[j * ldv + col] * scale : 0.0f;
        fh[z] = __uint_as_float(__float_as_uint(v) & HI_MASK);
        fl[z] = v - fh[z];
      }
      hi[e2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(fh[0], fh[1]));
      lo[e2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(fl[0], fl[1]));
    }
    u32x4* dst = VP + ((chunk * 2 + mh) * NT + nt) * 2 * 64;
    dst[lane] = hi;
    dst[64 + lane] = lo;
  }
  // the VALU column, unscaled
  const int64_t npad = (int64_t)nchunks * 32;
  if (gid < npad) VY[gid] = (vcol >= 0 && gid < n) ? V[gid * ldv + vcol] : 0.0f;
}

__global__ void kmv_reduce_f16_kernel(const float* __restrict__ part, int64_t split_stride, int JS, int64_t n, int t,
                                      float* __restrict__ out, int64_t ldo) {
  const int64_t total = n * t;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int64_t i = e / t;
    const int c = (int)(e - i * t);
    float s = 0.0f;
    for (int k = 0; k < JS; ++k) s += part[(int64_t)k * split_stride + e];
    out[i * ldo + c] = s;
  }
}

typedef void (*tileh_fn)(TileArgsH);

template <int KIND, int KH, int XP>
tileh_fn pick_h_nt_mi(int NT, int MI, int W) {
  if constexpr (KH <= 2) {
    if (MI == 2 && W == 8) return NT == 1 ? kmv_tile_f16_kernel<KIND, KH, XP, 1, 2, 8> : kmv_tile_f16_kernel<KIND, KH, XP, 2, 2, 8>;
    if (MI == 2) return NT == 1 ? kmv_tile_f16_kernel<KIND, KH, XP, 1, 2, 4> : kmv_tile_f16_kernel<KIND, KH, XP, 2, 2, 4>;
  }
  if (W == 8) return NT == 1 ? kmv_tile_f16_kernel<KIND, KH, XP, 1, 1, 8> : kmv_tile_f16_kernel<KIND, KH, XP, 2, 1, 8>;
  return NT == 1 ? kmv_tile_f16_kernel<KIND, KH, XP, 1, 1, 4> : kmv_tile_f16_kernel<KIND, KH, XP, 2, 1, 4>;
}

template <int KIND, int XP>
tileh_fn pick_h_kh(int KH, int NT, int MI, int W) {
  switch (KH) {
    case 1: return pick_h_nt_mi<KIND, 1, XP>(NT, MI, W);
    case 2: return pick_h_nt_mi<KIND, 2, XP>(NT, MI, W);
    case 3: return pick_h_nt_mi<KIND, 3, XP>(NT, MI, W);
    case 4: return pick_h_nt_mi<KIND, 4, XP>(NT, MI, W);
    case 6: return pick_h_nt_mi<KIND, 6, XP>(NT, MI, W);
    case 8: return pick_h_nt_mi<KIND, 8, XP>(NT, MI, W);
  }
  return nullptr;
}

tileh_fn pick_h(int kind, int KH, int XP, int NT, int MI, int W) {
  if (kind == GP_SE_ARD) return XP == 2 ? pick_h_kh<GP_SE_ARD, 2>(KH, NT, MI, W) : pick_h_kh<GP_SE_ARD, 3>(KH, NT, MI, W);
  return XP == 2 ? pick_h_kh<GP_MATERN32_ARD, 2>(KH, NT, MI, W) : pick_h_kh<GP_MATERN32_ARD, 3>(KH, NT, MI, W);
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct ScratchH {
  size_t off_colmax, off_vy, off_vp, off_part, total;
};

ScratchH scratch_layout(const gp_ctx* ctx, int t, int JS, int64_t rows) {
  ScratchH L;
  const int64_t nchunks = (ctx->n + 31) / 32;
  size_t o = 0;
  L.off_colmax = o; o += align_up((size_t)t * sizeof(unsigned), 256);
  L.off_vy = o; o += align_up((size_t)nchunks * 32 * sizeof(float), 256);
  L.off_vp = o; o += align_up((size_t)nchunks * 2 * 2 * 2 * 64 * 16, 256);      // NT = 2 images
  L.off_part = o;
  if (JS > 1) o += align_up((size_t)JS * rows * t * sizeof(float), 256);
  L.total = o;
  return L;
}

}  // namespace

int gp_kh_bucket(int d, int kernel) {
  // components: d coordinates, squared norm, one, and for SE the slot that carries the 2^15 shift
  const int comps = d + 2 + (kernel == GP_SE_ARD ? 1 : 0);
  const int need = (comps + 15) / 16;
  const int buckets[] = {1, 2, 3, 4, 6, 8};
  for (int b : buckets)
    if (need <= b) return b;
  return -1;
}

KmvPlan gp_plan_kmv_f16(const gp_ctx* ctx, int64_t rows, int64_t col_chunks) {
  KmvPlan pl;
  const int64_t chunks = col_chunks > 0 ? col_chunks : (ctx->n + 31) / 32;
  // two sub-tiles per wave halve the LDS operand traffic; past one k-step of distance operands the
  // second sub-tile no longer fits the register file without spills
  pl.MI = (ctx->KH == 1 && rows >= 8192) ? 2 : 1;
  if (ctx->mi_forced) pl.MI = (ctx->mi_forced == 2 && ctx->KH <= 2) ? 2 : 1;   // tuning aid
  pl.W = 4;   // 8-wave workgroups halve the L2-to-LDS traffic but measured no faster on MI355X
  if (ctx->w_forced) pl.W = ctx->w_forced;                                      // tuning aid
  const int rows_per_wg = 32 * pl.W * pl.MI;
  pl.row_blocks = (int)((rows + rows_per_wg - 1) / rows_per_wg);
  const int target = 2 * ctx->num_cu;
  int JS = 1;
  if (pl.row_blocks < target) {
    JS = (target + pl.row_blocks - 1) / pl.row_blocks;
    const int64_t max_js = chunks / 4 > 0 ? chunks / 4 : 1;
    if (JS > max_js) JS = (int)max_js;
    if (JS > 64) JS = 64;
  }
  pl.cps = (int)((chunks + JS - 1) / JS);
  pl.JS = (int)((chunks + pl.cps - 1) / pl.cps);
  return pl;
}

int gp_launch_colmax(gp_ctx* ctx, const float* dV, int64_t ldv, int t, unsigned* cm, const float* dV2, int64_t ldv2,
                     unsigned* cm2, bool cleared) {
  if (!cleared) {
    hipLaunchKernelGGL(clear_words_kernel, dim3((t + 255) / 256), dim3(256), 0, ctx->stream, cm, dV2 ? cm2 : nullptr, t);
    GP_HIP(ctx, hipGetLastError());
  }
  // few workgroups: every one ends with t atomic maxima on the same t words
  int blocks = (int)((ctx->n * (int64_t)t + 8191) / 8192);
  if (blocks > 2 * ctx->num_cu) blocks = 2 * ctx->num_cu;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(colmax_kernel, dim3(blocks, dV2 ? 2 : 1), dim3(256), (size_t)t * sizeof(unsigned), ctx->stream, dV,
                     ldv, dV2, ldv2, ctx->n, t, cm, cm2);
  GP_HIP(ctx, hipGetLastError());
  return GP_OK;
}

size_t gp_kmv_f16_scratch_bytes(const gp_ctx* ctx, int t, int64_t rows, int64_t col_chunks) {
  return scratch_layout(ctx, t, gp_plan_kmv_f16(ctx, rows, col_chunks).JS, rows).total;
}

int gp_kmv_launch_f16(gp_ctx* ctx, const float* dV, int64_t ldv, int t, float* dOut, int64_t ldo, int add_noise,
                      void* scratch, size_t scratch_bytes, const unsigned* colmax_ready, const KmvRows* rows,
                      KmvDeferred* defer, const KmvWindow* win) {
  const int64_t nrows = rows ? rows->m : ctx->n;
  const int XP = rows ? (rows->path == GP_PATH_F16X3 ? 3 : 2) : ctx->XP;
  const KmvPlan pl = gp_plan_kmv_f16(ctx, nrows, win ? win->nchunks : 0);
  const ScratchH L = scratch_layout(ctx, t, pl.JS, nrows);
  if (scratch_bytes < L.total || !scratch)
    return gp_fail(ctx, GP_ERR_WORKSPACE, "gp_kmv: scratch %zu < %zu bytes", scratch_bytes, L.total);
  hipStream_t st = ctx->stream;
  char* w = (char*)scratch;
  const unsigned* colmax = colmax_ready ? colmax_ready : (const unsigned*)(w + L.off_colmax);
  float* VY = (float*)(w + L.off_vy);
  u32x4* VP = (u32x4*)(w + L.off_vp);
  float* part = (float*)(w + L.off_part);
  const bool split = pl.JS > 1;
  // a column window is handed to the kernels as a point set of its own that starts at chunk 0
  const int nchunks = win ? win->nchunks : (int)((ctx->n + 31) / 32);
  const int64_t first = win ? (int64_t)win->chunk0 * 32 : 0;
  const int64_t ncontr = win ? ((first + (int64_t)nchunks * 32 < ctx->n ? first + (int64_t)nchunks * 32 : ctx->n) - first) : ctx->n;
  if (win && !colmax_ready) return gp_fail(ctx, GP_ERR_ARG, "gp_kmv: a column window needs the column maxima");
  const float* dVw = dV + first * ldv;

  if (!colmax_ready) {
    const int rc = gp_launch_colmax(ctx, dV, ldv, t, (unsigned*)(w + L.off_colmax));
    if (rc < 0) return rc;
  }

  TileArgsH a;
  for (int pc = 0; pc < 3; ++pc) {
    a.XA[pc] = (const u32x4*)ctx->dXAh[pc] + (win ? (int64_t)win->chunk0 * ctx->KH * 64 : 0);
    a.XB[pc] = (const u32x4*)(rows ? rows->XBh[pc] : ctx->dXBh[pc]);
  }
  a.VP = VP;
  a.VY = VY;
  a.V = dV;
  a.ldv = ldv;
  a.colmax = colmax;
  a.OUT = split ? part : dOut;
  a.ldo = split ? t : ldo;
  a.split_stride = split ? nrows * (int64_t)t : 0;
  a.n = nrows;
  a.diag = (rows || win) ? 0 : 1;
  a.nchunks = nchunks;
  a.JS = pl.JS;
  a.cps = pl.cps;
  a.a2 = (float)(ctx->a * ctx->a);
  a.sigma2 = (float)(ctx->sigma * ctx->sigma);
  a.add_noise = add_noise;

  int vcol = (t > 1 && t % 32 == 1) ? 0 : -1;
  int c = vcol >= 0 ? 1 : 0;
  const dim3 grid(pl.row_blocks * pl.JS), block(64 * pl.W);
  while (c < t) {
    const int rem = t - c;
    const int NT = rem > 32 ? 2 : 1;
    a.col0 = c;
    a.ncols = rem < 32 * NT ? rem : 32 * NT;
    a.vcol = vcol;
    {
      const int64_t threads = (int64_t)nchunks * 2 * NT * 64;
      const int64_t need = threads > (int64_t)nchunks * 32 ? threads : (int64_t)nchunks * 32;
      hipLaunchKernelGGL(pack_v_kernel, dim3((unsigned)((need + 255) / 256)), dim3(256), 0, st, dVw, ldv, ncontr, nchunks, NT,
                         a.col0, a.ncols, vcol, (const unsigned*)colmax, VP, VY);
      GP_HIP(ctx, hipGetLastError());
    }
    vcol = -1;
    tileh_fn fn = pick_h(ctx->kernel, ctx->KH, XP, NT, pl.MI, pl.W);
    if (!fn) return gp_fail(ctx, GP_ERR_ARG, "gp_kmv: no fp16 kernel for KH=%d", ctx->KH);
    const bool prof = gp_prof_begin(ctx, GP_PROF_TILE);
    hipLaunchKernelGGL(fn, grid, block, 0, st, a);
    GP_HIP(ctx, hipGetLastError());
    gp_prof_end(ctx, prof);
    c += a.ncols;
  }
  if (defer) {
    defer->part = part;
    defer->stride = a.split_stride;
    defer->JS = pl.JS;
  }
  if (split && !defer) {
    const int64_t total = nrows * (int64_t)t;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 4 * ctx->num_cu) blocks = 4 * ctx->num_cu;
    hipLaunchKernelGGL(kmv_reduce_f16_kernel, dim3(blocks), dim3(256), 0, st, (const float*)part, a.split_stride, pl.JS,
                       nrows, t, dOut, ldo);
    GP_HIP(ctx, hipGetLastError());
  }
  return GP_OK;
}
