// In-LDS complex FFT of 2^LOGQ points (256 .. 8192) for one workgroup of 512 threads: radix-16
// register passes (two radix-4 stages per LDS round trip), twiddles from an octant table in LDS,
// data padded by one element per 32.  Shared by the decode-attention softmax kernel (inverse, then
// forward transform) and the FFT prefill (forward transform).
#pragma once
#include "common.h"

namespace iwdft {

constexpr int kFftThreads = 512;
constexpr int kFftNBT = 8;   // most kept bins per thread                (|B| <= 4096)
constexpr int kFftEPT = 16;  // time samples per thread                  (Q   <= 8192)
constexpr int kFftMaxLogQ = 13;

__device__ __forceinline__ float2 mul_i(float2 a) { return make_float2(-a.y, a.x); }    // * (+j)
__device__ __forceinline__ float2 mul_mi(float2 a) { return make_float2(a.y, -a.x); }   // * (-j)
__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }
__device__ __forceinline__ float2 conjf2(float2 a) { return make_float2(a.x, -a.y); }

// exp(+j 2 pi p / M) through the hardware sine / cosine (argument in revolutions, exact for the
// power-of-two M this path requires; ~1e-6 absolute error, used only for the block twiddles of the
// score synthesis where 1e-6 of a score is far below the output tolerance).
__device__ __forceinline__ float2 cis_fast(uint32_t p, uint32_t M) {
  const float f = (float)p * rcp_pow2(M);
  return make_float2(__builtin_amdgcn_cosf(f), __builtin_amdgcn_sinf(f));
}

// LDS index of logical sample i: one float2 of padding after every 32 keeps the strided
// accesses of the late passes spread over all banks.
__device__ __forceinline__ int pad(int i) { return i + (i >> 5); }
__host__ __device__ constexpr int fft_lds_float2(int logQ) {
  return (1 << logQ) + (1 << logQ) / 32 + ((1 << logQ) / 8 + 1);
}

// tab[m] = exp(+j 2 pi m / Q) for m = 0 .. Q/8; any m in [0, Q/4] by reflection about pi/4.
__device__ __forceinline__ float2 tw_get(const float2* tab, int m, int q8) {
  if (m <= q8) return tab[m];
  const float2 t = tab[2 * q8 - m];
  return make_float2(t.y, t.x);
}

// Radix-4 butterfly of the inverse (sign +) decimation-in-frequency transform: combine, then
// multiply output m by w^m.
__device__ __forceinline__ void r4_dif(float2& a0, float2& a1, float2& a2, float2& a3, float2 w1) {
  const float2 w2 = cmul(w1, w1), w3 = cmul(w2, w1);
  const float2 t0 = cadd(a0, a2), t1 = csub(a0, a2), t2 = cadd(a1, a3), t3 = mul_i(csub(a1, a3));
  a0 = cadd(t0, t2);
  a1 = cmul(cadd(t1, t3), w1);
  a2 = cmul(csub(t0, t2), w2);
  a3 = cmul(csub(t1, t3), w3);
}
// Its transpose with conjugated constants (forward, decimation in time): multiply input m by
// conj(w)^m, then combine.  w1c is already conjugated.
__device__ __forceinline__ void r4_dit(float2& a0, float2& a1, float2& a2, float2& a3, float2 w1c) {
  const float2 w2 = cmul(w1c, w1c), w3 = cmul(w2, w1c);
  a1 = cmul(a1, w1c);
  a2 = cmul(a2, w2);
  a3 = cmul(a3, w3);
  const float2 t0 = cadd(a0, a2), t1 = csub(a0, a2), t2 = cadd(a1, a3), t3 = mul_mi(csub(a1, a3));
  a0 = cadd(t0, t2);
  a1 = cadd(t1, t3);
  a2 = csub(t0, t2);
  a3 = csub(t1, t3);
}

// Thread -> butterfly assignment of a pass whose innermost index j has LS bits: for LS < 4 the j
// bits are taken from lane bits 4.. so that 16 consecutive lanes (one LDS access phase) touch 16
// different butterfly groups, whose padded addresses fall into distinct banks.
template <int LS>
__device__ __forceinline__ int butterfly_of(int t) {
  if constexpr (LS >= 4 || LS == 0) return t;
  else return ((t >> (4 + LS)) << (4 + LS)) | ((t & 15) << LS) | ((t >> 4) & ((1 << LS) - 1));
}

// Two consecutive radix-4 stages (spans 4*s2 and s2) on the 16 samples p0 + m*s2 held in
// registers: one LDS round trip instead of two.  INV: inverse DIF order (wide span first);
// otherwise the forward DIT order (narrow span first, conjugated twiddles).
template <int LOGQ, int LS2, bool INV>
__device__ __forceinline__ void fft_pass16(float2* buf, const float2* tab, int tid) {
  constexpr int Q = 1 << LOGQ, s2 = 1 << LS2, NB = Q / 16;
  constexpr int sh1 = LOGQ - LS2 - 4;
#pragma unroll
  for (int it = 0; it < (NB + kFftThreads - 1) / kFftThreads; ++it) {
    const int t = it * kFftThreads + tid;
    if (NB % kFftThreads == 0 || t < NB) {
      const int bf = butterfly_of<LS2>(t);
      const int j = bf & (s2 - 1);
      float2* base = buf + pad(((bf >> LS2) << (LS2 + 4)) + j);
      float2 x[16];
#pragma unroll
      for (int m = 0; m < 16; ++m) x[m] = base[m * s2 + ((m * s2) >> 5)];
      // Twiddles of the pass from one table entry t = exp(+j 2 pi j / (16 s2)) (index < Q/16: inside the
      // octant table as it stands): group b of the wide stage uses t * exp(+j 2 pi b / 16), the narrow stage
      // t^4.
      const float2 t1 = tab[j << sh1];
      const float2 t2 = cmul(t1, t1);
      const float2 t4 = cmul(t2, t2);
      const float2 c1 = make_float2(0.92387953251128674f, 0.38268343236508977f);  // exp(j pi / 8)
      const float2 c2 = make_float2(0.70710678118654752f, 0.70710678118654752f);  // exp(j pi / 4)
      const float2 c3 = make_float2(0.38268343236508977f, 0.92387953251128674f);  // exp(j 3 pi / 8)
      if constexpr (INV) {
        r4_dif(x[0], x[4], x[8], x[12], t1);
        r4_dif(x[1], x[5], x[9], x[13], cmul(t1, c1));
        r4_dif(x[2], x[6], x[10], x[14], cmul(t1, c2));
        r4_dif(x[3], x[7], x[11], x[15], cmul(t1, c3));
#pragma unroll
        for (int a = 0; a < 4; ++a) r4_dif(x[4 * a], x[4 * a + 1], x[4 * a + 2], x[4 * a + 3], t4);
      } else {
        const float2 w = conjf2(t4);
#pragma unroll
        for (int a = 0; a < 4; ++a) r4_dit(x[4 * a], x[4 * a + 1], x[4 * a + 2], x[4 * a + 3], w);
        r4_dit(x[0], x[4], x[8], x[12], conjf2(t1));
        r4_dit(x[1], x[5], x[9], x[13], conjf2(cmul(t1, c1)));
        r4_dit(x[2], x[6], x[10], x[14], conjf2(cmul(t1, c2)));
        r4_dit(x[3], x[7], x[11], x[15], conjf2(cmul(t1, c3)));
      }
#pragma unroll
      for (int m = 0; m < 16; ++m) base[m * s2 + ((m * s2) >> 5)] = x[m];
    }
  }
  __syncthreads();
}

// One radix-4 stage of span 1 << LS.
template <int LOGQ, int LS, bool INV>
__device__ __forceinline__ void fft_pass4(float2* buf, const float2* tab, int tid) {
  constexpr int Q = 1 << LOGQ, q8 = Q >> 3, s = 1 << LS, NB = Q / 4;
#pragma unroll
  for (int it = 0; it < (NB + kFftThreads - 1) / kFftThreads; ++it) {
    const int t = it * kFftThreads + tid;
    if (NB % kFftThreads == 0 || t < NB) {
      const int bf = butterfly_of<LS>(t);
      const int j = bf & (s - 1);
      float2* base = buf + pad(((bf >> LS) << (LS + 2)) + j);
      const float2 w = tw_get(tab, j << (LOGQ - LS - 2), q8);
      float2 a0 = base[0], a1 = base[s + (s >> 5)], a2 = base[2 * s + ((2 * s) >> 5)],
             a3 = base[3 * s + ((3 * s) >> 5)];
      if constexpr (INV) r4_dif(a0, a1, a2, a3, w);
      else r4_dit(a0, a1, a2, a3, conjf2(w));
      base[0] = a0;
      base[s + (s >> 5)] = a1;
      base[2 * s + ((2 * s) >> 5)] = a2;
      base[3 * s + ((3 * s) >> 5)] = a3;
    }
  }
  __syncthreads();
}

// Stage plan for Q = 2^LOGQ: n4 = LOGQ/2 radix-4 stages with spans Q/4, Q/16, ..., taken two at a
// time (one single stage if n4 is odd), then one radix-2 stage of span 1 if LOGQ is odd.  The
// radix-2 stage is not run here: the caller applies it to the sample pairs it holds in registers.
// Inverse: natural order in, digit-reversed order out.
template <int LOGQ, int P = 0>
__device__ __forceinline__ void ifft_dif(float2* buf, const float2* tab, int tid) {
  constexpr int n4 = LOGQ >> 1;
  if constexpr (P < (n4 >> 1)) {
    fft_pass16<LOGQ, LOGQ - 4 * (P + 1), true>(buf, tab, tid);
    ifft_dif<LOGQ, P + 1>(buf, tab, tid);
  } else if constexpr (n4 & 1) {
    fft_pass4<LOGQ, (LOGQ & 1), true>(buf, tab, tid);
  }
}
// Forward: the transpose of the above with conjugated constants; takes the digit-reversed order the
// inverse produces (after the caller's radix-2 stage) and returns natural order.
template <int LOGQ, int P = ((LOGQ >> 1) >> 1)>
__device__ __forceinline__ void fft_dit(float2* buf, const float2* tab, int tid) {
  constexpr int n4 = LOGQ >> 1;
  if constexpr (P == (n4 >> 1) && (n4 & 1)) fft_pass4<LOGQ, (LOGQ & 1), false>(buf, tab, tid);
  if constexpr (P > 0) {
    fft_pass16<LOGQ, LOGQ - 4 * P, false>(buf, tab, tid);
    fft_dit<LOGQ, P - 1>(buf, tab, tid);
  }
}

// LDS position, in the digit-reversed order that fft_dit consumes and ifft_dif produces, of sample a (for
// odd LOGQ: a < Q/2; its partner a + Q/2 sits right behind it and the pair still needs / has had the
// radix-2 stage applied by the caller).
template <int LOGQ>
__device__ __forceinline__ int digit_pos(int a) {
  int p = 0;
#pragma unroll
  for (int t = 0; t < (LOGQ >> 1); ++t) p |= ((a >> (2 * t)) & 3) << (LOGQ - 2 * t - 2);
  return p;
}

// Two adjacent channels of one token row as a complex number (load), and back (store, bf16 rounded to
// nearest even).
template <bool BF16>
__device__ __forceinline__ float2 load_pair(const char* row) {
  if constexpr (BF16) {
    const uint32_t u = *(const uint32_t*)row;
    return make_float2(__uint_as_float(u << 16), __uint_as_float(u & 0xffff0000u));
  } else {
    return *(const float2*)row;
  }
}
template <bool BF16>
__device__ __forceinline__ void store_pair(char* row, float2 v) {
  if constexpr (BF16) *(uint32_t*)row = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
  else *(float2*)row = v;
}

}  // namespace iwdft
