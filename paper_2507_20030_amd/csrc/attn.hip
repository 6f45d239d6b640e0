// Decode attention over the reconstructed segment (Sec. 3.1.1 Eq. kv-attn over the middle part
// of Sec. 4.2.2 Eq. kv-concat) without ever writing K~ or V~ (Eq. reconstruct-idft) to memory.
//
// For one slice and one query head, with F the stored coefficients and gain folded in:
//   scores  s[a] = scale * q . K~[a]        = Re sum_k Y[k] e^{+j 2 pi k a / M},
//                                             Y[k] = (w_k scale / M) * sum_c q[c] F_K[c][k]
//   weights p[a] = exp(s[a] - max) ,  Z = sum_a p[a]
//   output  o[c] = sum_a p[a] V~[a][c] / Z  = Re sum_k F_V[c][k] * Pn[k],
//                                             Pn[k] = (w_k / (M Z)) * conj( sum_a p[a] e^{-j 2 pi k a / M} )
// The common slot shift (T-M) of the fixed-frame storage moves K~ and V~ together and drops out
// of softmax attention.  Three kernels:
//   A  attn_qc_kernel   streams F_K once, produces qc[k] = sum_c q[c] F_K[c][k]    (HBM-bound)
//   B  attn_fft_kernel  per (slice, pair of query heads): sparse spectrum -> M scores by
//                       inverse FFT in LDS, softmax, forward FFT, gather the kept bins -> Pn
//      attn_direct_kernel  same result by direct O(M |B|) sums (any M; reference path)
//   C  attn_out_kernel  streams F_V once, o[c] = Re sum_k F_V[c][k] Pn[k]           (HBM-bound)
#include "common.h"

namespace iwdft {

typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// ------------------------------------------------------------------------------------------ A
constexpr int kQcThreads = 256;
constexpr int kQcBins = kQcThreads * 2;

// grid: (slice * chunks + chunk) * passes + pass.  Lane = two adjacent bins, loop over channels.
template <bool BF16, int GT>
__global__ __launch_bounds__(kQcThreads) void attn_qc_kernel(Params P, const void* __restrict__ q,
                                                            float2* __restrict__ qc, int chunks, int passes) {
  __shared__ float qs[GT][kHeadDim];
  uint32_t bid = blockIdx.x;
  const int pass = bid % passes;
  bid /= passes;
  const int chunk = bid % chunks;
  const int slice = bid / chunks;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const int g0 = pass * GT;
  for (int e = threadIdx.x; e < GT * kHeadDim; e += kQcThreads) {
    const int g = g0 + e / kHeadDim;
    qs[e / kHeadDim][e % kHeadDim] =
        (g < P.G) ? load_kv<BF16>(q, ((int64_t)slice * P.G + g) * kHeadDim + (e % kHeadDim)) : 0.f;
  }
  __syncthreads();
  const int i0 = chunk * kQcBins + threadIdx.x * 2;
  if (i0 >= L.Bp) return;
  const v4f* row = (const v4f*)(P.FK + L.coef_off + (int64_t)s * kHeadDim * L.Bp + i0);
  const int64_t stride = L.Bp / 2;
  v4f acc[GT];
#pragma unroll
  for (int g = 0; g < GT; ++g) acc[g] = (v4f)(0.f);
  constexpr int U = 8;
#pragma unroll 1
  for (int d = 0; d < kHeadDim; d += U) {
    v4f f[U];
#pragma unroll
    for (int u = 0; u < U; ++u) f[u] = __builtin_nontemporal_load(row + (d + u) * stride);
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int g = 0; g < GT; ++g) acc[g] += qs[g][d + u] * f[u];
  }
#pragma unroll
  for (int g = 0; g < GT; ++g)
    if (g0 + g < P.G)
      *(v4f*)(qc + L.ws_off + ((int64_t)s * P.G + g0 + g) * L.Bp + i0) = acc[g];
}

// ------------------------------------------------------------------------------------------ C
constexpr int kOutThreads = 256;
constexpr int kOutDC = 16;  // channels per block

// Sum V values per lane over the whole wave; on return lane L holds the total of value
// L >> (6 - log2 V)  (V <= 64, power of two).  Each step halves the number of live values.
template <int CNT, int OFF, int V>
__device__ __forceinline__ void wave_reduce_step(float (&v)[V], int lane) {
  if constexpr (OFF >= 1) {
    if constexpr (CNT > 1) {
      constexpr int half = CNT / 2;
      const bool upper = (lane & OFF) != 0;
#pragma unroll
      for (int i = 0; i < half; ++i) {
        const float send = upper ? v[i] : v[i + half];
        const float keep = upper ? v[i + half] : v[i];
        v[i] = keep + __shfl_xor(send, OFF);
      }
      wave_reduce_step<half, OFF / 2, V>(v, lane);
    } else {
      v[0] += __shfl_xor(v[0], OFF);
      wave_reduce_step<1, OFF / 2, V>(v, lane);
    }
  }
}
template <int V>
__device__ __forceinline__ float wave_reduce_scatter(float (&v)[V], int lane) {
  wave_reduce_step<V, 32, V>(v, lane);
  return v[0];
}

// grid: (slice * 8 + dchunk) * passes + pass.  Lane = two adjacent bins; a block walks all bins
// of its slice for 16 channels, so no cross-block reduction is needed.
template <bool BF16, int GT>
__global__ __launch_bounds__(kOutThreads) void attn_out_kernel(Params P, const float2* __restrict__ Pn,
                                                              void* __restrict__ out, int passes) {
  constexpr int V = kOutDC * GT;
  constexpr int VR = V > 64 ? 64 : V;  // values per reduction round
  __shared__ float red[kOutThreads / 64][V];
  uint32_t bid = blockIdx.x;
  const int pass = bid % passes;
  bid /= passes;
  const int dc = bid % (kHeadDim / kOutDC);
  const int slice = bid / (kHeadDim / kOutDC);
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const int g0 = pass * GT;
  const int d0 = dc * kOutDC;
  const int64_t stride = L.Bp / 2;
  const v4f* Fv = (const v4f*)(P.FV + L.coef_off + ((int64_t)s * kHeadDim + d0) * L.Bp);
  const float2* Prow = Pn + L.ws_off + ((int64_t)s * P.G + g0) * L.Bp;

  float acc[V];
#pragma unroll
  for (int v = 0; v < V; ++v) acc[v] = 0.f;

  for (int i0 = threadIdx.x * 2; i0 < L.Bp; i0 += kOutThreads * 2) {
    v4f p[GT];
#pragma unroll
    for (int g = 0; g < GT; ++g)
      p[g] = (g0 + g < P.G) ? *(const v4f*)(Prow + (int64_t)g * L.Bp + i0) : (v4f)(0.f);
    v4f f[kOutDC];
#pragma unroll
    for (int dd = 0; dd < kOutDC; ++dd) f[dd] = __builtin_nontemporal_load(Fv + dd * stride + i0 / 2);
#pragma unroll
    for (int dd = 0; dd < kOutDC; ++dd)
#pragma unroll
      for (int g = 0; g < GT; ++g)
        acc[dd * GT + g] += f[dd].x * p[g].x - f[dd].y * p[g].y + f[dd].z * p[g].z - f[dd].w * p[g].w;
  }

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int r = 0; r < V / VR; ++r) {
    float part[VR];
#pragma unroll
    for (int v = 0; v < VR; ++v) part[v] = acc[r * VR + v];
    const float tot = wave_reduce_scatter<VR>(part, lane);
    constexpr int rep = 64 / VR;  // lanes holding the same value
    if ((lane % rep) == 0) red[wave][r * VR + lane / rep] = tot;
  }
  __syncthreads();
  for (int v = threadIdx.x; v < V; v += kOutThreads) {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < kOutThreads / 64; ++w) tot += red[w][v];
    const int dd = v / GT, g = v % GT;
    if (g0 + g < P.G) store_kv<BF16>(out, ((int64_t)slice * P.G + g0 + g) * kHeadDim + d0 + dd, tot);
  }
}

// ------------------------------------------------------------------------------------- B (FFT)
constexpr int kFftThreads = 512;
constexpr int kFftNBT = 8;   // kept bins per thread held in registers  (|B| <= 4096)
constexpr int kFftEPT = 16;  // time samples per thread                  (Q   <= 8192)
constexpr int kFftMaxLogQ = 13;

__device__ __forceinline__ float2 mul_i(float2 a) { return make_float2(-a.y, a.x); }    // * (+j)
__device__ __forceinline__ float2 mul_mi(float2 a) { return make_float2(a.y, -a.x); }   // * (-j)
__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }
__device__ __forceinline__ float2 conjf2(float2 a) { return make_float2(a.x, -a.y); }

// In-place inverse (sign +) decimation-in-frequency transform, natural order in, digit-reversed
// order out.  Radix-4 stages with spans Q/4, Q/16, ...; one final radix-2 stage when log2 Q is odd.
__device__ void ifft_dif(float2* buf, int logQ, int tid) {
  const int Q = 1 << logQ;
  int ls = logQ;  // log2 of the current span
  for (int st = 0; st < logQ / 2; ++st) {
    ls -= 2;
    const int s = 1 << ls;
    for (int bf = tid; bf < Q / 4; bf += kFftThreads) {
      const int j = bf & (s - 1);
      const int p0 = ((bf >> ls) << (ls + 2)) + j;
      const float2 a0 = buf[p0], a1 = buf[p0 + s], a2 = buf[p0 + 2 * s], a3 = buf[p0 + 3 * s];
      const float2 t0 = cadd(a0, a2), t1 = csub(a0, a2), t2 = cadd(a1, a3), t3 = mul_i(csub(a1, a3));
      const float2 w1 = cis((uint32_t)j, (uint32_t)(4 * s));
      const float2 w2 = cmul(w1, w1), w3 = cmul(w2, w1);
      buf[p0] = cadd(t0, t2);
      buf[p0 + s] = cmul(cadd(t1, t3), w1);
      buf[p0 + 2 * s] = cmul(csub(t0, t2), w2);
      buf[p0 + 3 * s] = cmul(csub(t1, t3), w3);
    }
    __syncthreads();
  }
  if (logQ & 1) {
    for (int bf = tid; bf < Q / 2; bf += kFftThreads) {
      const float2 a = buf[2 * bf], b = buf[2 * bf + 1];
      buf[2 * bf] = cadd(a, b);
      buf[2 * bf + 1] = csub(a, b);
    }
    __syncthreads();
  }
}

// The transpose of ifft_dif with conjugated constants: forward (sign -) transform that takes the
// digit-reversed order ifft_dif produces and returns natural order.
__device__ void fft_dit(float2* buf, int logQ, int tid) {
  const int Q = 1 << logQ;
  if (logQ & 1) {
    for (int bf = tid; bf < Q / 2; bf += kFftThreads) {
      const float2 a = buf[2 * bf], b = buf[2 * bf + 1];
      buf[2 * bf] = cadd(a, b);
      buf[2 * bf + 1] = csub(a, b);
    }
    __syncthreads();
  }
  int ls = (logQ & 1) - 2;
  for (int st = 0; st < logQ / 2; ++st) {
    ls += 2;
    const int s = 1 << ls;
    for (int bf = tid; bf < Q / 4; bf += kFftThreads) {
      const int j = bf & (s - 1);
      const int p0 = ((bf >> ls) << (ls + 2)) + j;
      const float2 w1 = conjf2(cis((uint32_t)j, (uint32_t)(4 * s)));
      const float2 w2 = cmul(w1, w1), w3 = cmul(w2, w1);
      const float2 a0 = buf[p0], a1 = cmul(buf[p0 + s], w1), a2 = cmul(buf[p0 + 2 * s], w2),
                   a3 = cmul(buf[p0 + 3 * s], w3);
      const float2 t0 = cadd(a0, a2), t1 = csub(a0, a2), t2 = cadd(a1, a3), t3 = mul_mi(csub(a1, a3));
      buf[p0] = cadd(t0, t2);
      buf[p0 + s] = cadd(t1, t3);
      buf[p0 + 2 * s] = csub(t0, t2);
      buf[p0 + 3 * s] = csub(t1, t3);
    }
    __syncthreads();
  }
}

// Block-wide max / sum of two values at once (one per packed query head).
__device__ __forceinline__ float2 block_max2(float2 v, float2* scratch, int tid) {
  v.x = wave_max(v.x);
  v.y = wave_max(v.y);
  __syncthreads();
  if ((tid & 63) == 0) scratch[tid >> 6] = v;
  __syncthreads();
  float2 r = scratch[0];
  for (int w = 1; w < kFftThreads / 64; ++w) {
    r.x = fmaxf(r.x, scratch[w].x);
    r.y = fmaxf(r.y, scratch[w].y);
  }
  return r;
}
__device__ __forceinline__ float2 block_sum2(float2 v, float2* scratch, int tid) {
  v.x = wave_sum(v.x);
  v.y = wave_sum(v.y);
  __syncthreads();
  if ((tid & 63) == 0) scratch[tid >> 6] = v;
  __syncthreads();
  float2 r = scratch[0];
  for (int w = 1; w < kFftThreads / 64; ++w) {
    r.x += scratch[w].x;
    r.y += scratch[w].y;
  }
  return r;
}

// grid: slice * pairs + pair.  Two query heads share one complex transform: head g0 travels in
// the real part, head g0+1 in the imaginary part (each head's spectrum is made Hermitian first,
// so its time-domain signal is real).  Time index a = Pb * a' + b: block b of Q = M / Pb samples
// comes from the spectrum folded modulo Q with twiddle e^{j 2 pi k b / M}; softmax runs online
// across the Pb blocks.
__global__ __launch_bounds__(kFftThreads) void attn_fft_kernel(Params P, const float2* __restrict__ qc,
                                                              float2* __restrict__ Pn, float scale,
                                                              int pairs, int logQ) {
  extern __shared__ float2 buf[];
  __shared__ float2 scratch[kFftThreads / 64];
  const int tid = threadIdx.x;
  const int pair = blockIdx.x % pairs;
  const int slice = blockIdx.x / pairs;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const int g0 = pair * 2;
  const bool has1 = (g0 + 1) < P.G;
  const int Q = 1 << logQ;
  const uint32_t Pb = P.M >> logQ;
  const float2* q0 = qc + L.ws_off + ((int64_t)s * P.G + g0) * L.Bp;
  const float2* q1 = q0 + L.Bp;

  float2 Y0[kFftNBT], Y1[kFftNBT], A0[kFftNBT], A1[kFftNBT];
  uint32_t kk[kFftNBT];
  const float gain = 0.5f * scale / (float)P.M;  // 0.5: each bin is split into k and its mirror
#pragma unroll
  for (int j = 0; j < kFftNBT; ++j) {
    const int i = j * kFftThreads + tid;
    Y0[j] = Y1[j] = A0[j] = A1[j] = make_float2(0.f, 0.f);
    kk[j] = 0;
    if (i < L.nb) {
      kk[j] = (uint32_t)P.bins[L.bin_off + i];
      const float w = P.weights[L.bin_off + i] * gain;
      const float2 a = q0[i];
      Y0[j] = make_float2(a.x * w, a.y * w);
      if (has1) {
        const float2 b = q1[i];
        Y1[j] = make_float2(b.x * w, b.y * w);
      }
    }
  }
  float2 m = make_float2(-INFINITY, -INFINITY), Z = make_float2(0.f, 0.f);

  for (uint32_t b = 0; b < Pb; ++b) {
    for (int e = tid; e < Q; e += kFftThreads) buf[e] = make_float2(0.f, 0.f);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kFftNBT; ++j) {
      if (j * kFftThreads + tid < L.nb) {
        const float2 tw = cis(mulmod(kk[j], b, P.M, P.Mmask), P.M);
        const float2 z0 = cmul(Y0[j], tw), z1 = cmul(Y1[j], tw);
        const int r = kk[j] & (Q - 1), rm = (Q - r) & (Q - 1);
        atomicAdd(&buf[r].x, z0.x - z1.y);   //      z0  + j z1
        atomicAdd(&buf[r].y, z0.y + z1.x);
        atomicAdd(&buf[rm].x, z0.x + z1.y);  // conj z0  + j conj z1
        atomicAdd(&buf[rm].y, z1.x - z0.y);
      }
    }
    __syncthreads();
    ifft_dif(buf, logQ, tid);

    float2 v[kFftEPT];
    float2 lm = make_float2(-INFINITY, -INFINITY);
#pragma unroll
    for (int j = 0; j < kFftEPT; ++j) {
      const int e = j * kFftThreads + tid;
      if (e < Q) {
        v[j] = buf[e];
        lm.x = fmaxf(lm.x, v[j].x);
        lm.y = fmaxf(lm.y, v[j].y);
      }
    }
    const float2 bm = block_max2(lm, scratch, tid);
    const float2 mn = make_float2(fmaxf(m.x, bm.x), fmaxf(m.y, bm.y));
    const float2 f = make_float2(__expf(m.x - mn.x), __expf(m.y - mn.y));  // exp(-inf) = 0 first time
    m = mn;
    float2 ls = make_float2(0.f, 0.f);
#pragma unroll
    for (int j = 0; j < kFftEPT; ++j) {
      const int e = j * kFftThreads + tid;
      if (e < Q) {
        const float2 p = make_float2(__expf(v[j].x - mn.x), has1 ? __expf(v[j].y - mn.y) : 0.f);
        ls.x += p.x;
        ls.y += p.y;
        buf[e] = p;
      }
    }
    const float2 bs = block_sum2(ls, scratch, tid);
    Z = make_float2(Z.x * f.x + bs.x, Z.y * f.y + bs.y);
    __syncthreads();
    fft_dit(buf, logQ, tid);
#pragma unroll
    for (int j = 0; j < kFftNBT; ++j) {
      if (j * kFftThreads + tid < L.nb) {
        const float2 tw = cis(mulmod(kk[j], b, P.M, P.Mmask), P.M);
        const int r = kk[j] & (Q - 1), rm = (Q - r) & (Q - 1);
        const float2 w1 = buf[r], w2 = buf[rm];
        const float2 p0 = make_float2(0.5f * (w1.x + w2.x), 0.5f * (w1.y - w2.y));
        const float2 p1 = make_float2(0.5f * (w1.y + w2.y), 0.5f * (w2.x - w1.x));
        A0[j] = cadd(make_float2(A0[j].x * f.x, A0[j].y * f.x), cmul(conjf2(tw), p0));
        A1[j] = cadd(make_float2(A1[j].x * f.y, A1[j].y * f.y), cmul(conjf2(tw), p1));
      }
    }
    __syncthreads();
  }

  float2* o0 = Pn + L.ws_off + ((int64_t)s * P.G + g0) * L.Bp;
  float2* o1 = o0 + L.Bp;
  const float inv_M = 1.0f / (float)P.M;
#pragma unroll
  for (int j = 0; j < kFftNBT; ++j) {
    const int i = j * kFftThreads + tid;
    if (i < L.Bp) {  // padding entries are written as zeros: kernel C reads whole rows
      float2 r0 = make_float2(0.f, 0.f), r1 = r0;
      if (i < L.nb) {
        const float w = P.weights[L.bin_off + i] * inv_M;
        const float c0 = w / Z.x;
        r0 = make_float2(A0[j].x * c0, -A0[j].y * c0);
        if (has1) {
          const float c1 = w / Z.y;
          r1 = make_float2(A1[j].x * c1, -A1[j].y * c1);
        }
      }
      o0[i] = r0;
      if (has1) o1[i] = r1;
    }
  }
}

// ---------------------------------------------------------------------------------- B (direct)
constexpr int kDirThreads = 256;
constexpr int kDirStage = 1024;

// grid: slice * G + g.  Evaluates the score and weight sums term by term; O(M |B|) per head.
__global__ __launch_bounds__(kDirThreads) void attn_direct_kernel(Params P, const float2* __restrict__ qc,
                                                                 float2* __restrict__ Pn, float scale,
                                                                 float* __restrict__ scores) {
  __shared__ float2 Ys[kDirStage];
  __shared__ uint32_t ks[kDirStage];
  __shared__ float redf[kDirThreads / 64];
  const int tid = threadIdx.x;
  const int g = blockIdx.x % P.G;
  const int slice = blockIdx.x / P.G;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const float2* qrow = qc + L.ws_off + ((int64_t)s * P.G + g) * L.Bp;
  float* sc = scores + (int64_t)blockIdx.x * P.M;
  const float gain = scale / (float)P.M;

  for (int c0 = 0; c0 < L.nb; c0 += kDirStage) {
    const int cn = min(kDirStage, L.nb - c0);
    __syncthreads();
    for (int e = tid; e < cn; e += kDirThreads) {
      const float w = P.weights[L.bin_off + c0 + e] * gain;
      const float2 a = qrow[c0 + e];
      Ys[e] = make_float2(a.x * w, a.y * w);
      ks[e] = (uint32_t)P.bins[L.bin_off + c0 + e];
    }
    __syncthreads();
    for (uint32_t a = tid; a < P.M; a += kDirThreads) {
      float acc = c0 ? sc[a] : 0.f;
      for (int e = 0; e < cn; ++e) {
        const float2 w = cis(mulmod(ks[e], a, P.M, P.Mmask), P.M);
        acc += Ys[e].x * w.x - Ys[e].y * w.y;
      }
      sc[a] = acc;
    }
  }
  __syncthreads();
  float lm = -INFINITY;
  for (uint32_t a = tid; a < P.M; a += kDirThreads) lm = fmaxf(lm, sc[a]);
  lm = wave_max(lm);
  if ((tid & 63) == 0) redf[tid >> 6] = lm;
  __syncthreads();
  float mx = redf[0];
  for (int w = 1; w < kDirThreads / 64; ++w) mx = fmaxf(mx, redf[w]);
  __syncthreads();
  float lsum = 0.f;
  for (uint32_t a = tid; a < P.M; a += kDirThreads) {
    const float p = expf(sc[a] - mx);
    sc[a] = p;
    lsum += p;
  }
  lsum = wave_sum(lsum);
  if ((tid & 63) == 0) redf[tid >> 6] = lsum;
  __syncthreads();
  float Z = 0.f;
  for (int w = 0; w < kDirThreads / 64; ++w) Z += redf[w];

  float2* orow = Pn + L.ws_off + ((int64_t)s * P.G + g) * L.Bp;
  const float inv_M = 1.0f / (float)P.M;
  for (int i = tid; i < L.Bp; i += kDirThreads) {
    float2 r = make_float2(0.f, 0.f);
    if (i < L.nb) {
      const uint32_t k = (uint32_t)P.bins[L.bin_off + i];
      float re = 0.f, im = 0.f;
      uint32_t ph = 0;
      for (uint32_t a = 0; a < P.M; ++a) {
        const float2 w = cis(ph, P.M);
        const float p = sc[a];
        re += p * w.x;
        im += p * w.y;  // conj of sum p e^{-j..} = sum p e^{+j..}
        ph += k;
        if (ph >= P.M) ph -= P.M;
      }
      const float c = P.weights[L.bin_off + i] * inv_M / Z;
      r = make_float2(re * c, im * c);
    }
    orow[i] = r;
  }
}

// --------------------------------------------------------------------------------------- host
template <bool BF16>
static hipError_t launch_attn_t(const Params& P, const void* q, void* out, float scale, float2* qc,
                                float2* Pn, float* direct_scratch, bool use_fft, hipStream_t st) {
  const int GT = P.G >= 8 ? 8 : (P.G > 2 ? 4 : P.G);  // 1, 2, 4 or 8 heads per pass
  const int passes = (P.G + GT - 1) / GT;
  const int chunks = (P.max_Bp + kQcBins - 1) / kQcBins;
  const uint64_t gridA = (uint64_t)P.n_slices * chunks * passes;
  const uint64_t gridC = (uint64_t)P.n_slices * (kHeadDim / kOutDC) * passes;
  const uint64_t gridBd = (uint64_t)P.n_slices * P.G;
  if (gridA > 0x7fffffffull || gridC > 0x7fffffffull || gridBd > 0x7fffffffull)
    return hipErrorInvalidConfiguration;

#define IWDFT_GT_SWITCH(KERNEL, GRID, THREADS, ...)                                                 \
  switch (GT) {                                                                                     \
    case 1: KERNEL<BF16, 1><<<dim3((uint32_t)(GRID)), dim3(THREADS), 0, st>>>(__VA_ARGS__); break;  \
    case 2: KERNEL<BF16, 2><<<dim3((uint32_t)(GRID)), dim3(THREADS), 0, st>>>(__VA_ARGS__); break;  \
    case 4: KERNEL<BF16, 4><<<dim3((uint32_t)(GRID)), dim3(THREADS), 0, st>>>(__VA_ARGS__); break;  \
    default: KERNEL<BF16, 8><<<dim3((uint32_t)(GRID)), dim3(THREADS), 0, st>>>(__VA_ARGS__); break; \
  }

  IWDFT_GT_SWITCH(attn_qc_kernel, gridA, kQcThreads, P, q, qc, chunks, passes)
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  if (use_fft) {
    int logM = 0;
    while ((1u << logM) < P.M) ++logM;
    const int logQ = logM < kFftMaxLogQ ? logM : kFftMaxLogQ;
    const int pairs = (P.G + 1) / 2;
    const size_t lds = sizeof(float2) << logQ;
    static bool attr_set = false;  // raising the limit is idempotent; a race only repeats it
    if (!attr_set) {
      e = hipFuncSetAttribute((const void*)attn_fft_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)(sizeof(float2) << kFftMaxLogQ));
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    attn_fft_kernel<<<dim3((uint32_t)((uint64_t)P.n_slices * pairs)), dim3(kFftThreads), lds, st>>>(
        P, qc, Pn, scale, pairs, logQ);
  } else {
    attn_direct_kernel<<<dim3((uint32_t)gridBd), dim3(kDirThreads), 0, st>>>(P, qc, Pn, scale, direct_scratch);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;

  IWDFT_GT_SWITCH(attn_out_kernel, gridC, kOutThreads, P, Pn, out, passes)
#undef IWDFT_GT_SWITCH
  return hipGetLastError();
}

hipError_t launch_attn(const Params& P, const void* q, void* out, float scale, float2* qc, float2* Pn,
                       float* direct_scratch, bool use_fft, hipStream_t st) {
  return P.kv_dtype == 1 ? launch_attn_t<true>(P, q, out, scale, qc, Pn, direct_scratch, use_fft, st)
                         : launch_attn_t<false>(P, q, out, scale, qc, Pn, direct_scratch, use_fft, st);
}

}  // namespace iwdft
