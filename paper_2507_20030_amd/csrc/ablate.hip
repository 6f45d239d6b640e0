// The frequency-ablation tools of Sec. 3.2: the greedy per-layer mask (host integer work) and the
// device routine that removes one frequency chunk from a K or V tensor (Eq. freq-zero followed by the
// inverse DFT), which the offline study runs once per (layer, chunk).
#include <algorithm>
#include <cmath>
#include <vector>

#include "common.h"
#include "fft_lds.h"

namespace iwdft {

namespace {
constexpr int kAbPairs = kHeadDim / 2;

}  // namespace

// One workgroup = two adjacent channels of one slice, packed as one complex signal: forward transform,
// weights h[k] = 1 - ([k in chunk] + [M-k in chunk]) / 2 (the real part of the inverse transform of a
// real signal's spectrum with the chunk zeroed; symmetric, so both packed channels stay real), inverse
// transform, 1/M.  Block ids are dealt so that the 64 workgroups of a slice share one XCD's L2.
template <int LOGQ, bool BF16>
__global__ __launch_bounds__(kFftThreads, 4) void ablate_kernel(const char* __restrict__ x, char* __restrict__ out,
                                                               int n_slices, int per_xcd, int lo, int hi) {
  extern __shared__ float2 smem[];
  constexpr int Q = 1 << LOGQ;
  constexpr int kElem = BF16 ? 2 : 4;
  constexpr int kRow = kHeadDim * kElem;
  float2* buf = smem;
  float2* tab = smem + Q + (Q >> 5);
  const int tid = threadIdx.x;
  const uint32_t idx = blockIdx.x >> 3;
  const uint32_t slice = (blockIdx.x & 7u) * (uint32_t)per_xcd + idx / kAbPairs;
  if (slice >= (uint32_t)n_slices) return;
  const int64_t base = (int64_t)slice * Q * kRow + (idx % kAbPairs) * 2 * kElem;
  const char* X = x + base;
  char* Y = out + base;

  for (int m = tid; m <= (Q >> 3); m += kFftThreads) tab[m] = cis((uint32_t)m, (uint32_t)Q);

  constexpr int H = (LOGQ & 1) ? Q / 2 : Q;  // samples walked per thread loop (odd: pairs a, a + Q/2)
  constexpr int IT = (H + kFftThreads - 1) / kFftThreads;
  {
    float2 za[IT], zc[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int a = it * kFftThreads + tid;
      if (H % kFftThreads == 0 || a < H) {
        za[it] = load_pair<BF16>(X + (int64_t)a * kRow);
        if (LOGQ & 1) zc[it] = load_pair<BF16>(X + (int64_t)(a + H) * kRow);
      }
    }
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int a = it * kFftThreads + tid;
      if (H % kFftThreads == 0 || a < H) {
        const int p = digit_pos<LOGQ>(a);
        if (LOGQ & 1) {
          buf[pad(p)] = cadd(za[it], zc[it]);
          buf[pad(p + 1)] = csub(za[it], zc[it]);
        } else {
          buf[pad(p)] = za[it];
        }
      }
    }
  }
  __syncthreads();
  fft_dit<LOGQ>(buf, tab, tid);  // natural-order spectrum
  const float inv = 1.0f / (float)Q;
  for (int k = tid; k < Q; k += kFftThreads) {
    const int km = (Q - k) & (Q - 1);
    const float h = 1.0f - 0.5f * (float)((k >= lo && k < hi) + (km >= lo && km < hi));
    float2 v = buf[pad(k)];
    buf[pad(k)] = make_float2(v.x * h * inv, v.y * h * inv);
  }
  __syncthreads();
  ifft_dif<LOGQ>(buf, tab, tid);
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const int a = it * kFftThreads + tid;
    if (H % kFftThreads == 0 || a < H) {
      const int p = digit_pos<LOGQ>(a);
      if (LOGQ & 1) {
        const float2 u = buf[pad(p)], w = buf[pad(p + 1)];
        store_pair<BF16>(Y + (int64_t)a * kRow, cadd(u, w));
        store_pair<BF16>(Y + (int64_t)(a + H) * kRow, csub(u, w));
      } else {
        store_pair<BF16>(Y + (int64_t)a * kRow, buf[pad(p)]);
      }
    }
  }
}

// M > 8192 (a power of two): the subtractive form.  Zeroing the chunk and taking the real part equals
//   x[n] - (1/M) Re sum_{k in chunk} X[k] e^{+j 2 pi k n / M},
// so only the chunk's coefficients are needed: they are formed like the FFT prefill does it (M / 8192
// decimated 8192-point transforms per channel pair, accumulated per bin in registers, at most 4096 bins at
// a time) and turned back like the FFT reconstruction does it (Hermitian halves folded modulo 8192, one
// inverse transform per residue of the token index), subtracting from the input row (first piece of the
// chunk) or from what the previous piece left in the output.
template <bool BF16>
__global__ __launch_bounds__(kFftThreads, 2) void ablate_long_kernel(const char* __restrict__ x, char* __restrict__ out,
                                                                    int n_slices, int per_xcd, uint32_t M, int lo,
                                                                    int hi) {
  extern __shared__ float2 smem[];
  constexpr int LOGQ = kFftMaxLogQ, Q = 1 << LOGQ, H = Q / 2, IT = H / kFftThreads;
  static_assert(LOGQ & 1, "written for the odd transform length 2^13");
  constexpr int kElem = BF16 ? 2 : 4;
  constexpr int kRow = kHeadDim * kElem;
  constexpr int kPiece = kFftNBT * kFftThreads;  // bins handled at a time
  float2* buf = smem;
  float2* tab = smem + Q + (Q >> 5);
  const int tid = threadIdx.x;
  const uint32_t idx = blockIdx.x >> 3;
  const uint32_t slice = (blockIdx.x & 7u) * (uint32_t)per_xcd + idx / kAbPairs;
  if (slice >= (uint32_t)n_slices) return;
  const int64_t base = (int64_t)slice * M * kRow + (idx % kAbPairs) * 2 * kElem;
  const char* X = x + base;
  char* Y = out + base;
  const uint32_t Pb = M >> LOGQ;
  const int64_t step = (int64_t)Pb * kRow;  // bytes between consecutive samples of one residue
  const float gain = 0.5f / (float)M;

  for (int m = tid; m <= (Q >> 3); m += kFftThreads) tab[m] = cis((uint32_t)m, (uint32_t)Q);

  for (int lo_p = lo; lo_p < hi; lo_p += kPiece) {
    const int hi_p = hi < lo_p + kPiece ? hi : lo_p + kPiece;
    float2 acc0[kFftNBT], acc1[kFftNBT];
#pragma unroll
    for (int j = 0; j < kFftNBT; ++j) acc0[j] = acc1[j] = make_float2(0.f, 0.f);

    // forward: X[k] of both channels for the bins of this piece
    for (uint32_t b = 0; b < Pb; ++b) {
      int lt = tid;
      asm volatile("" : "+v"(lt));  // keeps the passes' address arithmetic out of long-lived registers
      const char* Xb = X + (int64_t)b * kRow;
#pragma unroll
      for (int g0 = 0; g0 < IT; g0 += 4) {
        float2 za[4], zc[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int a = (g0 + it) * kFftThreads + lt;
          za[it] = load_pair<BF16>(Xb + (int64_t)a * step);
          zc[it] = load_pair<BF16>(Xb + (int64_t)(a + H) * step);
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int p = digit_pos<LOGQ>((g0 + it) * kFftThreads + lt);
          buf[pad(p)] = cadd(za[it], zc[it]);
          buf[pad(p + 1)] = csub(za[it], zc[it]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      __syncthreads();
      fft_dit<LOGQ>(buf, tab, lt);
#pragma unroll
      for (int j = 0; j < kFftNBT; ++j) {
        const uint32_t k = (uint32_t)(lo_p + j * kFftThreads + tid);
        if ((int)k < hi_p) {
          const int r = k & (Q - 1), rm = (Q - r) & (Q - 1);
          const float2 w1 = buf[pad(r)], w2 = buf[pad(rm)];
          const float2 d0 = make_float2(0.5f * (w1.x + w2.x), 0.5f * (w1.y - w2.y));
          const float2 d1 = make_float2(0.5f * (w1.y + w2.y), 0.5f * (w2.x - w1.x));
          const float2 tw = conjf2(cis_poly2((k * b) & (M - 1u), M));
          acc0[j] = cadd(acc0[j], cmul(tw, d0));
          acc1[j] = cadd(acc1[j], cmul(tw, d1));
        }
      }
      __syncthreads();
    }

    // inverse: y[n] = (1/M) Re sum_k X[k] e^{+j 2 pi k n / M}, residue by residue, subtracted in place
    for (uint32_t b = 0; b < Pb; ++b) {
      int lt = tid;
      asm volatile("" : "+v"(lt));
      for (int e = tid; e < Q + (Q >> 5); e += kFftThreads) buf[e] = make_float2(0.f, 0.f);
      __syncthreads();
      // the bins of a piece are consecutive and at most Q many: distinct slots k mod Q, and distinct mirror
      // slots; a mirror slot may coincide with a direct one, so the mirrors are added in a second round
#pragma unroll
      for (int round = 0; round < 2; ++round) {
#pragma unroll
        for (int j = 0; j < kFftNBT; ++j) {
          const uint32_t k = (uint32_t)(lo_p + j * kFftThreads + tid);
          if ((int)k < hi_p) {
            const float2 tw = cis_poly2((k * b) & (M - 1u), M);
            const float2 z0 = cmul(make_float2(acc0[j].x * gain, acc0[j].y * gain), tw);
            const float2 z1 = cmul(make_float2(acc1[j].x * gain, acc1[j].y * gain), tw);
            const int r = k & (Q - 1), rm = (Q - r) & (Q - 1);
            if (round == 0) buf[pad(r)] = make_float2(z0.x - z1.y, z0.y + z1.x);                 //      z0 + j z1
            else buf[pad(rm)] = cadd(buf[pad(rm)], make_float2(z0.x + z1.y, z1.x - z0.y));       // conj z0 + j conj z1
          }
        }
        __syncthreads();
      }
      ifft_dif<LOGQ>(buf, tab, lt);
      const char* src = (lo_p == lo) ? X : (const char*)Y;  // later pieces continue from their own output
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        const int a = it * kFftThreads + tid;
        const int p = digit_pos<LOGQ>(a);
        const float2 u = buf[pad(p)], w = buf[pad(p + 1)];
        const int64_t o0 = ((int64_t)a * Pb + b) * kRow, o1 = ((int64_t)(a + H) * Pb + b) * kRow;
        const float2 x0 = load_pair<BF16>(src + o0), x1 = load_pair<BF16>(src + o1);
        store_pair<BF16>(Y + o0, csub(x0, cadd(u, w)));
        store_pair<BF16>(Y + o1, csub(x1, csub(u, w)));
      }
      __syncthreads();
    }
  }
}

template <bool BF16>
static hipError_t launch_ablate_t(const void* x, void* out, int n_slices, int logQ, int lo, int hi, hipStream_t st) {
  const int per_xcd = (n_slices + 7) / 8;
  const uint64_t blocks = (uint64_t)per_xcd * kAbPairs * 8;
  if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
  const size_t lds = sizeof(float2) * (size_t)fft_lds_float2(logQ);
  hipError_t e = hipSuccess;
#define IWDFT_AB_CASE(LQ)                                                                                    \
  {                                                                                                          \
    static LdsLimit lim;                                                                                     \
    e = lim.ensure((const void*)ablate_kernel<LQ, BF16>, (int)lds);                                          \
    if (e != hipSuccess) return e;                                                                           \
    ablate_kernel<LQ, BF16><<<dim3((uint32_t)blocks), dim3(kFftThreads), lds, st>>>((const char*)x, (char*)out, \
                                                                                   n_slices, per_xcd, lo, hi); \
  }
  switch (logQ) {
    case 8: IWDFT_AB_CASE(8) break;
    case 9: IWDFT_AB_CASE(9) break;
    case 10: IWDFT_AB_CASE(10) break;
    case 11: IWDFT_AB_CASE(11) break;
    case 12: IWDFT_AB_CASE(12) break;
    case 13: IWDFT_AB_CASE(13) break;
    default: return hipErrorInvalidValue;
  }
#undef IWDFT_AB_CASE
  return hipGetLastError();
}

hipError_t launch_ablate(const void* x, void* out, int n_slices, uint32_t M, int kv_dtype, int lo, int hi,
                         hipStream_t st) {
  int logM = 0;
  while ((1u << logM) < M) ++logM;
  if (logM <= kFftMaxLogQ)
    return kv_dtype == 1 ? launch_ablate_t<true>(x, out, n_slices, logM, lo, hi, st)
                         : launch_ablate_t<false>(x, out, n_slices, logM, lo, hi, st);
  const int per_xcd = (n_slices + 7) / 8;
  const uint64_t blocks = (uint64_t)per_xcd * kAbPairs * 8;
  if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
  const size_t lds = sizeof(float2) * (size_t)fft_lds_float2(kFftMaxLogQ);
  static LdsLimit lim16, lim32;
  hipError_t e = kv_dtype == 1 ? lim16.ensure((const void*)ablate_long_kernel<true>, (int)lds)
                               : lim32.ensure((const void*)ablate_long_kernel<false>, (int)lds);
  if (e != hipSuccess) return e;
  if (kv_dtype == 1)
    ablate_long_kernel<true><<<dim3((uint32_t)blocks), dim3(kFftThreads), lds, st>>>((const char*)x, (char*)out, n_slices,
                                                                                   per_xcd, M, lo, hi);
  else
    ablate_long_kernel<false><<<dim3((uint32_t)blocks), dim3(kFftThreads), lds, st>>>((const char*)x, (char*)out, n_slices,
                                                                                    per_xcd, M, lo, hi);
  return hipGetLastError();
}

// chunk c of C = bins [floor(c M / C), floor((c + 1) M / C))
int64_t chunk_edge(int64_t c, int64_t M, int64_t C) { return (c * M) / C; }

int select_chunks(const float* delta, int n_chunks, double r, std::vector<int>* keep) {
  for (int c = 0; c < n_chunks; ++c)
    if (std::isnan(delta[c])) return -1;
  volatile double scaled = r * (double)n_chunks;  // volatile: the product is rounded before the add
  double n = std::floor(scaled + 0.5);
  if (n < 1.0) n = 1.0;
  if (n > (double)n_chunks) n = (double)n_chunks;
  std::vector<int> order(n_chunks);
  for (int c = 0; c < n_chunks; ++c) order[c] = c;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return delta[a] > delta[b]; });
  keep->assign(order.begin(), order.begin() + (int)n);
  std::sort(keep->begin(), keep->end());
  return 0;
}

}  // namespace iwdft
