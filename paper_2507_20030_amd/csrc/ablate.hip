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
  return kv_dtype == 1 ? launch_ablate_t<true>(x, out, n_slices, logM, lo, hi, st)
                       : launch_ablate_t<false>(x, out, n_slices, logM, lo, hi, st);
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
