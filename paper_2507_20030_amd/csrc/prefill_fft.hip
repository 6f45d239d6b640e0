// Prefill transform through FFTs (Sec. 3.1.2 Eq. dft-full computed the way Sec. 3.1.2 / Sec. 4.2.1
// suggest, O(M log M) per channel, followed by the pruning of Eq. freq-zero): for every slice, channel
// and kept bin k the same U_M[k] = sum_n x[n] e^{-j 2 pi k n / M} as the dense contraction, for DFT
// lengths that are a power of two.
//
// One workgroup transforms two channels of one slice at a time, packed as the real and imaginary part
// of one complex signal z = x_c0 + j x_c1; the two spectra are separated afterwards with
// X_c0[k] = (Z[k] + conj Z[-k]) / 2, X_c1[k] = (Z[k] - conj Z[-k]) / (2j).  M > 8192: the token axis is
// decimated by Pb = M / 8192, n = Pb a + b, so that
//   U[k] = sum_b e^{-j 2 pi k b / M} * DFT_8192( x[Pb a + b] )[k mod 8192],
// one in-LDS transform per residue b, accumulated per kept bin in registers (only the kept bins are
// ever formed).  Each thread reads 4 bytes (bf16 pair) of a 256-byte token row, so the 64 workgroups
// of one (slice, tensor) are placed on one XCD next to each other in time and share the rows in that
// XCD's L2: HBM delivers every row once.
#include "common.h"
#include "fft_lds.h"

namespace iwdft {

constexpr int kPairs = kHeadDim / 2;  // channel pairs = workgroups per (slice, tensor)

// hardware block id -> (xcd = id & 7, idx = id >> 3); XCD x owns the (slice, tensor) pairs
// x * per_xcd .. (x + 1) * per_xcd - 1, 64 consecutive idx each.
template <int LOGQ, bool BF16, bool MULTI>
__global__ __launch_bounds__(kFftThreads, 4) void prefill_fft_kernel(Params P, const void* __restrict__ K,
                                                                    const void* __restrict__ V, int per_xcd,
                                                                    int n_st) {
  extern __shared__ float2 smem[];
  constexpr int Q = 1 << LOGQ;
  constexpr int kElem = BF16 ? 2 : 4;
  constexpr int kRow = kHeadDim * kElem;  // bytes per token row
  float2* buf = smem;
  float2* tab = smem + Q + (Q >> 5);
  const int tid = threadIdx.x;
  const uint32_t idx = blockIdx.x >> 3;
  const uint32_t st = (blockIdx.x & 7u) * (uint32_t)per_xcd + idx / kPairs;
  if (st >= (uint32_t)n_st) return;
  const int pair = idx % kPairs;
  const int tensor = st & 1;
  const int slice = st >> 1;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const int32_t* bins = P.bins + L.bin_off;
  const int64_t N = (int64_t)P.S + P.M + P.R;  // tokens per slice in the caller's tensor
  const char* X = (const char*)(tensor ? V : K) + ((int64_t)slice * N + P.S) * kRow + pair * 2 * kElem;
  const uint32_t Pb = MULTI ? (P.M >> LOGQ) : 1u;

  for (int m = tid; m <= (Q >> 3); m += kFftThreads) tab[m] = cis((uint32_t)m, (uint32_t)Q);

  float2 acc0[kFftNBT], acc1[kFftNBT];
  uint32_t kk[kFftNBT];
#pragma unroll
  for (int j = 0; j < kFftNBT; ++j) {
    acc0[j] = acc1[j] = make_float2(0.f, 0.f);
    const int i = j * kFftThreads + tid;
    kk[j] = (uint32_t)bins[i < L.nb ? i : L.nb - 1];
  }

  for (uint32_t b = 0; b < Pb; ++b) {
    // The thread index is made opaque per iteration so that the address arithmetic of the transform
    // passes is recomputed (a few instructions) instead of being hoisted out of the residue loop into
    // long-lived registers that would spill.
    int lt = tid;
    if (MULTI) asm volatile("" : "+v"(lt));
    const char* Xb = X + (int64_t)b * kRow;
    const int64_t step = (int64_t)Pb * kRow;  // bytes between consecutive samples of this residue
    if constexpr (LOGQ & 1) {
      constexpr int H = Q / 2, IT = (H + kFftThreads - 1) / kFftThreads;
      // MULTI: loads in groups of four sample pairs (the per-bin running sums leave few registers)
      constexpr int GRP = (MULTI && IT > 4) ? 4 : IT;
#pragma unroll
      for (int g0 = 0; g0 < IT; g0 += GRP) {
        float2 za[GRP], zc[GRP];
#pragma unroll
        for (int it = 0; it < GRP; ++it) {
          const int a = (g0 + it) * kFftThreads + lt;
          if (H % kFftThreads == 0 || a < H) {
            za[it] = load_pair<BF16>(Xb + (int64_t)a * step);
            zc[it] = load_pair<BF16>(Xb + (int64_t)(a + H) * step);
          }
        }
#pragma unroll
        for (int it = 0; it < GRP; ++it) {
          const int a = (g0 + it) * kFftThreads + lt;
          if (H % kFftThreads == 0 || a < H) {  // first radix-2 stage of the decimation-in-time order
            const int p = digit_pos<LOGQ>(a);
            buf[pad(p)] = cadd(za[it], zc[it]);
            buf[pad(p + 1)] = csub(za[it], zc[it]);
          }
        }
        if (GRP < IT) __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      constexpr int IT = (Q + kFftThreads - 1) / kFftThreads;
      float2 za[IT];
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        const int a = it * kFftThreads + lt;
        if (Q % kFftThreads == 0 || a < Q) za[it] = load_pair<BF16>(Xb + (int64_t)a * step);
      }
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        const int a = it * kFftThreads + lt;
        if (Q % kFftThreads == 0 || a < Q) buf[pad(digit_pos<LOGQ>(a))] = za[it];
      }
    }
    __syncthreads();  // (the first time also publishes tab)
    fft_dit<LOGQ>(buf, tab, lt);
#pragma unroll
    for (int j = 0; j < kFftNBT; ++j) {
      if (j * kFftThreads + tid < L.nb) {
        const int r = kk[j] & (Q - 1), rm = (Q - r) & (Q - 1);
        const float2 w1 = buf[pad(r)], w2 = buf[pad(rm)];
        const float2 d0 = make_float2(0.5f * (w1.x + w2.x), 0.5f * (w1.y - w2.y));
        const float2 d1 = make_float2(0.5f * (w1.y + w2.y), 0.5f * (w2.x - w1.x));
        if constexpr (MULTI) {
          const float2 tw = conjf2(cis_poly2((kk[j] * b) & (P.M - 1u), P.M));  // e^{-j 2 pi k b / M}
          acc0[j] = cadd(acc0[j], cmul(tw, d0));
          acc1[j] = cadd(acc1[j], cmul(tw, d1));
        } else {
          acc0[j] = d0;
          acc1[j] = d1;
        }
      }
    }
    if (MULTI) __syncthreads();
  }

  float2* F0 = (tensor ? P.FV : P.FK) + L.coef_off + ((int64_t)s * kHeadDim + pair * 2) * L.Bp;
  float2* F1 = F0 + L.Bp;
#pragma unroll
  for (int j = 0; j < kFftNBT; ++j) {
    const int i = j * kFftThreads + tid;
    if (i < L.nb) {
      F0[i] = acc0[j];
      F1[i] = acc1[j];
    }
  }
}

bool prefill_fft_ok(const Params& P) {
  return P.Mmask != 0 && P.M >= 256 && P.max_nb <= kFftNBT * kFftThreads;
}

template <bool BF16>
static hipError_t launch_prefill_fft_t(const Params& P, const void* K, const void* V, hipStream_t st) {
  int logM = 0;
  while ((1u << logM) < P.M) ++logM;
  const int logQ = logM < kFftMaxLogQ ? logM : kFftMaxLogQ;
  const int n_st = P.n_slices * 2;
  const int per_xcd = (n_st + 7) / 8;
  const uint64_t blocks = (uint64_t)per_xcd * kPairs * 8;
  if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
  const size_t lds = sizeof(float2) * (size_t)fft_lds_float2(logQ);
  hipError_t e = hipSuccess;
#define IWDFT_PF_CASE(LQ, MULTI)                                                                        \
  {                                                                                                     \
    static LdsLimit lim;                                                                                \
    e = lim.ensure((const void*)prefill_fft_kernel<LQ, BF16, MULTI>, (int)lds);                         \
    if (e != hipSuccess) return e;                                                                      \
    prefill_fft_kernel<LQ, BF16, MULTI><<<dim3((uint32_t)blocks), dim3(kFftThreads), lds, st>>>(P, K, V, \
                                                                                                per_xcd, n_st); \
  }
  if (logM > logQ) IWDFT_PF_CASE(kFftMaxLogQ, true)
  else switch (logQ) {
    case 8: IWDFT_PF_CASE(8, false) break;
    case 9: IWDFT_PF_CASE(9, false) break;
    case 10: IWDFT_PF_CASE(10, false) break;
    case 11: IWDFT_PF_CASE(11, false) break;
    case 12: IWDFT_PF_CASE(12, false) break;
    default: IWDFT_PF_CASE(13, false) break;
  }
#undef IWDFT_PF_CASE
  return hipGetLastError();
}

hipError_t launch_prefill_fft(const Params& P, const void* K, const void* V, hipStream_t st) {
  if (!prefill_fft_ok(P)) return hipErrorInvalidValue;
  hipError_t e = launch_prefill_edges(P, K, V, st);
  if (e != hipSuccess) return e;
  return P.kv_dtype == 1 ? launch_prefill_fft_t<true>(P, K, V, st) : launch_prefill_fft_t<false>(P, K, V, st);
}

}  // namespace iwdft
