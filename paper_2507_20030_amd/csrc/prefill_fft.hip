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
// ever formed).  Each thread reads a few bytes (1, 2 or 4 bf16 pairs) of a 256-byte token row, so the
// workgroups of one (slice, tensor) are placed on one XCD next to each other in time and share the rows
// in that XCD's L2: HBM delivers every row once.
#include "common.h"
#include "fft_lds.h"

namespace iwdft {

constexpr int kPairs = kHeadDim / 2;  // channel pairs per (slice, tensor)

// One token sample of NP adjacent channel pairs as NW 32-bit words (NW = NP for bf16, 2 NP for fp32), fetched
// with one load of 4 NW bytes.
template <int NW>
struct Raw {
  uint32_t w[NW];
};
template <int NW>
__device__ __forceinline__ Raw<NW> load_raw(const char* p) {
  Raw<NW> r;
  if constexpr (NW == 1) {
    r.w[0] = *(const uint32_t*)p;
  } else if constexpr (NW == 2) {
    const uint2 u = *(const uint2*)p;
    r.w[0] = u.x, r.w[1] = u.y;
  } else {
    static_assert(NW == 4, "1, 2 or 4 words per sample");
    const uint4 u = *(const uint4*)p;
    r.w[0] = u.x, r.w[1] = u.y, r.w[2] = u.z, r.w[3] = u.w;
  }
  return r;
}
// The first channel pair of a sample as a complex number (first channel real, second imaginary), and the
// sample with that pair dropped and the next one moved to the front: the pairs are taken in turn inside a
// run-time loop while the words stay in registers (no run-time index).
template <bool BF16, int NW>
__device__ __forceinline__ float2 raw_front(const Raw<NW>& r) {
  if constexpr (BF16) return make_float2(__uint_as_float(r.w[0] << 16), __uint_as_float(r.w[0] & 0xffff0000u));
  else return make_float2(__uint_as_float(r.w[0]), __uint_as_float(r.w[1]));
}
template <bool BF16, int NW>
__device__ __forceinline__ void raw_pop(Raw<NW>& r) {
  constexpr int W = BF16 ? 1 : 2;
#pragma unroll
  for (int n = 0; n + W < NW; ++n) r.w[n] = r.w[n + W];
}

// hardware block id -> (xcd = id & 7, idx = id >> 3); XCD x owns the (slice, tensor) pairs
// x * per_xcd .. (x + 1) * per_xcd - 1, 64 / NP consecutive idx each.
// NP = channel pairs per workgroup: every thread fetches its samples of NP adjacent pairs with one load
// (4 NP bytes of a token row for bf16) and the pairs are then transformed one after the other from
// registers, so that a 128-byte line of a token row is requested by 32 / NP workgroups instead of 32.
// NBT = kept bins per thread; 0: any number of kept bins -- the threads walk the bin list in strides of the workgroup
// and, in the decimated form, keep the running sums over the residues in the output rows themselves (every bin
// belongs to one thread, which reads back its own earlier store).
template <int LOGQ, bool BF16, bool MULTI, int NBT, int NP>
__global__ __launch_bounds__(kFftThreads, (MULTI && NBT > 4 && NP > 1) ? 2 : 4) void prefill_fft_kernel(Params P, const void* __restrict__ K,
                                                                    const void* __restrict__ V, int per_xcd,
                                                                    int n_st) {
  extern __shared__ float2 smem[];
  constexpr int Q = 1 << LOGQ;
  constexpr int kElem = BF16 ? 2 : 4;
  constexpr int kRow = kHeadDim * kElem;  // bytes per token row
  constexpr int NW = NP * (BF16 ? 1 : 2);
  constexpr int kGroups = kPairs / NP;    // workgroups per (slice, tensor)
  float2* buf = smem;
  float2* tab = smem + Q + (Q >> 5);
  const int tid = threadIdx.x;
  const uint32_t idx = blockIdx.x >> 3;
  const uint32_t st = (blockIdx.x & 7u) * (uint32_t)per_xcd + idx / kGroups;
  if (st >= (uint32_t)n_st) return;
  const int pair0 = (idx % kGroups) * NP;
  const int tensor = st & 1;
  const int slice = st >> 1;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const int32_t* bins = P.bins + L.bin_off;
  const int64_t N = (int64_t)P.S + P.M + P.R;  // tokens per slice in the caller's tensor
  const char* X = (const char*)(tensor ? V : K) + ((int64_t)slice * N + P.S) * kRow + pair0 * 2 * kElem;
  const uint32_t Pb = MULTI ? (P.M >> LOGQ) : 1u;
  float2* F = (tensor ? P.FV : P.FK) + L.coef_off + ((int64_t)s * kHeadDim + pair0 * 2) * L.Bp;

  for (int m = tid; m <= (Q >> 3); m += kFftThreads) tab[m] = P.tw8[m];  // exp(+j 2 pi m / Q), host-made

  // MULTI: running sums over the residues, per pair, channel and kept bin of this thread
  constexpr int NBR = NBT ? NBT : 1;  // register-held bins per thread
  float2 acc[MULTI ? NP : 1][2][NBR];
  uint32_t kk[NBR];
#pragma unroll
  for (int j = 0; j < NBT; ++j) {
#pragma unroll
    for (int p = 0; p < (MULTI ? NP : 1); ++p) acc[p][0][j] = acc[p][1][j] = make_float2(0.f, 0.f);
    const int i = j * kFftThreads + tid;
    kk[j] = (uint32_t)bins[i < L.nb ? i : L.nb - 1];
  }

  // samples per thread: IT sample pairs (a, a + Q/2) when the first radix-2 stage is taken here (odd LOGQ),
  // IT single samples otherwise
  constexpr bool kOdd = (LOGQ & 1) != 0;
  constexpr int H = kOdd ? Q / 2 : Q;
  constexpr int IT = (H + kFftThreads - 1) / kFftThreads;

  for (uint32_t b = 0; b < Pb; ++b) {
    // The thread index is made opaque per iteration so that the address arithmetic of the transform
    // passes is recomputed (a few instructions) instead of being hoisted out of the residue loop into
    // long-lived registers that would spill.
    int lt = tid;
    if (MULTI) asm volatile("" : "+v"(lt));
    const char* Xb = X + (int64_t)b * kRow;
    const int64_t step = (int64_t)Pb * kRow;  // bytes between consecutive samples of this residue
    // Thread -> sample assignment: consecutive threads own consecutive LDS positions of the digit-reversed
    // order (their stores fall into distinct banks) and fetch the samples that belong there; every sample is
    // a token row of its own, so the order of the loads is free.
    Raw<NW> za[IT], zc[kOdd ? IT : 1];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int i = it * kFftThreads + lt;
      if (H % kFftThreads == 0 || i < H) {
        const int a = digit_pos<kOdd ? LOGQ - 1 : LOGQ>(i);  // digit reversal is its own inverse
        za[it] = load_raw<NW>(Xb + (int64_t)a * step);
        if constexpr (kOdd) zc[it] = load_raw<NW>(Xb + (int64_t)(a + H) * step);
      }
    }
    // One pair after the other: scatter into the digit-reversed order of the decimation-in-time passes,
    // transform, separate the two channels' spectra at the kept bins.
    auto one_pair = [&](int p, auto& accp) {
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        const int i = it * kFftThreads + lt;
        if (H % kFftThreads == 0 || i < H) {
          const int pos = kOdd ? 2 * i : i;
          const float2 u = raw_front<BF16, NW>(za[it]);
          raw_pop<BF16, NW>(za[it]);
          if constexpr (kOdd) {  // first radix-2 stage
            const float2 v = raw_front<BF16, NW>(zc[it]);
            raw_pop<BF16, NW>(zc[it]);
            buf[pad(pos)] = cadd(u, v);
            buf[pad(pos + 1)] = csub(u, v);
          } else {
            buf[pad(pos)] = u;
          }
        }
      }
      __syncthreads();  // (the first time also publishes tab)
      fft_dit<LOGQ>(buf, tab, lt);
      float2* F0 = F + (int64_t)(2 * p) * L.Bp;
      if constexpr (NBT == 0) {
        for (int i = tid; i < L.nb; i += kFftThreads) {
          const uint32_t kj = (uint32_t)bins[i];
          const int r = kj & (Q - 1), rm = (Q - r) & (Q - 1);
          const float2 w1 = buf[pad(r)], w2 = buf[pad(rm)];
          float2 d0 = make_float2(0.5f * (w1.x + w2.x), 0.5f * (w1.y - w2.y));
          float2 d1 = make_float2(0.5f * (w1.y + w2.y), 0.5f * (w2.x - w1.x));
          if constexpr (MULTI) {
            const float2 tw = conjf2(cis_poly2((kj * b) & (P.M - 1u), P.M));  // e^{-j 2 pi k b / M}
            d0 = cmul(tw, d0);
            d1 = cmul(tw, d1);
            if (b) {
              d0 = cadd(F0[i], d0);
              d1 = cadd(F0[L.Bp + i], d1);
            }
          }
          F0[i] = d0;
          F0[L.Bp + i] = d1;
        }
      }
#pragma unroll
      for (int j = 0; j < NBT; ++j) {
        const int i = j * kFftThreads + tid;
        if (i < L.nb) {
          // decimated form with several pairs: the bin index is fetched again (an L1 / L2 hit) instead of being kept --
          // the registers it frees are what the kernel would otherwise spill
          const uint32_t kj = (MULTI && NP > 1) ? (uint32_t)bins[i] : kk[j];
          const int r = kj & (Q - 1), rm = (Q - r) & (Q - 1);
          const float2 w1 = buf[pad(r)], w2 = buf[pad(rm)];
          const float2 d0 = make_float2(0.5f * (w1.x + w2.x), 0.5f * (w1.y - w2.y));
          const float2 d1 = make_float2(0.5f * (w1.y + w2.y), 0.5f * (w2.x - w1.x));
          if constexpr (MULTI) {
            const float2 tw = conjf2(cis_poly2((kj * b) & (P.M - 1u), P.M));  // e^{-j 2 pi k b / M}
            accp[0][j] = cadd(accp[0][j], cmul(tw, d0));
            accp[1][j] = cadd(accp[1][j], cmul(tw, d1));
          } else {
            F0[i] = d0;
            F0[L.Bp + i] = d1;
          }
        }
      }
      __syncthreads();  // the next scatter overwrites buf
    };
    if constexpr (MULTI) {
#pragma unroll
      for (int p = 0; p < NP; ++p) one_pair(p, acc[p]);
    } else {
#pragma unroll 1
      for (int p = 0; p < NP; ++p) one_pair(p, acc[0]);
    }
  }

  if constexpr (MULTI && NBT > 0) {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      float2* F0 = F + (int64_t)(2 * p) * L.Bp;
#pragma unroll
      for (int j = 0; j < NBT; ++j) {
        const int i = j * kFftThreads + tid;
        if (i < L.nb) {
          F0[i] = acc[p][0][j];
          F0[L.Bp + i] = acc[p][1][j];
        }
      }
    }
  }
}

bool prefill_fft_ok(const Params& P) { return P.Mmask != 0 && P.M >= 256; }

template <bool BF16>
static hipError_t launch_prefill_fft_t(const Params& P, const void* K, const void* V, hipStream_t st) {
  int logM = 0;
  while ((1u << logM) < P.M) ++logM;
  const int logQ = logM < kFftMaxLogQ ? logM : kFftMaxLogQ;
  const int n_st = P.n_slices * 2;
  const int per_xcd = (n_st + 7) / 8;
  const size_t lds = sizeof(float2) * (size_t)fft_lds_float2(logQ);
  const int per_thread = (P.max_nb + kFftThreads - 1) / kFftThreads;
  // 16-byte sample loads need 16-byte aligned tensors (and rows, which are 256 or 512 bytes)
  const bool wide = (((uintptr_t)K | (uintptr_t)V) & 15u) == 0;
  hipError_t e = hipSuccess;
#define IWDFT_PF_CASE(LQ, MULTI, NBT, NP)                                                                    \
  {                                                                                                          \
    const uint64_t blocks = (uint64_t)per_xcd * (kPairs / (NP)) * 8;                                         \
    if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;                                         \
    static LdsLimit lim;                                                                                     \
    e = lim.ensure((const void*)prefill_fft_kernel<LQ, BF16, MULTI, NBT, NP>, (int)lds);                     \
    if (e != hipSuccess) return e;                                                                           \
    prefill_fft_kernel<LQ, BF16, MULTI, NBT, NP><<<dim3((uint32_t)blocks), dim3(kFftThreads), lds, st>>>(    \
        P, K, V, per_xcd, n_st);                                                                             \
  }
  // Pairs per workgroup: as many as the register budget (128) holds next to the transform -- the staged samples
  // take 16 registers per further bf16 pair, the running sums of the decimated form 4 per pair and kept bin.
#define IWDFT_PF_SINGLE(LQ)                                                                                  \
  {                                                                                                          \
    constexpr int kNpSingle = BF16 ? 4 : (LQ < 13 ? 2 : 1);                                                  \
    if (wide) IWDFT_PF_CASE(LQ, false, 8, kNpSingle)                                                         \
    else IWDFT_PF_CASE(LQ, false, 8, 1)                                                                      \
  }
  if (per_thread > kFftNBT) {  // more than 4096 kept bins in some layer (so M >= 8192): the bin-strided form
    constexpr int kNpBig = BF16 ? 2 : 1;
    if (logM > logQ) {
      if (wide) IWDFT_PF_CASE(kFftMaxLogQ, true, 0, kNpBig)
      else IWDFT_PF_CASE(kFftMaxLogQ, true, 0, 1)
    } else {
      if (wide) IWDFT_PF_CASE(kFftMaxLogQ, false, 0, kNpBig)
      else IWDFT_PF_CASE(kFftMaxLogQ, false, 0, 1)
    }
  } else if (logM > logQ) {
    if (per_thread <= 4) {
      constexpr int kNpMulti = BF16 ? 2 : 1;
      if (wide) IWDFT_PF_CASE(kFftMaxLogQ, true, 4, kNpMulti)
      else IWDFT_PF_CASE(kFftMaxLogQ, true, 4, 1)
    } else {
      // 5 .. 8 kept bins per thread: the running sums alone take 32 registers per pair, so the kernel that shares
      // its loads among four pairs gets the 256-register budget (one workgroup per CU); measured against one pair
      // per workgroup at 128 registers: 46 -> 43.5 ms (M = 32768, 2048 slices), 26.6 -> 20.5 ms (M = 131072, 256).
      constexpr int kNpMulti8 = BF16 ? 4 : 1;
      if (wide) IWDFT_PF_CASE(kFftMaxLogQ, true, 8, kNpMulti8)
      else IWDFT_PF_CASE(kFftMaxLogQ, true, 8, 1)
    }
  } else switch (logQ) {
    case 8: IWDFT_PF_SINGLE(8) break;
    case 9: IWDFT_PF_SINGLE(9) break;
    case 10: IWDFT_PF_SINGLE(10) break;
    case 11: IWDFT_PF_SINGLE(11) break;
    case 12: IWDFT_PF_SINGLE(12) break;
    default: IWDFT_PF_SINGLE(13) break;
  }
#undef IWDFT_PF_SINGLE
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
