// Prefill transform (Sec. 3.1.2 Eq. dft-full at the kept bins; Sec. 4.2.1 Eq. prefill-dft;
// Sec. 3.2 Eq. freq-zero realised as "never compute a discarded bin"):
//     F_M[k] = U_M[k] = sum_{n<M} x[n] exp(-j 2 pi k n / M)
// for every slice, channel and kept bin -- a dense contraction over the token axis of the
// cos / -sin basis against the K/V tile, run on the matrix cores.
//
// Work decomposition.  One workgroup (4 waves) owns 128 kept bins x the 256 channels of one
// slice (128 of K, 128 of V) and walks the token axis in tiles of 64.  MFMA roles are chosen so
// that lanes run along bins in the result (coalesced stores into the [channel][bin] state):
//     D[channel][bin] += A[channel][token] * B[token][bin]      v_mfma_f32_32x32x16_f16
//   A = X^T  : the K/V tile, converted to fp16 and transposed through LDS (token-contiguous rows)
//   B = basis: generated in registers.  A lane owns ONE bin k; for the 8 tokens it feeds to an
//       MFMA it needs exp(-j 2 pi k (n_base + i) / M) = base * t_i, with t_i = exp(-j 2 pi k i/M)
//       fixed for the whole kernel and base re-derived exactly (integer phase, sincospi) at every
//       64-token tile and stepped by exp(-j 2 pi k 16/M) in between.
// Precision.  bf16 inputs are exact in fp16; the basis is split into fp16 hi + lo parts (two MFMAs
// per product), which keeps ~20 bits of every basis value; fp32 inputs are split the same way
// (three MFMAs: x_hi*b_hi + x_hi*b_lo + x_lo*b_hi).  Accumulation is fp32.
#include "common.h"

namespace iwdft {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPfThreads = 256;
constexpr int kPfBins = 128;       // bins per workgroup (32 per wave)
constexpr int kPfTok = 64;         // tokens per tile
constexpr int kPfCh = 2 * kHeadDim;  // K and V channels of one slice
constexpr int kPfRS = kPfTok + 8;  // LDS row stride in halves (144 B: conflict-free b128 reads)
constexpr int kPfBlk = kPfCh / 32; // 32-channel MFMA row blocks

__device__ __forceinline__ uint32_t pack_rtz(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a, b));
}
__device__ __forceinline__ float half_lo_f32(uint32_t pk) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)(pk & 0xffffu));
}
__device__ __forceinline__ float half_hi_f32(uint32_t pk) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)(pk >> 16));
}

// Raw tile registers of one thread: 4 items, each = 2 tokens x 8 channels.
template <bool BF16>
struct TileRegs {
  uint4 v[BF16 ? 8 : 16];
};

template <bool BF16>
__device__ __forceinline__ void load_tile(TileRegs<BF16>& r, const void* __restrict__ K,
                                          const void* __restrict__ V, int64_t slice_base, uint32_t n0,
                                          uint32_t M, int tid) {
  const int p = tid & 31;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int q = (tid >> 5) + 8 * it;  // 8-channel group 0..31 (0..15 K, 16..31 V)
    const void* X = (q >> 4) ? V : K;
    const int ch = (q & 15) * 8;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const uint32_t n = n0 + 2 * p + t;
      const int64_t e = slice_base + (int64_t)n * kHeadDim + ch;  // element index
      if constexpr (BF16) {
        r.v[it * 2 + t] = (n < M) ? *(const uint4*)((const uint16_t*)X + e) : make_uint4(0, 0, 0, 0);
      } else {
        r.v[(it * 2 + t) * 2] = (n < M) ? *(const uint4*)((const float*)X + e) : make_uint4(0, 0, 0, 0);
        r.v[(it * 2 + t) * 2 + 1] = (n < M) ? *(const uint4*)((const float*)X + e + 4) : make_uint4(0, 0, 0, 0);
      }
    }
  }
}

// Converts to fp16 (hi, and lo for fp32 inputs) and writes token pairs transposed into LDS:
// element (channel c, token n) of part `part` lives at lds[(part * 256 + c) * kPfRS + n].
template <bool BF16>
__device__ __forceinline__ void store_tile(const TileRegs<BF16>& r, _Float16* __restrict__ buf, int tid) {
  const int p = tid & 31;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int q = (tid >> 5) + 8 * it;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float x0, x1;
      if constexpr (BF16) {
        const uint4 a = r.v[it * 2], b = r.v[it * 2 + 1];
        const uint32_t wa = (&a.x)[j >> 1], wb = (&b.x)[j >> 1];
        x0 = __uint_as_float((j & 1) ? (wa & 0xffff0000u) : (wa << 16));
        x1 = __uint_as_float((j & 1) ? (wb & 0xffff0000u) : (wb << 16));
      } else {
        const uint4 a = r.v[(it * 2) * 2 + (j >> 2)], b = r.v[(it * 2 + 1) * 2 + (j >> 2)];
        x0 = __uint_as_float((&a.x)[j & 3]);
        x1 = __uint_as_float((&b.x)[j & 3]);
      }
      const int c = q * 8 + j;
      const uint32_t hi = pack_rtz(x0, x1);
      *(uint32_t*)(buf + c * kPfRS + 2 * p) = hi;
      if constexpr (!BF16) {
        const uint32_t lo = pack_rtz(x0 - half_lo_f32(hi), x1 - half_hi_f32(hi));
        *(uint32_t*)(buf + (kPfCh + c) * kPfRS + 2 * p) = lo;
      }
    }
  }
}

// grid: 8 * per_xcd workgroups; id -> (id % 8) * per_xcd + id / 8 so that workgroups that run on
// the same XCD at the same time are the bin tiles of the same slice and share its K/V tile in L2.
template <bool BF16>
__global__ __launch_bounds__(kPfThreads) void prefill_mfma_kernel(Params P, const void* __restrict__ K,
                                                                 const void* __restrict__ V, int nt,
                                                                 int per_xcd, int total) {
  extern __shared__ _Float16 lds[];
  constexpr int kParts = BF16 ? 1 : 2;
  constexpr int kBufHalves = kParts * kPfCh * kPfRS;

  const int logical = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (logical >= total) return;
  const int tile = logical % nt;
  const int slice = logical / nt;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  if (tile * kPfBins >= L.nb) return;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5;  // which 8 of the 16 tokens of an MFMA this lane feeds
  const int bi = tile * kPfBins + wave * 32 + (lane & 31);
  const bool valid = bi < L.nb;
  const uint32_t k = valid ? (uint32_t)P.bins[L.bin_off + bi] : 0u;
  const uint32_t M = P.M, Mmask = P.Mmask;

  float2 tw[8];  // exp(-j 2 pi k i / M), i = 0..7
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float2 c = cis(mulmod(k, (uint32_t)i, M, Mmask), M);
    tw[i] = make_float2(c.x, -c.y);
  }
  float2 r16;
  {
    const float2 c = cis(mulmod(k, 16u, M, Mmask), M);
    r16 = make_float2(c.x, -c.y);
  }

  floatx16 acc_re[kPfBlk], acc_im[kPfBlk];
#pragma unroll
  for (int b = 0; b < kPfBlk; ++b) {
    acc_re[b] = (floatx16)(0.f);
    acc_im[b] = (floatx16)(0.f);
  }

  const int64_t slice_base = (int64_t)slice * M * kHeadDim;
  const uint32_t n_tiles = (M + kPfTok - 1) / kPfTok;
  TileRegs<BF16> regs;
  load_tile<BF16>(regs, K, V, slice_base, 0, M, tid);
  store_tile<BF16>(regs, lds, tid);
  __syncthreads();

  for (uint32_t t = 0; t < n_tiles; ++t) {
    const _Float16* cur = lds + (t & 1) * kBufHalves;
    _Float16* nxt = lds + ((t + 1) & 1) * kBufHalves;
    const bool more = (t + 1) < n_tiles;
    if (more) load_tile<BF16>(regs, K, V, slice_base, (t + 1) * kPfTok, M, tid);

    // exact basis phase at the first token this lane feeds in this tile
    float2 base;
    {
      const uint32_t nb0 = t * kPfTok + 8 * g;
      const float2 c = cis(mulmod(k, nb0, M, Mmask), M);
      base = make_float2(c.x, -c.y);
    }
#pragma unroll
    for (int st = 0; st < kPfTok / 16; ++st) {
      // basis for tokens t*64 + 16*st + 8*g + i : hi / lo halves of cos and -sin
      u32x4 ch, cl, sh, sl;
#pragma unroll
      for (int i = 0; i < 8; i += 2) {
        const float2 z0 = cmul(base, tw[i]), z1 = cmul(base, tw[i + 1]);
        const uint32_t chi = pack_rtz(z0.x, z1.x), shi = pack_rtz(z0.y, z1.y);
        ch[i >> 1] = chi;
        sh[i >> 1] = shi;
        cl[i >> 1] = pack_rtz(z0.x - half_lo_f32(chi), z1.x - half_hi_f32(chi));
        sl[i >> 1] = pack_rtz(z0.y - half_lo_f32(shi), z1.y - half_hi_f32(shi));
      }
      base = cmul(base, r16);
      const half8 bch = __builtin_bit_cast(half8, ch), bcl = __builtin_bit_cast(half8, cl);
      const half8 bsh = __builtin_bit_cast(half8, sh), bsl = __builtin_bit_cast(half8, sl);

      half8 a[kPfBlk];
#pragma unroll
      for (int b = 0; b < kPfBlk; ++b)
        a[b] = *(const half8*)(cur + (b * 32 + (lane & 31)) * kPfRS + 16 * st + 8 * g);
#pragma unroll
      for (int b = 0; b < kPfBlk; ++b) acc_re[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[b], bch, acc_re[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < kPfBlk; ++b) acc_im[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[b], bsh, acc_im[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < kPfBlk; ++b) acc_re[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[b], bcl, acc_re[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < kPfBlk; ++b) acc_im[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[b], bsl, acc_im[b], 0, 0, 0);
      if constexpr (!BF16) {
#pragma unroll
        for (int b = 0; b < kPfBlk; ++b) {
          const half8 al = *(const half8*)(cur + (kPfCh + b * 32 + (lane & 31)) * kPfRS + 16 * st + 8 * g);
          acc_re[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bch, acc_re[b], 0, 0, 0);
          acc_im[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, bsh, acc_im[b], 0, 0, 0);
        }
      }
    }
    if (more) store_tile<BF16>(regs, nxt, tid);
    __syncthreads();
  }

  if (!valid) return;
  // D layout of the 32x32 MFMA: register i of a lane is row 8*(i/4) + 4*(lane/32) + i%4, column lane%32.
#pragma unroll
  for (int b = 0; b < kPfBlk; ++b) {
    float2* F = (b < kPfBlk / 2 ? P.FK : P.FV) + L.coef_off + (int64_t)s * kHeadDim * L.Bp + bi;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int c = (b % (kPfBlk / 2)) * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
      F[(int64_t)c * L.Bp] = make_float2(acc_re[b][i], acc_im[b][i]);
    }
  }
}

hipError_t launch_prefill(const Params& P, const void* K, const void* V, hipStream_t st) {
  const int nt = (P.max_nb + kPfBins - 1) / kPfBins;
  const uint64_t total = (uint64_t)P.n_slices * nt;
  if (total > 0x3fffffffull) return hipErrorInvalidConfiguration;
  const int per_xcd = (int)((total + 7) / 8);
  const bool bf16 = P.kv_dtype == 1;
  const size_t lds = sizeof(_Float16) * 2 * (bf16 ? 1 : 2) * kPfCh * kPfRS;
  static bool attr_set = false;  // idempotent; a race only repeats the call
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)prefill_mfma_kernel<true>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)(sizeof(_Float16) * 2 * kPfCh * kPfRS));
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void*)prefill_mfma_kernel<false>,
                              hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)(sizeof(_Float16) * 4 * kPfCh * kPfRS));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  if (bf16)
    prefill_mfma_kernel<true><<<dim3((uint32_t)(per_xcd * 8)), dim3(kPfThreads), lds, st>>>(P, K, V, nt, per_xcd, (int)total);
  else
    prefill_mfma_kernel<false><<<dim3((uint32_t)(per_xcd * 8)), dim3(kPfThreads), lds, st>>>(P, K, V, nt, per_xcd, (int)total);
  return hipGetLastError();
}

}  // namespace iwdft
