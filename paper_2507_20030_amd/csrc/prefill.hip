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
// Precision.  bf16 inputs are exact in fp16 while 2^-14 <= |x| <= 65504 (smaller ones land in fp16 subnormals and
// lose bits, larger ones overflow -- the documented input range of this path); the basis is split into fp16 hi + lo parts (two MFMAs
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

// Raw tile registers of one thread.  fp32 inputs: 4 items of 2 tokens x 8 channels; bf16 inputs: 2 items of
// 4 tokens x 8 channels (one 16-byte load per token either way).
template <bool BF16>
struct TileRegs {
  uint4 v[BF16 ? 8 : 16];
};

// FULL: the tile lies entirely inside [0, M) and needs no bounds checks.
template <bool BF16, bool FULL>
__device__ __forceinline__ void load_tile(TileRegs<BF16>& r, const void* __restrict__ K,
                                          const void* __restrict__ V, int64_t slice_base, uint32_t n0,
                                          uint32_t M, int tid) {
  if constexpr (BF16) {
    const int p = tid & 15;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int q = (tid >> 4) + 16 * it;  // 8-channel group 0..31 (0..15 K, 16..31 V)
      const void* X = (q >> 4) ? V : K;
      const int ch = (q & 15) * 8;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint32_t n = n0 + 4 * p + t;
        const int64_t e = slice_base + (int64_t)n * kHeadDim + ch;  // element index
        r.v[it * 4 + t] = (FULL || n < M) ? *(const uint4*)((const uint16_t*)X + e) : make_uint4(0, 0, 0, 0);
      }
    }
  } else {
    const int p = tid & 31;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int q = (tid >> 5) + 8 * it;
      const void* X = (q >> 4) ? V : K;
      const int ch = (q & 15) * 8;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint32_t n = n0 + 2 * p + t;
        const int64_t e = slice_base + (int64_t)n * kHeadDim + ch;
        r.v[(it * 2 + t) * 2] = (FULL || n < M) ? *(const uint4*)((const float*)X + e) : make_uint4(0, 0, 0, 0);
        r.v[(it * 2 + t) * 2 + 1] = (FULL || n < M) ? *(const uint4*)((const float*)X + e + 4) : make_uint4(0, 0, 0, 0);
      }
    }
  }
}

// Converts quarters [Q0, Q1) of a thread's tile registers to fp16 (hi, and lo for fp32 inputs) and writes them
// transposed into LDS: element (channel c, token n) of part `part` lives at lds[(part * 256 + c) * kPfRS + n].
// bf16: a quarter = 4 channels of one item, each written as 4 adjacent tokens (8 bytes); fp32: a quarter = one
// item, each channel written as a token pair (4 bytes per part).
template <bool BF16, int Q0 = 0, int Q1 = 4>
__device__ __forceinline__ void store_tile(const TileRegs<BF16>& r, _Float16* __restrict__ buf, int tid) {
  if constexpr (BF16) {
    const int p = tid & 15;
#pragma unroll
    for (int qd = Q0; qd < Q1; ++qd) {
      const int it = qd >> 1;
      const int q = (tid >> 4) + 16 * it;
#pragma unroll
      for (int j = (qd & 1) * 4; j < (qd & 1) * 4 + 4; ++j) {
        float x[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint4 a = r.v[it * 4 + t];
          const uint32_t w = (&a.x)[j >> 1];
          x[t] = __uint_as_float((j & 1) ? (w & 0xffff0000u) : (w << 16));
        }
        const int c = q * 8 + j;
        *(uint2*)(buf + c * kPfRS + 4 * p) = make_uint2(pack_rtz(x[0], x[1]), pack_rtz(x[2], x[3]));
      }
    }
  } else {
    const int p = tid & 31;
#pragma unroll
    for (int it = Q0; it < Q1; ++it) {
      const int q = (tid >> 5) + 8 * it;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint4 a = r.v[(it * 2) * 2 + (j >> 2)], b = r.v[(it * 2 + 1) * 2 + (j >> 2)];
        const float x0 = __uint_as_float((&a.x)[j & 3]);
        const float x1 = __uint_as_float((&b.x)[j & 3]);
        const int c = q * 8 + j;
        const uint32_t hi = pack_rtz(x0, x1);
        *(uint32_t*)(buf + c * kPfRS + 2 * p) = hi;
        const uint32_t lo = pack_rtz(x0 - half_lo_f32(hi), x1 - half_hi_f32(hi));
        *(uint32_t*)(buf + (kPfCh + c) * kPfRS + 2 * p) = lo;
      }
    }
  }
}

// Basis operands of one MFMA k-step for this lane's bin: hi / lo fp16 halves of cos and -sin.
struct BasisRegs {
  half8 ch, cl, sh, sl;
};

// base = exp(-j theta) at the first of this lane's 8 tokens; tw[i] = exp(-j 2 pi k i / M).
__device__ __forceinline__ BasisRegs make_basis(float2 base, const float2 (&tw)[8]) {
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
  BasisRegs r;
  r.ch = __builtin_bit_cast(half8, ch);
  r.cl = __builtin_bit_cast(half8, cl);
  r.sh = __builtin_bit_cast(half8, sh);
  r.sl = __builtin_bit_cast(half8, sl);
  return r;
}

// grid: 8 * per_xcd workgroups; id -> (id % 8) * per_xcd + id / 8 so that workgroups that run on
// the same XCD at the same time are the bin tiles of the same slice and share its K/V tile in L2.
// FULL: M is a power of two and a multiple of the 64-token tile: no bounds checks in the token
// loop and phases reduce with a mask.
// The token loop is software-pipelined by hand: the basis registers and the LDS operands of k-step
// s+1 are produced while the 32 MFMAs of k-step s are in flight, and the loop body is one basic
// block so that the scheduler can interleave the two instruction streams.  (Explicit
// sched_group_barrier patterns were measured and were 5-40 % slower than the default schedule.
// A single wave overlaps vector-ALU work with its own MFMAs only partly: ~2 clocks per VALU
// instruction up to ~6 per MFMA, 4 clocks beyond.  Beyond that the matrix cores are power-limited on
// this instruction: back to back from registers they sustain 2.4-2.5 PFLOP/s on zero operands and
// 1.6-1.7 on random ones.)
template <bool BF16, bool FULL>
__global__ __launch_bounds__(kPfThreads) void prefill_mfma_kernel(Params P, const void* __restrict__ K,
                                                                 const void* __restrict__ V, int nt,
                                                                 int per_xcd, int total) {
  extern __shared__ _Float16 lds[];
  constexpr int kParts = BF16 ? 1 : 2;
  constexpr int kBufHalves = kParts * kPfCh * kPfRS;
  constexpr int kSteps = kPfTok / 16;

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

  // a slice holds S sink + M transformed + R recent tokens; the transform starts after the sinks
  const int64_t slice_base = ((int64_t)slice * ((int64_t)P.S + M + P.R) + P.S) * kHeadDim;
  const uint32_t n_tiles = (M + kPfTok - 1) / kPfTok;
  const int a_off = (lane & 31) * kPfRS + 8 * g;  // this lane's row / token group inside a channel block
  TileRegs<BF16> regs;
  load_tile<BF16, FULL>(regs, K, V, slice_base, 0, M, tid);
  store_tile<BF16>(regs, lds, tid);
  __syncthreads();

  // operands of k-step 0 of tile 0
  float2 base;
  {
    const float2 c = cis(mulmod(k, (uint32_t)(8 * g), M, Mmask), M);
    base = make_float2(c.x, -c.y);
  }
  BasisRegs bc = make_basis(base, tw);
  half8 ac[kPfBlk], acl[BF16 ? 1 : kPfBlk];
#pragma unroll
  for (int b = 0; b < kPfBlk; ++b) {
    ac[b] = *(const half8*)(lds + b * 32 * kPfRS + a_off);
    if constexpr (!BF16) acl[b] = *(const half8*)(lds + (kPfCh + b * 32) * kPfRS + a_off);
  }

  // One 64-token tile: loads tile t_load into rl, converts rs (the tile after t) into the other LDS buffer,
  // and runs the MFMAs of tile t.
  auto tile_body = [&](uint32_t t, uint32_t t_load, TileRegs<BF16>& rl, TileRegs<BF16>& rs) __attribute__((always_inline)) {
    const _Float16* cur = lds + (t & 1) * kBufHalves;
    _Float16* nxt = lds + ((t + 1) & 1) * kBufHalves;
    load_tile<BF16, FULL>(rl, K, V, slice_base, t_load * kPfTok, M, tid);

#pragma unroll
    for (int st = 0; st < kSteps; ++st) {
      // ---- produce the operands of the next k-step --------------------------------------------
      BasisRegs bn;
      half8 an[kPfBlk], anl[BF16 ? 1 : kPfBlk];
      if (st + 1 < kSteps) {
        base = cmul(base, r16);
        bn = make_basis(base, tw);
#pragma unroll
        for (int b = 0; b < kPfBlk; ++b) {
          an[b] = *(const half8*)(cur + b * 32 * kPfRS + a_off + 16 * (st + 1));
          if constexpr (!BF16) anl[b] = *(const half8*)(cur + (kPfCh + b * 32) * kPfRS + a_off + 16 * (st + 1));
        }
      } else {
        // exact basis phase at the first token this lane feeds in the next tile
        const uint32_t nn = (t + 1) * kPfTok + 8 * g;
        const float2 c = FULL ? cis_poly2((k * nn) & (M - 1u), M) : cis_poly(mulmod(k, nn, M, Mmask), M);
        base = make_float2(c.x, -c.y);
        bn = make_basis(base, tw);
      }
      if (st == kSteps - 2) store_tile<BF16, 0, 2>(rs, nxt, tid);
      if (st == kSteps - 1) store_tile<BF16, 2, 4>(rs, nxt, tid);

      // ---- 32 (48 for fp32 inputs) MFMAs of this k-step ---------------------------------------
#pragma unroll
      for (int b = 0; b < kPfBlk; ++b) acc_re[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ac[b], bc.ch, acc_re[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < kPfBlk; ++b) acc_im[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ac[b], bc.sh, acc_im[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < kPfBlk; ++b) acc_re[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ac[b], bc.cl, acc_re[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < kPfBlk; ++b) acc_im[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ac[b], bc.sl, acc_im[b], 0, 0, 0);
      if constexpr (!BF16) {
#pragma unroll
        for (int b = 0; b < kPfBlk; ++b) {
          acc_re[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(acl[b], bc.ch, acc_re[b], 0, 0, 0);
          acc_im[b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(acl[b], bc.sh, acc_im[b], 0, 0, 0);
        }
      }
      bc = bn;
      if (st + 1 < kSteps) {
#pragma unroll
        for (int b = 0; b < kPfBlk; ++b) {
          ac[b] = an[b];
          if constexpr (!BF16) acl[b] = anl[b];
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < kPfBlk; ++b) {  // k-step 0 of the next tile
      ac[b] = *(const half8*)(nxt + b * 32 * kPfRS + a_off);
      if constexpr (!BF16) acl[b] = *(const half8*)(nxt + (kPfCh + b * 32) * kPfRS + a_off);
    }
  };
  // Tiles beyond the last one are harmless reloads of the last tile (keeps the body branch-free).
  const uint32_t last = n_tiles - 1;
  if constexpr (BF16) {
    // Two register sets: the global loads of a tile are issued two tiles before its MFMAs and one full tile
    // before its conversion, so their latency never sits on the matrix pipe's path.
    TileRegs<BF16> regs1;
    load_tile<BF16, FULL>(regs1, K, V, slice_base, (last < 1u ? last : 1u) * kPfTok, M, tid);
    uint32_t t = 0;
    for (; t + 1 < n_tiles; t += 2) {
      tile_body(t, t + 2 < last ? t + 2 : last, regs, regs1);
      tile_body(t + 1, t + 3 < last ? t + 3 : last, regs1, regs);
    }
    if (t < n_tiles) tile_body(t, last, regs, regs1);
  } else {
    for (uint32_t t = 0; t < n_tiles; ++t) tile_body(t, t + 1 < last ? t + 1 : last, regs, regs);
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

// Copies the exact tokens of a prefill (Sec. 4.2.1: the first S and the last R of every slice are
// not transformed) into the sink store and the recent ring (ring slot j = j-th oldest).
// grid: slice ; z: tensor.  One 16-byte chunk per thread and step.
template <bool BF16>
__global__ __launch_bounds__(256) void prefill_edges_kernel(Params P, const void* __restrict__ K,
                                                           const void* __restrict__ V) {
  constexpr int kElem = BF16 ? 2 : 4;
  constexpr int kRowChunks = kHeadDim * kElem / 16;  // 16-byte chunks per token row
  const int slice = blockIdx.x;
  const int tensor = blockIdx.y;
  const int64_t N = (int64_t)P.S + P.M + P.R;
  const uint4* src = (const uint4*)(tensor ? V : K) + (int64_t)slice * N * kRowChunks;
  uint4* sink = (uint4*)(tensor ? P.sinkV : P.sinkK) + (int64_t)slice * P.S * kRowChunks;
  uint4* ring = (uint4*)(tensor ? P.ringV : P.ringK) + (int64_t)slice * P.R * kRowChunks;
  for (int e = threadIdx.x; e < P.S * kRowChunks; e += 256) sink[e] = src[e];
  const uint4* tail = src + ((int64_t)P.S + P.M) * kRowChunks;
  for (int e = threadIdx.x; e < P.R * kRowChunks; e += 256) ring[e] = tail[e];
}

hipError_t launch_prefill_edges(const Params& P, const void* K, const void* V, hipStream_t st) {
  if (P.S + P.R == 0) return hipSuccess;
  if (P.kv_dtype == 1) prefill_edges_kernel<true><<<dim3((uint32_t)P.n_slices, 2), dim3(256), 0, st>>>(P, K, V);
  else prefill_edges_kernel<false><<<dim3((uint32_t)P.n_slices, 2), dim3(256), 0, st>>>(P, K, V);
  return hipGetLastError();
}

hipError_t launch_prefill(const Params& P, const void* K, const void* V, hipStream_t st) {
  {
    hipError_t e = launch_prefill_edges(P, K, V, st);
    if (e != hipSuccess) return e;
  }
  const int nt = (P.max_nb + kPfBins - 1) / kPfBins;
  const uint64_t total = (uint64_t)P.n_slices * nt;
  if (total > 0x3fffffffull) return hipErrorInvalidConfiguration;
  const int per_xcd = (int)((total + 7) / 8);
  const bool bf16 = P.kv_dtype == 1;
  const size_t lds = sizeof(_Float16) * 2 * (bf16 ? 1 : 2) * kPfCh * kPfRS;
  {
    static LdsLimit lim[4];
    const int lds16 = (int)(sizeof(_Float16) * 2 * kPfCh * kPfRS), lds32 = 2 * lds16;
    hipError_t e = lim[0].ensure((const void*)prefill_mfma_kernel<true, true>, lds16);
    if (e == hipSuccess) e = lim[1].ensure((const void*)prefill_mfma_kernel<true, false>, lds16);
    if (e == hipSuccess) e = lim[2].ensure((const void*)prefill_mfma_kernel<false, true>, lds32);
    if (e == hipSuccess) e = lim[3].ensure((const void*)prefill_mfma_kernel<false, false>, lds32);
    if (e != hipSuccess) return e;
  }
  const dim3 grid((uint32_t)(per_xcd * 8)), block(kPfThreads);
  const bool full = (P.M % kPfTok) == 0 && P.Mmask != 0;
  if (bf16 && full) prefill_mfma_kernel<true, true><<<grid, block, lds, st>>>(P, K, V, nt, per_xcd, (int)total);
  else if (bf16) prefill_mfma_kernel<true, false><<<grid, block, lds, st>>>(P, K, V, nt, per_xcd, (int)total);
  else if (full) prefill_mfma_kernel<false, true><<<grid, block, lds, st>>>(P, K, V, nt, per_xcd, (int)total);
  else prefill_mfma_kernel<false, false><<<grid, block, lds, st>>>(P, K, V, nt, per_xcd, (int)total);
  return hipGetLastError();
}

}  // namespace iwdft
