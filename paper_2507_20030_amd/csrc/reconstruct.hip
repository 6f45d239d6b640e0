// Materialising reconstruction (Sec. 3.1.2 Eq. inverse-swdft over the kept bins; Sec. 4.2.2
// Eq. reconstruct-idft): x~[a] = (1/M) Re sum_k w_k U_T[k] exp(+j 2 pi k a / M).
// With the fixed-frame storage U_T[k] = exp(-j 2 pi k t/M) F_T[k], t = (T-M) mod M, so the
// sum runs over F_T with the slot index shifted by t.  This is the sparse inverse DFT written
// as a tiled contraction [slots x bins] * [bins x channels]; decode attention never calls it
// (it consumes the coefficients directly), it exists to inspect / verify the state.
#include "common.h"

namespace iwdft {

constexpr int kRecSlots = 64;  // slots per block
constexpr int kRecBins = 32;   // bins per LDS tile

// grid: ((s * atiles) + atile) * 2 + tensor ; 256 threads, each 4 channels x 8 slots.
template <bool BF16>
__global__ __launch_bounds__(256) void reconstruct_kernel(Params P, int layer, uint32_t a0,
                                                         uint32_t n_slots, void* __restrict__ Kt,
                                                         void* __restrict__ Vt, uint32_t tsh, int atiles) {
  __shared__ float2 Fs[kRecBins][kHeadDim + 1];
  __shared__ float2 Tw[kRecBins][kRecSlots];
  uint32_t bid = blockIdx.x;
  const int tensor = bid & 1;
  bid >>= 1;
  const int at = bid % atiles;
  const int s = bid / atiles;
  void* out = tensor ? Vt : Kt;
  if (!out) return;
  const LayerInfo L = P.layers[layer];
  const float2* F = (tensor ? P.FV : P.FK) + L.coef_off + (int64_t)s * kHeadDim * L.Bp;
  const float inv_M = 1.0f / (float)P.M;
  const int tid = threadIdx.x;
  const int td = tid & 31, ta = tid >> 5;

  float acc[8][4];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[a][c] = 0.f;

  for (int i0 = 0; i0 < L.nb; i0 += kRecBins) {
    __syncthreads();
    {  // coefficient tile, pre-multiplied by w_k / M
      const int i = i0 + (tid & 31);
      const float w = (i < L.nb) ? P.weights[L.bin_off + i] * inv_M : 0.f;
      for (int d = tid >> 5; d < kHeadDim; d += 8) {
        float2 f = (i < L.nb) ? F[(int64_t)d * L.Bp + i] : make_float2(0.f, 0.f);
        Fs[tid & 31][d] = make_float2(f.x * w, f.y * w);
      }
    }
    for (int e = tid; e < kRecBins * kRecSlots; e += 256) {  // twiddle tile
      const int i = i0 + e / kRecSlots, a = e % kRecSlots;
      float2 w = make_float2(0.f, 0.f);
      const uint32_t slot = a0 + at * kRecSlots + a;
      if (i < L.nb && slot < a0 + n_slots) {
        const uint32_t k = (uint32_t)P.bins[L.bin_off + i];
        const uint32_t sh = (slot % P.M + P.M - tsh) % P.M;  // (slot - t) mod M
        w = cis(mulmod(k, sh, P.M, P.Mmask), P.M);
      }
      Tw[e / kRecSlots][a] = w;
    }
    __syncthreads();
#pragma unroll 4
    for (int i = 0; i < kRecBins; ++i) {
      float2 f[4], w[8];
#pragma unroll
      for (int c = 0; c < 4; ++c) f[c] = Fs[i][td * 4 + c];
#pragma unroll
      for (int a = 0; a < 8; ++a) w[a] = Tw[i][ta * 8 + a];
#pragma unroll
      for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[a][c] += f[c].x * w[a].x - f[c].y * w[a].y;
    }
  }
#pragma unroll
  for (int a = 0; a < 8; ++a) {
    const uint32_t rel = at * kRecSlots + ta * 8 + a;
    if (rel < n_slots) {
      const int64_t o = ((int64_t)s * n_slots + rel) * kHeadDim + td * 4;
#pragma unroll
      for (int c = 0; c < 4; ++c) store_kv<BF16>(out, o + c, acc[a][c]);
    }
  }
}

hipError_t launch_reconstruct(const Params& P, int layer, uint32_t a0, uint32_t n_slots, void* Kt,
                              void* Vt, uint32_t tsh, hipStream_t st) {
  const int atiles = (int)((n_slots + kRecSlots - 1) / kRecSlots);
  const uint64_t blocks = (uint64_t)P.batch * P.n_kv * atiles * 2;
  if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
  if (P.kv_dtype == 1)
    reconstruct_kernel<true><<<dim3((uint32_t)blocks), dim3(256), 0, st>>>(P, layer, a0, n_slots, Kt, Vt, tsh, atiles);
  else
    reconstruct_kernel<false><<<dim3((uint32_t)blocks), dim3(256), 0, st>>>(P, layer, a0, n_slots, Kt, Vt, tsh, atiles);
  return hipGetLastError();
}

}  // namespace iwdft
