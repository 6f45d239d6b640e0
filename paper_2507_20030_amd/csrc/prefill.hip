// Prefill transform (Sec. 3.1.2 Eq. dft-full at the kept bins; Sec. 4.2.1 Eq. prefill-dft):
// F_M[k] = U_M[k] = sum_{n<M} x[n] exp(-j 2 pi k n / M) for every slice, channel and kept bin.
#include "common.h"

namespace iwdft {

// Plain evaluation of the sums, one thread per (bin, channel).  grid: slice * tiles + tile, z: tensor.
template <bool BF16>
__global__ __launch_bounds__(256) void prefill_plain_kernel(Params P, const void* __restrict__ K,
                                                           const void* __restrict__ V, int tiles) {
  const int tensor = blockIdx.y;
  const int tile = blockIdx.x % tiles;
  const int slice = blockIdx.x / tiles;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const int i = tile * 2 + (threadIdx.x >> 7);
  const int d = threadIdx.x & 127;
  if (i >= L.nb) return;
  const uint32_t k = (uint32_t)P.bins[L.bin_off + i];
  const void* X = tensor ? V : K;
  const int64_t xb = (int64_t)slice * P.M * kHeadDim + d;
  float re = 0.f, im = 0.f;
  uint32_t ph = 0;  // (k * n) mod M, advanced incrementally
  for (uint32_t n = 0; n < P.M; ++n) {
    const float x = load_kv<BF16>(X, xb + (int64_t)n * kHeadDim);
    const float2 w = cis(ph, P.M);
    re += x * w.x;
    im -= x * w.y;
    ph += k;
    if (ph >= P.M) ph -= P.M;
  }
  float2* F = (tensor ? P.FV : P.FK) + L.coef_off + ((int64_t)s * kHeadDim + d) * L.Bp + i;
  *F = make_float2(re, im);
}

hipError_t launch_prefill(const Params& P, const void* K, const void* V, hipStream_t st) {
  const int tiles = (P.max_nb + 1) / 2;
  const uint64_t blocks = (uint64_t)P.n_slices * tiles;
  if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
  if (P.kv_dtype == 1)
    prefill_plain_kernel<true><<<dim3((uint32_t)blocks, 2), dim3(256), 0, st>>>(P, K, V, tiles);
  else
    prefill_plain_kernel<false><<<dim3((uint32_t)blocks, 2), dim3(256), 0, st>>>(P, K, V, tiles);
  return hipGetLastError();
}

}  // namespace iwdft
