// Streaming IWDFT update (Sec. 4.1 Eq. infi-dft; Sec. 4.2.2 Eq. update-iwdft) and the
// read-out of the paper-convention coefficients S_T.
//
// The update is a pure read-modify-write over every stored coefficient: 8 B read + 8 B
// written per coefficient per token, ~4 flops -- HBM-bound.  Lanes run along the bin axis
// (the contiguous one), so a lane's twiddle exp(+j 2 pi k (T-M)/M) is computed once, exactly
// (integer phase reduction, then sincospi), and reused for all the channels it walks over.
#include "common.h"

namespace iwdft {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kAppendThreads = 256;
constexpr int kAppendBinsPerBlock = kAppendThreads * 2;  // two bins (one 16-byte access) per lane

// grid: ((slice * chunks + chunk) * dsplit + ds) * 2 + tensor
template <bool BF16, int DROWS>
__global__ __launch_bounds__(kAppendThreads) void append_kernel(Params P, const void* __restrict__ tok_k,
                                                               const void* __restrict__ tok_v,
                                                               uint32_t tsh, int chunks,
                                                               int64_t x_slice_stride) {
  constexpr int dsplit = kHeadDim / DROWS;
  uint32_t bid = blockIdx.x;
  const int tensor = bid & 1;
  bid >>= 1;
  const int ds = bid % dsplit;
  bid /= dsplit;
  const int chunk = bid % chunks;
  const int slice = bid / chunks;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const int i0 = chunk * kAppendBinsPerBlock + threadIdx.x * 2;
  if (i0 >= L.nb) return;  // padding entries are never touched and stay zero

  const uint32_t k0 = (uint32_t)P.bins[L.bin_off + i0];
  const bool has1 = (i0 + 1) < L.nb;
  const uint32_t k1 = has1 ? (uint32_t)P.bins[L.bin_off + i0 + 1] : 0u;
  const float2 w0 = cis(mulmod(k0, tsh, P.M, P.Mmask), P.M);
  float2 w1 = cis(mulmod(k1, tsh, P.M, P.Mmask), P.M);
  if (!has1) w1 = make_float2(0.f, 0.f);

  const void* tok = tensor ? tok_v : tok_k;
  float2* F = tensor ? P.FV : P.FK;
  const int d0 = ds * DROWS;
  v4f* row = (v4f*)(F + L.coef_off + ((int64_t)s * kHeadDim + d0) * L.Bp + i0);
  const int64_t stride = L.Bp / 2;  // in 16-byte units
  const int64_t xbase = (int64_t)slice * x_slice_stride + d0;

  // All rows of the block in one pass: every load is issued before the first store (a loop over groups of rows
  // drains the memory pipeline of the wave between its iterations; measured on 1638 / 2048 / 4096-bin rows:
  // 16 rows x one pass 72 / 79 / 81 % of the HBM peak, 32 rows in 4 passes of 8: 67 / 75 / 77 %).
  constexpr int U = DROWS;
#pragma unroll 1
  for (int dd = 0; dd < DROWS; dd += U) {
    v4f f[U];
    float x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) f[u] = __builtin_nontemporal_load(row + (dd + u) * stride);
#pragma unroll
    for (int u = 0; u < U; ++u) x[u] = load_kv<BF16>(tok, xbase + dd + u) * P.x_scale;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      f[u].x += x[u] * w0.x;
      f[u].y += x[u] * w0.y;
      f[u].z += x[u] * w1.x;
      f[u].w += x[u] * w1.y;
      __builtin_nontemporal_store(f[u], row + (dd + u) * stride);
    }
  }
}

// Recent window: after the coefficients absorbed the oldest ring token, the new token takes its slot.
// grid: slice ; z: tensor; 128 threads = channels.
template <bool BF16>
__global__ __launch_bounds__(kHeadDim) void ring_push_kernel(Params P, const void* __restrict__ tok_k,
                                                            const void* __restrict__ tok_v, uint32_t pos) {
  const int slice = blockIdx.x;
  const void* tok = blockIdx.y ? tok_v : tok_k;
  void* ring = blockIdx.y ? P.ringV : P.ringK;
  const int64_t src = (int64_t)slice * kHeadDim + threadIdx.x;
  const int64_t dst = ((int64_t)slice * P.R + pos) * kHeadDim + threadIdx.x;
  if constexpr (BF16) ((uint16_t*)ring)[dst] = ((const uint16_t*)tok)[src];
  else ((float*)ring)[dst] = ((const float*)tok)[src];
}

hipError_t launch_absorb(const Params& P, const void* xk, const void* xv, int64_t x_stride, uint32_t tsh,
                         hipStream_t st) {
  constexpr int DROWS = 16;
  const int chunks = (P.max_nb + kAppendBinsPerBlock - 1) / kAppendBinsPerBlock;
  const uint64_t blocks = (uint64_t)P.n_slices * chunks * (kHeadDim / DROWS) * 2;
  if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
  if (P.kv_dtype == 1)
    append_kernel<true, DROWS><<<dim3((uint32_t)blocks), dim3(kAppendThreads), 0, st>>>(P, xk, xv, tsh, chunks, x_stride);
  else
    append_kernel<false, DROWS><<<dim3((uint32_t)blocks), dim3(kAppendThreads), 0, st>>>(P, xk, xv, tsh, chunks, x_stride);
  return hipGetLastError();
}

hipError_t launch_append(const Params& P, const void* tok_k, const void* tok_v, uint32_t tsh,
                         uint32_t ring_pos, hipStream_t st) {
  // What is absorbed: the new token (R == 0) or the token ageing out of the recent window.
  const int esz = P.kv_dtype == 1 ? 2 : 4;
  const void* xk = tok_k;
  const void* xv = tok_v;
  int64_t x_stride = kHeadDim;
  if (P.R > 0) {
    xk = (const char*)P.ringK + (size_t)ring_pos * kHeadDim * esz;
    xv = (const char*)P.ringV + (size_t)ring_pos * kHeadDim * esz;
    x_stride = (int64_t)P.R * kHeadDim;
  }
  hipError_t e = launch_absorb(P, xk, xv, x_stride, tsh, st);
  if (e != hipSuccess || P.R == 0) return e;
  if (P.kv_dtype == 1) ring_push_kernel<true><<<dim3((uint32_t)P.n_slices, 2), dim3(kHeadDim), 0, st>>>(P, tok_k, tok_v, ring_pos);
  else ring_push_kernel<false><<<dim3((uint32_t)P.n_slices, 2), dim3(kHeadDim), 0, st>>>(P, tok_k, tok_v, ring_pos);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Export: S_T[k] = exp(-j 2 pi k (T-M)/M) * F_T[k] / T, written [slice][bin][channel][re,im].
// grid: (slice_in_layer * tiles + tile) * 2 + tensor ; one block transposes 32 bins x 128 channels.
__global__ __launch_bounds__(256) void export_kernel(Params P, int layer, float* __restrict__ SK,
                                                    float* __restrict__ SV, uint32_t tsh, float inv_T,
                                                    int tiles) {
  __shared__ float2 tile[kHeadDim][33];
  uint32_t bid = blockIdx.x;
  const int tensor = bid & 1;
  bid >>= 1;
  const int t = bid % tiles;
  const int s = bid / tiles;
  float* out = tensor ? SV : SK;
  if (!out) return;
  const LayerInfo L = P.layers[layer];
  const float2* F = (tensor ? P.FV : P.FK) + L.coef_off + (int64_t)s * kHeadDim * L.Bp;
  const int i = t * 32 + (threadIdx.x & 31);
  float2 w = make_float2(0.f, 0.f);
  if (i < L.nb) {
    uint32_t k = (uint32_t)P.bins[L.bin_off + i];
    float2 c = cis(mulmod(k, tsh, P.M, P.Mmask), P.M);
    w = make_float2(c.x * inv_T, -c.y * inv_T);  // conj: exp(-j ...)
  }
  for (int d = threadIdx.x >> 5; d < kHeadDim; d += 8) {
    float2 f = (i < L.nb) ? F[(int64_t)d * L.Bp + i] : make_float2(0.f, 0.f);
    tile[d][threadIdx.x & 31] = cmul(f, w);
  }
  __syncthreads();
  const int d = threadIdx.x & 127;
  for (int ii = threadIdx.x >> 7; ii < 32; ii += 2) {
    int io = t * 32 + ii;
    if (io < L.nb) ((float2*)out)[((int64_t)s * L.nb + io) * kHeadDim + d] = tile[d][ii];
  }
}

hipError_t launch_export(const Params& P, int layer, float* SK, float* SV, uint32_t tsh, float inv_T,
                         hipStream_t st) {
  // tiles from the host copy of the geometry is not available here; max_Bp bounds every layer.
  const int tiles = P.max_Bp / 32;
  const uint64_t blocks = (uint64_t)P.batch * P.n_kv * tiles * 2;
  if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
  export_kernel<<<dim3((uint32_t)blocks), dim3(256), 0, st>>>(P, layer, SK, SV, tsh, inv_T, tiles);
  return hipGetLastError();
}

}  // namespace iwdft
