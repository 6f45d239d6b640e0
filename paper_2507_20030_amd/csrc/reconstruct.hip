// Materialising reconstruction (Sec. 3.1.2 Eq. inverse-swdft over the kept bins; Sec. 4.2.2
// Eq. reconstruct-idft): x~[a] = (1/M) Re sum_k w_k U_T[k] exp(+j 2 pi k a / M).
// With the fixed-frame storage U_T[k] = exp(-j 2 pi k t/M) F_T[k], t = (T-M) mod M, so the
// sum runs over F_T with the slot index shifted by t.  This is the sparse inverse DFT written
// as a tiled contraction [slots x bins] * [bins x channels]; decode attention never calls it
// (it consumes the coefficients directly), it exists to inspect / verify the state.
//
// Two kernels: the tiled direct contraction (any M, any slot range) and, for power-of-two M and long
// ranges, in-LDS inverse FFTs (reconstruct_fft_kernel below).
#include "common.h"
#include "fft_lds.h"

namespace iwdft {

constexpr int kRecSlots = 64;  // slots per block
constexpr int kRecBins = 32;   // bins per LDS tile

// grid: ((s * atiles) + atile) * 2 + tensor ; 256 threads, each 4 channels x 8 slots.
template <bool BF16>
__global__ __launch_bounds__(256) void reconstruct_kernel(Params P, int layer, uint32_t a0, uint32_t stride,
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
  const float inv_M = P.gain / (float)P.M;
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
      const uint32_t rel = at * kRecSlots + a;            // output row; its slot is a0 + stride * rel < M
      const uint32_t slot = a0 + stride * rel;
      if (i < L.nb && rel < n_slots) {
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

// All M slots of two adjacent channels of one slice per workgroup: the kept coefficients (times w_k / (2M))
// go to bin k and, conjugated, to bin M - k of an LDS spectrum -- channel c0 as it is, channel c1 times j,
// so that after the inverse transform the real part is channel c0 and the imaginary part channel c1 --
// folded modulo Q = min(M, 8192) with the collision rounds the attention kernel uses (Params::fold).
// M > Q: block b of the token axis, slots Pb a + b, comes from the spectrum with bin k turned by
// e^{j 2 pi k b / M}.  Rows go out rotated by the slot shift (T - M) mod M; slots outside [a0, a0 + n_slots)
// are skipped.  Block ids are dealt so that the 64 workgroups of a (slice, tensor) share one XCD's L2 and
// their 4-byte pieces of each 256-byte output row merge there.
template <int LOGQ, bool BF16, bool MULTI>
__global__ __launch_bounds__(kFftThreads, 4) void reconstruct_fft_kernel(Params P, int layer, uint32_t a0,
                                                                        uint32_t n_slots, void* __restrict__ Kt,
                                                                        void* __restrict__ Vt, uint32_t tsh,
                                                                        int per_xcd, int n_st) {
  extern __shared__ float2 smem[];
  constexpr int Q = 1 << LOGQ;
  constexpr int kElem = BF16 ? 2 : 4;
  constexpr int kRow = kHeadDim * kElem;
  constexpr int kPairs = kHeadDim / 2;
  float2* buf = smem;
  float2* tab = smem + Q + (Q >> 5);
  const int tid = threadIdx.x;
  const uint32_t idx = blockIdx.x >> 3;
  const uint32_t stn = (blockIdx.x & 7u) * (uint32_t)per_xcd + idx / kPairs;
  if (stn >= (uint32_t)n_st) return;
  const int pair = idx % kPairs;
  const int tensor = stn & 1;
  const int s = stn >> 1;  // slice within the layer
  char* out = (char*)(tensor ? Vt : Kt);
  if (!out) return;
  const LayerInfo L = P.layers[layer];
  const float2* F0 = (tensor ? P.FV : P.FK) + L.coef_off + ((int64_t)s * kHeadDim + pair * 2) * L.Bp;
  const float2* F1 = F0 + L.Bp;
  const int32_t* bins = P.bins + L.bin_off;
  const float* wts = P.weights + L.bin_off;
  const uint16_t* fold = P.fold + L.bin_off;
  const uint32_t Pb = MULTI ? (P.M >> LOGQ) : 1u;
  const float gain = 0.5f * P.gain / (float)P.M;
  char* orow = out + (int64_t)s * n_slots * kRow + pair * 2 * kElem;

  for (int m = tid; m <= (Q >> 3); m += kFftThreads) tab[m] = P.tw8[m];  // exp(+j 2 pi m / Q), host-made

  for (uint32_t b = 0; b < Pb; ++b) {
    int lt = tid;
    if (MULTI) asm volatile("" : "+v"(lt));  // keeps the passes' address arithmetic out of long-lived registers
    for (int e = tid; e < Q + (Q >> 5); e += kFftThreads) buf[e] = make_float2(0.f, 0.f);
    __syncthreads();
    for (int round = 0; round < L.fold_rounds; ++round) {
#pragma unroll
      for (int j = 0; j < kFftNBT; ++j) {
        const int i = j * kFftThreads + tid;
        if (i < L.nb) {
          const uint32_t k = (uint32_t)bins[i];
          const uint32_t fr = fold[i];
          const float w = wts[i] * gain;
          float2 tw = make_float2(1.f, 0.f);
          if (MULTI) tw = cis_poly2((k * b) & (P.M - 1u), P.M);
          const float2 f0 = F0[i], f1 = F1[i];
          const float2 z0 = cmul(make_float2(f0.x * w, f0.y * w), tw);
          const float2 z1 = cmul(make_float2(f1.x * w, f1.y * w), tw);
          const int r = k & (Q - 1), rm = (Q - r) & (Q - 1);
          if ((fr & 0xffu) == (uint32_t)round) {  //      z0  + j z1
            float2 v = make_float2(z0.x - z1.y, z0.y + z1.x);
            if (r == rm) v = make_float2(2.f * z0.x, 2.f * z1.x);  // ... plus the mirror term, same slot
            if (round) v = cadd(v, buf[pad(r)]);
            buf[pad(r)] = v;
          }
          if ((fr >> 8) == (uint32_t)round) {     // conj z0  + j conj z1
            float2 v = make_float2(z0.x + z1.y, z1.x - z0.y);
            if (round) v = cadd(v, buf[pad(rm)]);
            buf[pad(rm)] = v;
          }
        }
      }
      __syncthreads();
    }
    ifft_dif<LOGQ>(buf, tab, lt);
    constexpr int H = (LOGQ & 1) ? Q / 2 : Q;
    constexpr int IT = (H + kFftThreads - 1) / kFftThreads;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int a = it * kFftThreads + tid;
      if (H % kFftThreads == 0 || a < H) {
        const int p = digit_pos<LOGQ>(a);
        float2 y0 = buf[pad(p)], y1 = y0;
        if (LOGQ & 1) {
          const float2 c = buf[pad(p + 1)];
          y1 = csub(y0, c);
          y0 = cadd(y0, c);
        }
#pragma unroll
        for (int h = 0; h < ((LOGQ & 1) ? 2 : 1); ++h) {
          const uint32_t ap = (uint32_t)(a + h * H) * Pb + b;      // index of the un-shifted transform
          const uint32_t slot = (ap + tsh) & (P.M - 1u);          // where it sits after T - M appends
          const uint32_t rel = slot - a0;                          // wraps for slot < a0
          if (rel < n_slots) store_pair<BF16>(orow + (int64_t)rel * kRow, h ? y1 : y0);
        }
      }
    }
    if (MULTI) __syncthreads();
  }
}

bool reconstruct_fft_ok(const Params& P) {
  return P.Mmask != 0 && P.M >= 256 && P.max_nb <= kFftNBT * kFftThreads;
}

template <bool BF16>
static hipError_t launch_reconstruct_fft_t(const Params& P, int layer, uint32_t a0, uint32_t n_slots, void* Kt,
                                           void* Vt, uint32_t tsh, hipStream_t st) {
  int logM = 0;
  while ((1u << logM) < P.M) ++logM;
  const int logQ = logM < kFftMaxLogQ ? logM : kFftMaxLogQ;
  const int n_st = P.batch * P.n_kv * 2;
  const int per_xcd = (n_st + 7) / 8;
  const uint64_t blocks = (uint64_t)per_xcd * (kHeadDim / 2) * 8;
  if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
  const size_t lds = sizeof(float2) * (size_t)fft_lds_float2(logQ);
  hipError_t e = hipSuccess;
#define IWDFT_RC_CASE(LQ, MULTI)                                                                        \
  {                                                                                                     \
    static LdsLimit lim;                                                                                \
    e = lim.ensure((const void*)reconstruct_fft_kernel<LQ, BF16, MULTI>, (int)lds);                     \
    if (e != hipSuccess) return e;                                                                      \
    reconstruct_fft_kernel<LQ, BF16, MULTI><<<dim3((uint32_t)blocks), dim3(kFftThreads), lds, st>>>(    \
        P, layer, a0, n_slots, Kt, Vt, tsh, per_xcd, n_st);                                             \
  }
  if (logM > logQ) IWDFT_RC_CASE(kFftMaxLogQ, true)
  else switch (logQ) {
    case 8: IWDFT_RC_CASE(8, false) break;
    case 9: IWDFT_RC_CASE(9, false) break;
    case 10: IWDFT_RC_CASE(10, false) break;
    case 11: IWDFT_RC_CASE(11, false) break;
    case 12: IWDFT_RC_CASE(12, false) break;
    default: IWDFT_RC_CASE(13, false) break;
  }
#undef IWDFT_RC_CASE
  return hipGetLastError();
}

// use_fft: the caller knows the layer's fold schedule is valid (the attention path uses FFTs too).
hipError_t launch_reconstruct(const Params& P, int layer, uint32_t a0, uint32_t stride, uint32_t n_slots, void* Kt,
                              void* Vt, uint32_t tsh, bool use_fft, hipStream_t st) {
  // The transform produces all M slots; the direct contraction costs O(|B|) per requested slot.
  if (stride == 1 && use_fft && reconstruct_fft_ok(P) && (uint64_t)n_slots * 8 >= P.M)
    return P.kv_dtype == 1 ? launch_reconstruct_fft_t<true>(P, layer, a0, n_slots, Kt, Vt, tsh, st)
                           : launch_reconstruct_fft_t<false>(P, layer, a0, n_slots, Kt, Vt, tsh, st);
  const int atiles = (int)((n_slots + kRecSlots - 1) / kRecSlots);
  const uint64_t blocks = (uint64_t)P.batch * P.n_kv * atiles * 2;
  if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
  if (P.kv_dtype == 1)
    reconstruct_kernel<true><<<dim3((uint32_t)blocks), dim3(256), 0, st>>>(P, layer, a0, stride, n_slots, Kt, Vt, tsh, atiles);
  else
    reconstruct_kernel<false><<<dim3((uint32_t)blocks), dim3(256), 0, st>>>(P, layer, a0, stride, n_slots, Kt, Vt, tsh, atiles);
  return hipGetLastError();
}

}  // namespace iwdft
