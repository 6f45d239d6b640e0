// Decode attention over the reconstructed segment (Sec. 3.1.1 Eq. kv-attn over the middle part
// of Sec. 4.2.2 Eq. kv-concat) without ever writing K~ or V~ (Eq. reconstruct-idft) to memory.
//
// For one slice and one query head, with F the stored coefficients and gain folded in:
//   scores  s[a] = scale * q . K~[a]        = Re sum_k Y[k] e^{+j 2 pi k a / M},
//                                             Y[k] = (w_k scale / M) * sum_c q[c] F_K[c][k]
//   weights p[a] = exp(s[a] - max) ,  Z = sum_a p[a]
//   output  o[c] = sum_a p[a] V~[a][c] / Z  = Re sum_k F_V[c][k] * Pn[k],
//                                             Pn[k] = (w_k / (M Z)) * conj( sum_a p[a] e^{-j 2 pi k a / M} )
// The common slot shift (T-M) of the fixed-frame storage moves K~ and V~ together and drops out
// of softmax attention.  The S sink and R recent tokens that Eq. kv-concat keeps exact join the same
// softmax: kernel A also writes their raw scores q.k_e, kernel B folds them into max / Z and turns
// them into weights p_e / Z, kernel C adds sum_e (p_e / Z) v_e.  Three kernels:
//   A  attn_qc_kernel   streams F_K once, produces qc[k] = sum_c q[c] F_K[c][k]    (HBM-bound)
//   B  attn_fft_kernel  per (slice, pair of query heads): sparse spectrum -> M scores by
//                       inverse FFT in LDS, softmax, forward FFT, gather the kept bins -> Pn
//      attn_direct_kernel  same result by direct O(M |B|) sums (any M; reference path)
//   C  attn_out_kernel  streams F_V once, o[c] = Re sum_k F_V[c][k] Pn[k]           (HBM-bound)
// The fused decode step (launch_step) runs the same three kernels with the streaming update of
// Eq. infi-dft folded in: A and C either add the step's token(s) to every coefficient on its way through
// and write it back, or -- deferred write-back -- leave the coefficients alone and add the exact
// contribution of the tokens they do not hold yet (see StepUpdate).
#include "common.h"
#include "fft_lds.h"

namespace iwdft {

typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Row e of the exact tokens of a slice: sink tokens first, then the recent ring (slot order; the
// order is irrelevant to softmax attention as long as K and V use the same one).
template <bool BF16>
__device__ __forceinline__ const void* exact_row(const Params& P, bool value, int slice, int e) {
  constexpr int kElem = BF16 ? 2 : 4;
  const char* base;
  int64_t row;
  if (e < P.S) {
    base = (const char*)(value ? P.sinkV : P.sinkK);
    row = (int64_t)slice * P.S + e;
  } else {
    base = (const char*)(value ? P.ringV : P.ringK);
    row = (int64_t)slice * P.R + (e - P.S);
  }
  return base + row * kHeadDim * kElem;
}

// ------------------------------------------------------------------------------------------ A
// Block size of kernel A: the read-only form streams best with 256 threads; the read-modify-write
// form of the fused step measured ~10 % faster with 512 (206 -> 186 us on 32 x 8 x 2048 bins).
constexpr int qc_threads(bool upd) { return upd ? 512 : 256; }
constexpr int qc_bins(bool upd) { return qc_threads(upd) * 2; }

// Tokens of the fused decode step that the stored coefficients do not hold yet (see launch_step):
// row j of a slice is x[slice * stride + j * 128 + channel], j < np, and token j has the slot shift
// (tsh + j) mod M.  The kernels come in three modes:
//   kPlain  : coefficients are only read; the np pending tokens (possibly none) enter the result
//             through rank-np corrections -- F + sum_j x_j e^{j theta_j} is what attention sees,
//   kUpdate1: np == 1, the token is added to every coefficient on its way through, written back,
//   kUpdateN: the same for np <= kMaxPend tokens at once (the deferred write-back of several steps).
constexpr int kPlain = 0, kUpdate1 = 1, kUpdateN = 2;
constexpr int kPlainStream = 3;  // kernel C only: kPlain with streaming (non-temporal) coefficient loads
struct StepUpdate {
  const void* xk;
  const void* xv;
  int64_t stride;
  uint32_t tsh;
  int np;
  float* ps;  // kPlain with np > 0: [slice][query head][kMaxPend], Re sum_k e^{j theta_jk} Pn[k] (from kernel B)
  // Non-null: the step's token has not been filed yet; it is still in the caller's tensors ([slice][128])
  // and the kernels do the filing themselves.  Without a recent window (ring_slot < 0) the token is the
  // newest pending row (np - 1).  With one, the newest pending row is the token that ages out of the
  // window -- still in ring slot `ring_slot` -- and the step's token stands in for that slot among the
  // exact tokens; kernel C writes it there at its end.  In kPlain mode kernel A stores the K row and
  // kernel C the V row of the newest pending token into the pending rows for the steps to come.
  const void* nk;
  const void* nv;
  int ring_slot;
};

// Element `c` of pending row j of a slice (K: value = false, V: value = true).
template <bool BF16>
__device__ __forceinline__ float pend_elem(const Params& P, const StepUpdate& up, bool value, int slice, int j,
                                           int c) {
  if (up.nk && j == up.np - 1) {
    if (up.ring_slot >= 0)
      return load_kv<BF16>(value ? P.ringV : P.ringK, ((int64_t)slice * P.R + up.ring_slot) * kHeadDim + c);
    return load_kv<BF16>(value ? up.nv : up.nk, (int64_t)slice * kHeadDim + c);
  }
  return load_kv<BF16>(value ? up.xv : up.xk, (int64_t)slice * up.stride + j * kHeadDim + c);
}
// Keeps the newest pending token for later steps: row np - 1, channels [c0, c0 + n), one per thread.
template <bool BF16>
__device__ __forceinline__ void pend_keep(const Params& P, const StepUpdate& up, bool value, int slice, int c0,
                                          int n) {
  if (!up.nk || (int)threadIdx.x >= n) return;
  const int c = c0 + threadIdx.x;
  const float x = pend_elem<BF16>(P, up, value, slice, up.np - 1, c);  // exact: a storage-dtype value
  store_kv<BF16>(const_cast<void*>(value ? up.xv : up.xk),
                 (int64_t)slice * up.stride + (int64_t)(up.np - 1) * kHeadDim + c, x);
}
// Row e of the exact tokens during a fused step: the step's token stands in for the ring slot it is
// about to take.
template <bool BF16>
__device__ __forceinline__ const void* exact_row_step(const Params& P, const StepUpdate& up, bool value, int slice,
                                                      int e) {
  if (up.nk && up.ring_slot >= 0 && e == P.S + up.ring_slot)
    return (const char*)(value ? up.nv : up.nk) + (int64_t)slice * kHeadDim * (BF16 ? 2 : 4);
  return exact_row<BF16>(P, value, slice, e);
}

// (a.xy, a.zw) * (b.xy, b.zw): two complex products side by side.
__device__ __forceinline__ v4f cmul2(v4f a, v4f b) {
  v4f r;
  r.x = a.x * b.x - a.y * b.y;
  r.y = a.x * b.y + a.y * b.x;
  r.z = a.z * b.z - a.w * b.w;
  r.w = a.z * b.w + a.w * b.z;
  return r;
}

// Twiddles of a lane's two adjacent bins i0, i0 + 1 for slot shift p: (e^{j 2 pi k0 p / M}, e^{j 2 pi k1 p / M});
// a bin beyond the layer's list gets 0, which keeps padding entries at zero.
__device__ __forceinline__ v4f lane_twiddles(const Params& P, const LayerInfo& L, int i0, uint32_t p) {
  v4f tw = (v4f)(0.f);
  if (i0 < L.nb) {
    const float2 w0 = cis(mulmod((uint32_t)P.bins[L.bin_off + i0], p, P.M, P.Mmask), P.M);
    tw.x = w0.x;
    tw.y = w0.y;
    if (i0 + 1 < L.nb) {
      const float2 w1 = cis(mulmod((uint32_t)P.bins[L.bin_off + i0 + 1], p, P.M, P.Mmask), P.M);
      tw.z = w1.x;
      tw.w = w1.y;
    }
  }
  return tw;
}

// grid: (slice * chunks + chunk) * passes + pass.  Lane = two adjacent bins, loop over channels.
// Update modes (fused decode step): every K coefficient first absorbs the pending token(s) (the
// streaming update, Eq. infi-dft in the fixed frame: F += x e^{+j 2 pi k (T-M)/M}), is written back, and
// the updated value feeds qc, so that K coefficients are read once per step instead of twice (needs
// passes == 1).  kPlain with pending tokens: qc[k] += sum_j (q . k_j) e^{j theta_jk} instead.
// Shared memory of one block, in floats: q rows, pending K rows, the dots q . k_j.
constexpr int qc_smem_floats(int GT, int MODE) {
  return GT * kHeadDim + (MODE == kUpdate1 ? 1 : kMaxPend) * kHeadDim + (MODE == kPlain ? kMaxPend : 1) * GT;
}
// The work of logical block `bid` (wave-uniform) with THREADS threads; `sm` holds qc_smem_floats floats.
template <bool BF16, int GT, int MODE, int THREADS>
__device__ __forceinline__ void qc_body(const Params& P, const void* __restrict__ q, float2* __restrict__ qc,
                                        float* __restrict__ pe, int chunks, int passes, const StepUpdate& up,
                                        uint32_t bid, float* sm) {
  constexpr bool UPD = MODE != kPlain;
  constexpr int kQcThreads = THREADS, kQcBins = THREADS * 2;
  float (*qs)[kHeadDim] = (float (*)[kHeadDim])sm;                            // [GT][128]
  float (*xs)[kHeadDim] = qs + GT;                                             // pending K rows
  float (*dq)[GT] = (float (*)[GT])(xs + (MODE == kUpdate1 ? 1 : kMaxPend));   // q . k_j of the pending tokens
  const int pass = bid % passes;
  bid /= passes;
  const int chunk = bid % chunks;
  const int slice = bid / chunks;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const int g0 = pass * GT;
  for (int e = threadIdx.x; e < GT * kHeadDim; e += kQcThreads) {
    const int g = g0 + e / kHeadDim;
    qs[e / kHeadDim][e % kHeadDim] =
        (g < P.G) ? load_kv<BF16>(q, ((int64_t)slice * P.G + g) * kHeadDim + (e % kHeadDim)) : 0.f;
  }
  __syncthreads();
  if constexpr (MODE == kUpdateN) {
    for (int e = threadIdx.x; e < up.np * kHeadDim; e += kQcThreads)
      xs[e / kHeadDim][e % kHeadDim] = pend_elem<BF16>(P, up, false, slice, e / kHeadDim, e % kHeadDim);
    __syncthreads();
  }
  if constexpr (MODE == kPlain) {
    if (up.np > 0) {  // block-uniform
      // the pending rows go through LDS (coalesced loads, one per element), then one (token, head) dot per thread
      for (int e = threadIdx.x; e < up.np * kHeadDim; e += kQcThreads)
        xs[e / kHeadDim][e % kHeadDim] = pend_elem<BF16>(P, up, false, slice, e / kHeadDim, e % kHeadDim);
      __syncthreads();
      for (int idx = threadIdx.x; idx < up.np * GT; idx += kQcThreads) {
        const int j = idx / GT, g = idx % GT;
        float dot = 0.f;
#pragma unroll 8
        for (int c = 0; c < kHeadDim; ++c) dot += qs[g][c] * xs[j][c];
        dq[j][g] = dot;
      }
      if (chunk == 0 && pass == 0 && up.nk && (int)threadIdx.x < kHeadDim)  // keep the newest pending K row
        store_kv<BF16>(const_cast<void*>(up.xk),
                       (int64_t)slice * up.stride + (int64_t)(up.np - 1) * kHeadDim + threadIdx.x, xs[up.np - 1][threadIdx.x]);
      __syncthreads();
    }
  }
  const int E = P.S + P.R;
  if (chunk == 0 && E > 0) {  // raw scores q . k_e of the exact tokens, one (token, head) per thread
    for (int idx = threadIdx.x; idx < E * GT; idx += kQcThreads) {
      const int e = idx / GT, g = idx % GT;
      if (g0 + g >= P.G) continue;
      const void* kr = exact_row_step<BF16>(P, up, false, slice, e);
      float dot = 0.f;
      for (int c = 0; c < kHeadDim; c += 8) {
        if constexpr (BF16) {
          const uint4 w = *(const uint4*)((const uint16_t*)kr + c);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t u = (&w.x)[j];
            dot += qs[g][c + 2 * j] * __uint_as_float(u << 16) + qs[g][c + 2 * j + 1] * __uint_as_float(u & 0xffff0000u);
          }
        } else {
          const float4 w0 = *(const float4*)((const float*)kr + c), w1 = *(const float4*)((const float*)kr + c + 4);
          dot += qs[g][c] * w0.x + qs[g][c + 1] * w0.y + qs[g][c + 2] * w0.z + qs[g][c + 3] * w0.w +
                 qs[g][c + 4] * w1.x + qs[g][c + 5] * w1.y + qs[g][c + 6] * w1.z + qs[g][c + 7] * w1.w;
        }
      }
      pe[((int64_t)slice * P.G + g0 + g) * E + e] = dot;
    }
  }
  const int i0 = chunk * kQcBins + threadIdx.x * 2;
  if (i0 >= L.Bp) return;
  v4f* row = (v4f*)(P.FK + L.coef_off + (int64_t)s * kHeadDim * L.Bp + i0);
  const int64_t stride = L.Bp / 2;
  // twiddles of this lane's two bins; padding entries keep 0 and are not written
  const bool live = i0 < L.nb;
  v4f tw = (v4f)(0.f);
  if (UPD || up.np > 0) tw = lane_twiddles(P, L, i0, up.tsh);
  // kUpdateN: twiddles of the first kTwGroup pending tokens; the later groups are these times w^(8 g)
  constexpr int kTwGroup = 8;
  static_assert(kMaxPend % kTwGroup == 0, "pending tokens are handled in groups");
  v4f twn[MODE == kUpdateN ? kTwGroup : 1];
  v4f w8 = (v4f)(0.f);
  if constexpr (MODE == kUpdateN) {
    const v4f w = lane_twiddles(P, L, i0, 1u);  // one slot further per token
    twn[0] = tw;
#pragma unroll
    for (int j = 1; j < kTwGroup; ++j) twn[j] = cmul2(twn[j - 1], w);
    const v4f w2 = cmul2(w, w), w4 = cmul2(w2, w2);
    w8 = cmul2(w4, w4);
  }
  v4f acc[GT];
#pragma unroll
  for (int g = 0; g < GT; ++g) acc[g] = (v4f)(0.f);
  if constexpr (MODE == kPlain) {
    if (up.np > 0) {  // the pending tokens' share of qc
      const v4f w = lane_twiddles(P, L, i0, 1u);
      v4f t = tw;
      for (int j = 0; j < up.np; ++j) {
#pragma unroll
        for (int g = 0; g < GT; ++g) acc[g] += dq[j][g] * t;
        t = cmul2(t, w);
      }
    }
  }
  constexpr int U = 8;
#pragma unroll 1
  for (int d = 0; d < kHeadDim; d += U) {
    v4f f[U];
#pragma unroll
    for (int u = 0; u < U; ++u) f[u] = __builtin_nontemporal_load(row + (d + u) * stride);
    if constexpr (MODE == kUpdate1) {
      float x[U];
#pragma unroll
      for (int u = 0; u < U; ++u) x[u] = pend_elem<BF16>(P, up, false, slice, 0, d + u);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        f[u] += x[u] * tw;
        if (live) __builtin_nontemporal_store(f[u], row + (d + u) * stride);
      }
    }
    if constexpr (MODE == kUpdateN) {
      v4f shift = (v4f)(0.f);  // w^(8 g) of the current group of 8 tokens
      shift.x = shift.z = 1.f;
#pragma unroll
      for (int g8 = 0; g8 < kMaxPend; g8 += kTwGroup) {
        if (g8 < up.np) {
#pragma unroll
          for (int j = 0; j < kTwGroup; ++j) {
            if (g8 + j < up.np) {
              const v4f t = g8 ? cmul2(twn[j], shift) : twn[j];
#pragma unroll
              for (int u = 0; u < U; ++u) f[u] += xs[g8 + j][d + u] * t;
            }
          }
          shift = cmul2(shift, w8);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (live) __builtin_nontemporal_store(f[u], row + (d + u) * stride);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int g = 0; g < GT; ++g) acc[g] += qs[g][d + u] * f[u];
  }
#pragma unroll
  for (int g = 0; g < GT; ++g)
    if (g0 + g < P.G)
      *(v4f*)(qc + L.ws_off + ((int64_t)s * P.G + g0 + g) * L.Bp + i0) = acc[g];
}

template <bool BF16, int GT, int MODE>
__global__ __launch_bounds__(qc_threads(MODE != kPlain)) void attn_qc_kernel(Params P, const void* __restrict__ q,
                                                            float2* __restrict__ qc, float* __restrict__ pe,
                                                            int chunks, int passes, StepUpdate up) {
  __shared__ float sm[qc_smem_floats(GT, MODE)];
  qc_body<BF16, GT, MODE, qc_threads(MODE != kPlain)>(P, q, qc, pe, chunks, passes, up, blockIdx.x, sm);
}

// ------------------------------------------------------------------------------------------ C
constexpr int kOutThreads = 256;
// Channels per block: 16, or 8 where 16 channels x 8 query heads of accumulators would leave one wave per SIMD.
// (8 query heads, update modes: 256 registers + spills at 16 channels; measured 11.8 -> 7.5 ms per write-back launch on
// 10240 slices x 1638 bins.  The read-only form is faster with 16.)
constexpr int out_dc(int GT, int MODE) {
  const bool upd = MODE == kUpdate1 || MODE == kUpdateN;
  return (GT == 8 && upd) ? 8 : 16;
}

// Sum V values per lane over the whole wave; on return lane L holds the total of value
// L >> (6 - log2 V)  (V <= 64, power of two).  Each step halves the number of live values.
template <int CNT, int OFF, int V>
__device__ __forceinline__ void wave_reduce_step(float (&v)[V], int lane) {
  if constexpr (OFF >= 1) {
    if constexpr (CNT > 1) {
      constexpr int half = CNT / 2;
      const bool upper = (lane & OFF) != 0;
#pragma unroll
      for (int i = 0; i < half; ++i) {
        const float send = upper ? v[i] : v[i + half];
        const float keep = upper ? v[i + half] : v[i];
        v[i] = keep + __shfl_xor(send, OFF);
      }
      wave_reduce_step<half, OFF / 2, V>(v, lane);
    } else {
      v[0] += __shfl_xor(v[0], OFF);
      wave_reduce_step<1, OFF / 2, V>(v, lane);
    }
  }
}
template <int V>
__device__ __forceinline__ float wave_reduce_scatter(float (&v)[V], int lane) {
  wave_reduce_step<V, 32, V>(v, lane);
  return v[0];
}

// logical block: (slice * (128 / channels per block) + dchunk) * passes + pass.  Lane = two adjacent bins; a block walks all
// bins of its slice for 16 channels, so no cross-block reduction is needed.  Hardware block ids are
// dealt round-robin to the 8 XCDs; they are remapped so that the 8 channel chunks of a slice run on
// ONE XCD and fetch the slice's Pn rows into that XCD's L2 once instead of eight times.
// The coefficient loads are ordinary (cacheable) loads on purpose: what they leave in the
// memory-side cache is V state the next append reads first (measured: append 357 -> 326 us on the
// 32 x 8 x 2048-bin workload, this kernel +5 us).
// Update modes (fused decode step): every V coefficient absorbs the pending token(s) on its way through
// (written back, the updated value is what attention uses), so V coefficients are read once per step
// too.  There the state is touched once per step and nothing gains from caching it: streaming
// (non-temporal) loads and stores measured 195 -> 177 us.  kPlain with pending tokens: the output gets
// sum_j ps[j] v_j added at the end, and the loads stream as well (no append follows that could reuse them).
template <bool BF16, int GT, int MODE>
__global__ __launch_bounds__(kOutThreads) void attn_out_kernel(Params P, const float2* __restrict__ Pn,
                                                              void* __restrict__ out, const float* __restrict__ pe,
                                                              int passes, int per_xcd, int total, StepUpdate up) {
  constexpr bool UPD = MODE == kUpdate1 || MODE == kUpdateN;
  constexpr bool PLAIN = !UPD;
  constexpr bool STREAM = MODE != kPlain;  // nothing re-reads the V coefficients soon: bypass the caches
  constexpr int kOutDC = out_dc(GT, MODE);
  constexpr int V = kOutDC * GT;
  constexpr int VR = V > 64 ? 64 : V;  // values per reduction round
  __shared__ float red[kOutThreads / 64][V];
  uint32_t bid = (blockIdx.x & 7u) * (uint32_t)per_xcd + (blockIdx.x >> 3);
  if (bid >= (uint32_t)total) return;
  const int pass = bid % passes;
  bid /= passes;
  const int dc = bid % (kHeadDim / kOutDC);
  const int slice = bid / (kHeadDim / kOutDC);
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const int g0 = pass * GT;
  const int d0 = dc * kOutDC;
  const int64_t stride = L.Bp / 2;
  v4f* Fv = (v4f*)(P.FV + L.coef_off + ((int64_t)s * kHeadDim + d0) * L.Bp);
  const float2* Prow = Pn + L.ws_off + ((int64_t)s * P.G + g0) * L.Bp;

  float acc[V];
#pragma unroll
  for (int v = 0; v < V; ++v) acc[v] = 0.f;
  float xr[MODE == kUpdate1 ? kOutDC : 1];
  if constexpr (MODE == kUpdate1) {
#pragma unroll
    for (int dd = 0; dd < kOutDC; ++dd) xr[dd] = pend_elem<BF16>(P, up, true, slice, 0, d0 + dd);
  }
  __shared__ float xs[MODE == kUpdateN ? kMaxPend : 1][kOutDC];  // pending V rows, this block's channels
  if constexpr (MODE == kUpdateN) {
    for (int e = threadIdx.x; e < up.np * kOutDC; e += kOutThreads)
      xs[e / kOutDC][e % kOutDC] =
          pend_elem<BF16>(P, up, true, slice, e / kOutDC, d0 + (e % kOutDC));
    __syncthreads();
  }

  for (int i0 = threadIdx.x * 2; i0 < L.Bp; i0 += kOutThreads * 2) {
    v4f p[GT];
#pragma unroll
    for (int g = 0; g < GT; ++g)
      p[g] = (g0 + g < P.G) ? *(const v4f*)(Prow + (int64_t)g * L.Bp + i0) : (v4f)(0.f);
    v4f f[kOutDC];
#pragma unroll
    for (int dd = 0; dd < kOutDC; ++dd)
      f[dd] = STREAM ? __builtin_nontemporal_load(Fv + dd * stride + i0 / 2) : Fv[dd * stride + i0 / 2];
    if constexpr (MODE == kUpdateN) {
      if (i0 < L.nb) {  // padding entries are never written
        v4f t = (v4f)(0.f), w = (v4f)(0.f);
        const uint32_t k0 = (uint32_t)P.bins[L.bin_off + i0];
        const float2 a0 = cis_poly(mulmod(k0, up.tsh, P.M, P.Mmask), P.M), b0 = cis_poly(k0, P.M);
        t.x = a0.x, t.y = a0.y, w.x = b0.x, w.y = b0.y;
        if (i0 + 1 < L.nb) {
          const uint32_t k1 = (uint32_t)P.bins[L.bin_off + i0 + 1];
          const float2 a1 = cis_poly(mulmod(k1, up.tsh, P.M, P.Mmask), P.M), b1 = cis_poly(k1, P.M);
          t.z = a1.x, t.w = a1.y, w.z = b1.x, w.w = b1.y;
        }
        for (int j = 0; j < up.np; ++j) {
#pragma unroll
          for (int dd = 0; dd < kOutDC; ++dd) f[dd] += xs[j][dd] * t;
          t = cmul2(t, w);
        }
#pragma unroll
        for (int dd = 0; dd < kOutDC; ++dd) __builtin_nontemporal_store(f[dd], Fv + dd * stride + i0 / 2);
      }
    }
    if constexpr (MODE == kUpdate1) {
      if (i0 < L.nb) {  // padding entries are never written
        v4f tw = (v4f)(0.f);
        const float2 w0 = cis_poly(mulmod((uint32_t)P.bins[L.bin_off + i0], up.tsh, P.M, P.Mmask), P.M);
        tw.x = w0.x;
        tw.y = w0.y;
        if (i0 + 1 < L.nb) {
          const float2 w1 = cis_poly(mulmod((uint32_t)P.bins[L.bin_off + i0 + 1], up.tsh, P.M, P.Mmask), P.M);
          tw.z = w1.x;
          tw.w = w1.y;
        }
#pragma unroll
        for (int dd = 0; dd < kOutDC; ++dd) {
          f[dd] += xr[dd] * tw;
          __builtin_nontemporal_store(f[dd], Fv + dd * stride + i0 / 2);
        }
      }
    }
#pragma unroll
    for (int dd = 0; dd < kOutDC; ++dd)
#pragma unroll
      for (int g = 0; g < GT; ++g)
        acc[dd * GT + g] += f[dd].x * p[g].x - f[dd].y * p[g].y + f[dd].z * p[g].z - f[dd].w * p[g].w;
  }

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int r = 0; r < V / VR; ++r) {
    float part[VR];
#pragma unroll
    for (int v = 0; v < VR; ++v) part[v] = acc[r * VR + v];
    const float tot = wave_reduce_scatter<VR>(part, lane);
    constexpr int rep = 64 / VR;  // lanes holding the same value
    if ((lane % rep) == 0) red[wave][r * VR + lane / rep] = tot;
  }
  // Exact tokens (weights already divided by the softmax sum): every thread takes a share of the tokens for one
  // (channel, head) of the block, so that the rows are fetched side by side instead of one after the other.
  static_assert(V <= kOutThreads && kOutThreads % V == 0, "one or more threads per output value");
  constexpr int kParts = kOutThreads / V;
  __shared__ float exs[kOutThreads];
  const int E = P.S + P.R;
  const int np_plain = PLAIN ? up.np : 0;  // pending tokens of the deferred write-back: rows weighted by kernel B's ps
  if (E + np_plain > 0) {  // block-uniform
    const int v = threadIdx.x % V, part = threadIdx.x / V;
    const int dd = v / GT, g = v % GT;
    float a = 0.f;
    if (g0 + g < P.G) {
      const float* w = pe + ((int64_t)slice * P.G + g0 + g) * E;
      for (int e = part; e < E; e += kParts)
        a += w[e] * load_kv<BF16>(exact_row_step<BF16>(P, up, true, slice, e), d0 + dd);
      if constexpr (PLAIN) {
        const float* sj = up.ps + ((int64_t)slice * P.G + g0 + g) * kMaxPend;
        for (int j = part; j < np_plain; j += kParts) a += sj[j] * pend_elem<BF16>(P, up, true, slice, j, d0 + dd);
      }
    }
    exs[threadIdx.x] = a;
  }
  __syncthreads();
  for (int v = threadIdx.x; v < V; v += kOutThreads) {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < kOutThreads / 64; ++w) tot += red[w][v];
    const int dd = v / GT, g = v % GT;
    if (g0 + g < P.G) {
      if (E + np_plain > 0) {
#pragma unroll
        for (int part = 0; part < kParts; ++part) tot += exs[part * V + v];
      }
      store_kv<BF16>(out, ((int64_t)slice * P.G + g0 + g) * kHeadDim + d0 + dd, tot);
    }
  }
  if constexpr (PLAIN) {
    if (up.np > 0 && pass == 0) pend_keep<BF16>(P, up, true, slice, d0, kOutDC);  // this block's 16 channels
  }
  if (up.nk && up.ring_slot >= 0 && pass == 0) {
    // The step's token takes the ring slot (K and V, this block's 16 channels) once every read of the old
    // content by this block is done; no other block touches these channels, and kernel A is long finished.
    __syncthreads();
    if (threadIdx.x < kOutDC) {
      const int64_t src = (int64_t)slice * kHeadDim + d0 + threadIdx.x;
      const int64_t dst = ((int64_t)slice * P.R + up.ring_slot) * kHeadDim + d0 + threadIdx.x;
      store_kv<BF16>(P.ringK, dst, load_kv<BF16>(up.nk, src));
      store_kv<BF16>(P.ringV, dst, load_kv<BF16>(up.nv, src));
    }
  }
}

// ------------------------------------------------------------------------------------- B (FFT)
// Block-wide max / sum of two values at once (one per packed query head).  One barrier each: the two use
// different scratch rows and always alternate, so the barrier of the one separates the reads of the other from
// its next writes.
__device__ __forceinline__ float2 block_max2(float2 v, float2* scratch, int tid) {
  v.x = wave_max(v.x);
  v.y = wave_max(v.y);
  if ((tid & 63) == 0) scratch[tid >> 6] = v;
  __syncthreads();
  float2 r = scratch[0];
  for (int w = 1; w < kFftThreads / 64; ++w) {
    r.x = fmaxf(r.x, scratch[w].x);
    r.y = fmaxf(r.y, scratch[w].y);
  }
  return r;
}
__device__ __forceinline__ float2 block_sum2(float2 v, float2* scratch, int tid) {
  v.x = wave_sum(v.x);
  v.y = wave_sum(v.y);
  if ((tid & 63) == 0) scratch[kFftThreads / 64 + (tid >> 6)] = v;
  __syncthreads();
  float2 r = scratch[kFftThreads / 64];
  for (int w = 1; w < kFftThreads / 64; ++w) {
    r.x += scratch[kFftThreads / 64 + w].x;
    r.y += scratch[kFftThreads / 64 + w].y;
  }
  return r;
}

__device__ __forceinline__ int64_t s_global_head(int slice, int G, int g) { return (int64_t)slice * G + g; }

// Softmax over the Q time samples of one block, two heads side by side (real / imaginary part), on sample pairs held in
// registers; the radix-2 stage that ends the inverse transform and the one that starts the forward transform (odd
// log2 Q) are applied right here.  Online across blocks: (mx, Z) are the running maximum and sum; returns the factor
// exp2(old max - new max) by which everything accumulated so far has to be scaled.
template <int LOGQ>
__device__ __forceinline__ float2 softmax_block(float2* buf, int tid, bool has1, float2* scratch, float2& mx, float2& Z) {
  constexpr int Q = 1 << LOGQ;
  float2 v[kFftEPT];
  float2 lm = make_float2(-INFINITY, -INFINITY);
#pragma unroll
  for (int j = 0; j < kFftEPT / 2; ++j) {
    const int bf = j * kFftThreads + tid;
    if (2 * bf < Q) {
      float2 a = buf[pad(2 * bf)], c = buf[pad(2 * bf + 1)];
      if (LOGQ & 1) {
        const float2 t = a;
        a = cadd(t, c);
        c = csub(t, c);
      }
      v[2 * j] = a;
      v[2 * j + 1] = c;
      lm.x = fmaxf(lm.x, fmaxf(a.x, c.x));
      lm.y = fmaxf(lm.y, fmaxf(a.y, c.y));
    }
  }
  const float2 bm = block_max2(lm, scratch, tid);
  const float2 mn = make_float2(fmaxf(mx.x, bm.x), fmaxf(mx.y, bm.y));
  // exp2(-inf) = 0 the first time
  const float2 f = make_float2(__builtin_amdgcn_exp2f(mx.x - mn.x), __builtin_amdgcn_exp2f(mx.y - mn.y));
  mx = mn;
  float2 ls = make_float2(0.f, 0.f);
#pragma unroll
  for (int j = 0; j < kFftEPT / 2; ++j) {
    const int bf = j * kFftThreads + tid;
    if (2 * bf < Q) {
      float2 a = make_float2(__builtin_amdgcn_exp2f(v[2 * j].x - mn.x),
                             has1 ? __builtin_amdgcn_exp2f(v[2 * j].y - mn.y) : 0.f);
      float2 c = make_float2(__builtin_amdgcn_exp2f(v[2 * j + 1].x - mn.x),
                             has1 ? __builtin_amdgcn_exp2f(v[2 * j + 1].y - mn.y) : 0.f);
      ls.x += a.x + c.x;
      ls.y += a.y + c.y;
      if (LOGQ & 1) {
        const float2 t = a;
        a = cadd(t, c);
        c = csub(t, c);
      }
      buf[pad(2 * bf)] = a;
      buf[pad(2 * bf + 1)] = c;
    }
  }
  const float2 bs = block_sum2(ls, scratch, tid);  // its barrier also publishes the writes above
  Z = make_float2(Z.x * f.x + bs.x, Z.y * f.y + bs.y);
  return f;
}

// grid: slice * pairs + pair.  Two query heads share one complex transform: head g0 travels in
// the real part, head g0+1 in the imaginary part (each head's spectrum is made Hermitian first,
// so its time-domain signal is real).  Time index a = Pb * a' + b: block b of Q = M / Pb samples
// comes from the spectrum folded modulo Q with twiddle e^{j 2 pi k b / M}; softmax runs online
// across the Pb blocks (MULTI); with Pb == 1 nothing is carried between iterations.
// Folding uses no atomics: entries that share a slot are added in successive rounds (host-made
// schedule in P.fold), which also fixes the summation order.  NBT = kept bins per thread.
// Register budget: 128 VGPRs (two workgroups per CU) except for the multi-block kernel with 8 bins
// per thread, whose per-bin inputs and running sums (~80 registers) then spill; that one gets 256
// VGPRs and one workgroup per CU (measured 1.5x faster than spilling at two per CU).
// The work of logical block `bid` (wave-uniform); smem: fft_lds_float2(LOGQ) float2.
template <int LOGQ, int NBT, bool MULTI>
__device__ __forceinline__ void fft_body(const Params& P, const float2* __restrict__ qc, float2* __restrict__ Pn,
                                         float* __restrict__ pe, float scale, int pairs, int np, uint32_t ptsh,
                                         float* __restrict__ ps, uint32_t bid, float2* smem) {
  __shared__ float2 scratch[2 * (kFftThreads / 64)];  // row 0: block_max2, row 1: block_sum2
  __shared__ float pscr[kFftThreads / 64][2 * kMaxPend];
  const int tid = threadIdx.x;
  constexpr int Q = 1 << LOGQ;
  float2* buf = smem;                 // Q samples, padded
  float2* tab = smem + Q + (Q >> 5);  // Q/8 + 1 twiddles
  const int pair = bid % pairs;
  const int slice = bid / pairs;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const int g0 = pair * 2;
  const bool has1 = (g0 + 1) < P.G;
  const uint32_t Pb = MULTI ? (P.M >> LOGQ) : 1u;
  const float2* q0 = qc + L.ws_off + ((int64_t)s * P.G + g0) * L.Bp;
  const float2* q1 = has1 ? q0 + L.Bp : q0;
  const int32_t* bins = P.bins + L.bin_off;
  const float* wts = P.weights + L.bin_off;
  const uint16_t* fold = P.fold + L.bin_off;
  // log2(e) is folded into the scores so that softmax can use the bare exp2 instruction;
  // 0.5: each bin is split into k and its mirror.
  const float gain = 0.5f * 1.44269504088896341f * scale * P.gain / (float)P.M;

  for (int m = tid; m <= (Q >> 3); m += kFftThreads) tab[m] = P.tw8[m];  // exp(+j 2 pi m / Q), host-made

  float2 A0[NBT], A1[NBT];  // running sums over blocks (MULTI) / the single result
  // The 128-register multi-block kernel fetches its bin indices again at every use (L1 / L2 hits) instead of
  // keeping them: fewer spilled registers (12 -> 7).
  constexpr bool kReloadK = MULTI && NBT <= 4;
  uint32_t kkr[kReloadK ? 1 : NBT];
#pragma unroll
  for (int j = 0; j < NBT; ++j) {
    A0[j] = A1[j] = make_float2(0.f, 0.f);
    const int i = j * kFftThreads + tid;
    if constexpr (!kReloadK) kkr[j] = (uint32_t)bins[i < L.nb ? i : L.nb - 1];
  }
  auto KK = [&](int j) -> uint32_t {
    if constexpr (kReloadK) { const int i = j * kFftThreads + tid; return (uint32_t)bins[i < L.nb ? i : L.nb - 1]; }
    else return kkr[j];
  };
  float2 mx = make_float2(-INFINITY, -INFINITY), Z = make_float2(0.f, 0.f);

  // Exact tokens open the online softmax: their raw scores q . k_e come from kernel A.
  const int E = P.S + P.R;
  float* pe0 = pe + ((int64_t)s_global_head(slice, P.G, g0)) * E;
  float* pe1 = pe0 + E;
  const float escale = 1.44269504088896341f * scale;  // scores live in log2 units (exp2 softmax)
  if (E > 0) {
    float2 lm = make_float2(-INFINITY, -INFINITY);
    for (int e = tid; e < E; e += kFftThreads) {
      lm.x = fmaxf(lm.x, pe0[e] * escale);
      if (has1) lm.y = fmaxf(lm.y, pe1[e] * escale);
    }
    mx = block_max2(lm, scratch, tid);
    float2 ls = make_float2(0.f, 0.f);
    for (int e = tid; e < E; e += kFftThreads) {
      ls.x += __builtin_amdgcn_exp2f(pe0[e] * escale - mx.x);
      if (has1) ls.y += __builtin_amdgcn_exp2f(pe1[e] * escale - mx.y);
    }
    Z = block_sum2(ls, scratch, tid);
  }

  constexpr bool kTight = MULTI && NBT <= 4;  // 128-VGPR multi-block variant: fight hoisting
  for (uint32_t b = 0; b < Pb; ++b) {
    if (kTight) {
      // Per-bin inputs are re-read every iteration (L2 hits) instead of being kept in ~50 VGPRs.
      asm volatile("" : "+s"(q0), "+s"(q1), "+s"(wts), "+s"(fold));
    }
    // The thread index is made opaque per iteration so that the address arithmetic of the six
    // transform passes is recomputed (a few instructions) instead of being hoisted out of the
    // block loop into ~40 long-lived registers.
    int lt = tid;
    if (kTight) asm volatile("" : "+v"(lt));
    for (int e = tid; e < Q + (Q >> 5); e += kFftThreads) buf[e] = make_float2(0.f, 0.f);
    __syncthreads();
    // Folded entry of bin j of this thread: (z0, z1) for the two heads, from inputs loaded as a group (all
    // loads are issued before the first use: one latency, not one per bin).
    auto place = [&](int j, uint32_t frj, float2 z0, float2 z1, int round) {
      const int r = KK(j) & (Q - 1), rm = (Q - r) & (Q - 1);
      if ((frj & 0xffu) == (uint32_t)round) {  //      z0  + j z1
        float2 v = make_float2(z0.x - z1.y, z0.y + z1.x);
        if (r == rm) v = make_float2(2.f * z0.x, 2.f * z1.x);  // ... plus the mirror term, same slot
        if (round) v = cadd(v, buf[pad(r)]);
        buf[pad(r)] = v;
      }
      if ((frj >> 8) == (uint32_t)round) {     // conj z0  + j conj z1
        float2 v = make_float2(z0.x + z1.y, z1.x - z0.y);
        if (round) v = cadd(v, buf[pad(rm)]);
        buf[pad(rm)] = v;
      }
    };
    // The entries are formed once and the rounds only place them, except in the 8-bins-per-thread kernel with
    // the 128-register budget, which has no room to keep them and forms them again in every round.
    constexpr bool kKeep = MULTI || NBT <= 4;
    // The block twiddles e^{j 2 pi k b / M} serve the folding and, conjugated, the pruning below; the kernel with
    // the 256-register budget keeps them, the others form them twice.
    constexpr bool kKeepTw = MULTI && NBT > 4;
    float2 twk[kKeepTw ? NBT : 1];
    float2 z0[kKeep ? NBT : 1], z1[kKeep ? NBT : 1];
    uint32_t fr[NBT];
    for (int round = 0; round < L.fold_rounds; ++round) {
      if (!kKeep || round == 0) {
        float ww[NBT];
        float2 y0[NBT], y1[NBT];
#pragma unroll
        for (int j = 0; j < NBT; ++j) {
          const int i = j * kFftThreads + tid;
          const int ic = i < L.nb ? i : L.nb - 1;
          ww[j] = wts[ic] * gain;
          y0[j] = q0[ic];
          y1[j] = q1[ic];
          fr[j] = i < L.nb ? (uint32_t)fold[ic] : 0xffffu;  // 0xff: no round matches
        }
#pragma unroll
        for (int j = 0; j < NBT; ++j) {
          float2 twj = make_float2(1.f, 0.f);
          if (MULTI) twj = cis_fast((KK(j) * b) & (P.M - 1u), P.M);
          if constexpr (kKeepTw) twk[j] = twj;
          const float w = ww[j];
          const float2 a0 = cmul(make_float2(y0[j].x * w, y0[j].y * w), twj);
          const float2 a1 = has1 ? cmul(make_float2(y1[j].x * w, y1[j].y * w), twj) : make_float2(0.f, 0.f);
          if constexpr (kKeep) {
            z0[j] = a0;
            z1[j] = a1;
          } else {
            place(j, fr[j], a0, a1, round);
          }
        }
      }
      if constexpr (kKeep) {
#pragma unroll
        for (int j = 0; j < NBT; ++j) place(j, fr[j], z0[j], z1[j], round);
      }
      __syncthreads();
    }
    ifft_dif<LOGQ>(buf, tab, lt);

    const float2 f = softmax_block<LOGQ>(buf, tid, has1, scratch, mx, Z);
    fft_dit<LOGQ>(buf, tab, lt);
#pragma unroll
    for (int j = 0; j < NBT; ++j) {
      const int r = KK(j) & (Q - 1), rm = (Q - r) & (Q - 1);
      const float2 w1 = buf[pad(r)], w2 = buf[pad(rm)];
      const float2 p0 = make_float2(0.5f * (w1.x + w2.x), 0.5f * (w1.y - w2.y));
      const float2 p1 = make_float2(0.5f * (w1.y + w2.y), 0.5f * (w2.x - w1.x));
      if (MULTI) {
        const float2 twc = conjf2(kKeepTw ? twk[j] : cis_fast((KK(j) * b) & (P.M - 1u), P.M));
        A0[j] = cadd(make_float2(A0[j].x * f.x, A0[j].y * f.x), cmul(twc, p0));
        A1[j] = cadd(make_float2(A1[j].x * f.y, A1[j].y * f.y), cmul(twc, p1));
      } else {
        A0[j] = p0;
        A1[j] = p1;
      }
    }
    __syncthreads();
  }

  float2* o0 = Pn + L.ws_off + ((int64_t)s * P.G + g0) * L.Bp;
  float2* o1 = o0 + L.Bp;
  const float inv_M = P.gain / (float)P.M;
  const float iz0 = inv_M / Z.x, iz1 = has1 ? inv_M / Z.y : 0.f;
  // Pending tokens of the fused decode step (not yet inside F_V): token j adds
  // v_j * Re sum_k e^{j theta_jk} Pn[k] to the output; the sums are formed here, where Pn is at hand.
  float sp[2 * kMaxPend];  // [token][head g0, head g0 + 1]
#pragma unroll
  for (int v = 0; v < 2 * kMaxPend; ++v) sp[v] = 0.f;
#pragma unroll
  for (int j = 0; j < NBT; ++j) {
    const int i = j * kFftThreads + tid;
    if (i < L.Bp) {  // padding entries are written as zeros: kernel C reads whole rows
      float2 r0 = make_float2(0.f, 0.f), r1 = r0;
      if (i < L.nb) {
        const float w = wts[i];
        r0 = make_float2(A0[j].x * (w * iz0), -A0[j].y * (w * iz0));
        r1 = make_float2(A1[j].x * (w * iz1), -A1[j].y * (w * iz1));
        if (np > 0) {  // block-uniform
          // hardware sine / cosine (~1e-6 absolute): these are weights of value rows, far inside the tolerance
          // u_n = Re(t step^n r) for n = 0 .. np - 1 obeys u_{n+1} = 2 cos(phi) u_n - u_{n-1} (phi = the step's angle):
          // one multiply-add per token and head instead of a complex rotation (at most 15 steps: no error growth
          // that matters next to the 1e-6 of the hardware sine)
          const float2 t = cis_fast((KK(j) * ptsh) & (P.M - 1u), P.M);
          const float2 step = cis_fast(KK(j), P.M);
          const float2 t1 = cmul(t, step);
          const float c2 = 2.f * step.x;
          float a0 = t.x * r0.x - t.y * r0.y, a1 = t1.x * r0.x - t1.y * r0.y;  // head g0: u_0, u_1
          float b0 = t.x * r1.x - t.y * r1.y, b1 = t1.x * r1.x - t1.y * r1.y;  // head g0 + 1
#pragma unroll
          for (int jp = 0; jp < kMaxPend; ++jp) {
            if (jp < np) {
              sp[2 * jp] += a0;
              sp[2 * jp + 1] += b0;
              const float a2 = c2 * a1 - a0, b2 = c2 * b1 - b0;
              a0 = a1, a1 = a2;
              b0 = b1, b1 = b2;
            }
          }
        }
      }
      o0[i] = r0;
      if (has1) o1[i] = r1;
    }
  }
  if (np > 0) {
    // all 2 * kMaxPend sums over the wave at once: afterwards lane l holds the total of entry l / rep
    const float tot = wave_reduce_scatter<2 * kMaxPend>(sp, tid & 63);
    constexpr int rep = 64 / (2 * kMaxPend);  // lanes that end up with the same total
    if ((tid & 63) % rep == 0) pscr[tid >> 6][(tid & 63) / rep] = tot;
    __syncthreads();
    if (tid < 2 * np) {
      float sum = 0.f;
      for (int w = 0; w < kFftThreads / 64; ++w) sum += pscr[w][tid];
      const int jp = tid >> 1, head = tid & 1;
      if (head == 0 || has1) ps[((int64_t)s_global_head(slice, P.G, g0) + head) * kMaxPend + jp] = sum;
    }
  }
  for (int e = tid; e < E; e += kFftThreads) {  // raw scores -> weights p_e / Z (same thread, same entry)
    pe0[e] = __builtin_amdgcn_exp2f(pe0[e] * escale - mx.x) / Z.x;
    if (has1) pe1[e] = __builtin_amdgcn_exp2f(pe1[e] * escale - mx.y) / Z.y;
  }
}

template <int LOGQ, int NBT, bool MULTI>
__global__ __launch_bounds__(kFftThreads, (MULTI && NBT > 4) ? 2 : 4) void attn_fft_kernel(Params P, const float2* __restrict__ qc,
                                                                 float2* __restrict__ Pn, float* __restrict__ pe,
                                                                 float scale, int pairs, int np, uint32_t ptsh,
                                                                 float* __restrict__ ps) {
  extern __shared__ float2 smem[];
  fft_body<LOGQ, NBT, MULTI>(P, qc, Pn, pe, scale, pairs, np, ptsh, ps, blockIdx.x, smem);
}

// ------------------------------------------------------------------------- B (FFT, > 4096 kept bins)
// The same computation for layers that keep more bins than the kernel above holds in registers (8 per thread): the
// threads walk the bin list in strides of the workgroup, nothing per bin stays in registers.  Folding re-reads the
// inputs in every round and block; the running sums over blocks (MULTI) live in the output rows themselves -- every bin
// belongs to one thread, which reads back its own earlier store, scales it by the online-softmax factor and adds the
// block's term -- and a last sweep turns them into the normalised weights.  No pending tokens (write_every is 1).
template <int LOGQ, bool MULTI>
__global__ __launch_bounds__(kFftThreads, 4) void attn_fft_big_kernel(Params P, const float2* __restrict__ qc,
                                                                     float2* __restrict__ Pn, float* __restrict__ pe,
                                                                     float scale, int pairs) {
  extern __shared__ float2 smem[];
  __shared__ float2 scratch[2 * (kFftThreads / 64)];
  const int tid = threadIdx.x;
  constexpr int Q = 1 << LOGQ;
  float2* buf = smem;
  float2* tab = smem + Q + (Q >> 5);
  const int pair = blockIdx.x % pairs;
  const int slice = blockIdx.x / pairs;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const int g0 = pair * 2;
  const bool has1 = (g0 + 1) < P.G;
  const uint32_t Pb = MULTI ? (P.M >> LOGQ) : 1u;
  const float2* q0 = qc + L.ws_off + ((int64_t)s * P.G + g0) * L.Bp;
  const float2* q1 = has1 ? q0 + L.Bp : q0;
  float2* o0 = Pn + L.ws_off + ((int64_t)s * P.G + g0) * L.Bp;
  float2* o1 = o0 + L.Bp;  // written only if has1
  const int32_t* bins = P.bins + L.bin_off;
  const float* wts = P.weights + L.bin_off;
  const uint16_t* fold = P.fold + L.bin_off;
  const float gain = 0.5f * 1.44269504088896341f * scale * P.gain / (float)P.M;  // log2 units; 0.5: bin + mirror

  for (int m = tid; m <= (Q >> 3); m += kFftThreads) tab[m] = P.tw8[m];

  float2 mx = make_float2(-INFINITY, -INFINITY), Z = make_float2(0.f, 0.f);
  const int E = P.S + P.R;
  float* pe0 = pe + ((int64_t)s_global_head(slice, P.G, g0)) * E;
  float* pe1 = pe0 + E;
  const float escale = 1.44269504088896341f * scale;
  if (E > 0) {  // exact tokens open the online softmax (raw scores from kernel A)
    float2 lm = make_float2(-INFINITY, -INFINITY);
    for (int e = tid; e < E; e += kFftThreads) {
      lm.x = fmaxf(lm.x, pe0[e] * escale);
      if (has1) lm.y = fmaxf(lm.y, pe1[e] * escale);
    }
    mx = block_max2(lm, scratch, tid);
    float2 ls = make_float2(0.f, 0.f);
    for (int e = tid; e < E; e += kFftThreads) {
      ls.x += __builtin_amdgcn_exp2f(pe0[e] * escale - mx.x);
      if (has1) ls.y += __builtin_amdgcn_exp2f(pe1[e] * escale - mx.y);
    }
    Z = block_sum2(ls, scratch, tid);
  }

  for (uint32_t b = 0; b < Pb; ++b) {
    for (int e = tid; e < Q + (Q >> 5); e += kFftThreads) buf[e] = make_float2(0.f, 0.f);
    __syncthreads();
    for (int round = 0; round < L.fold_rounds; ++round) {
      for (int i = tid; i < L.nb; i += kFftThreads) {
        const uint32_t fr = fold[i];
        const bool direct = (fr & 0xffu) == (uint32_t)round, mirror = (fr >> 8) == (uint32_t)round;
        if (!direct && !mirror) continue;
        const uint32_t k = (uint32_t)bins[i];
        const float w = wts[i] * gain;
        const float2 y0 = q0[i], y1 = q1[i];
        const float2 tw = MULTI ? cis_fast((k * b) & (P.M - 1u), P.M) : make_float2(1.f, 0.f);
        const float2 z0 = cmul(make_float2(y0.x * w, y0.y * w), tw);
        const float2 z1 = has1 ? cmul(make_float2(y1.x * w, y1.y * w), tw) : make_float2(0.f, 0.f);
        const int r = k & (Q - 1), rm = (Q - r) & (Q - 1);
        if (direct) {  //      z0  + j z1
          float2 v = make_float2(z0.x - z1.y, z0.y + z1.x);
          if (r == rm) v = make_float2(2.f * z0.x, 2.f * z1.x);  // ... plus the mirror term, same slot
          if (round) v = cadd(v, buf[pad(r)]);
          buf[pad(r)] = v;
        }
        if (mirror) {  // conj z0  + j conj z1
          float2 v = make_float2(z0.x + z1.y, z1.x - z0.y);
          if (round) v = cadd(v, buf[pad(rm)]);
          buf[pad(rm)] = v;
        }
      }
      __syncthreads();
    }
    ifft_dif<LOGQ>(buf, tab, tid);
    const float2 f = softmax_block<LOGQ>(buf, tid, has1, scratch, mx, Z);
    fft_dit<LOGQ>(buf, tab, tid);
    for (int i = tid; i < L.nb; i += kFftThreads) {
      const uint32_t k = (uint32_t)bins[i];
      const int r = k & (Q - 1), rm = (Q - r) & (Q - 1);
      const float2 w1 = buf[pad(r)], w2 = buf[pad(rm)];
      float2 p0 = make_float2(0.5f * (w1.x + w2.x), 0.5f * (w1.y - w2.y));
      float2 p1 = make_float2(0.5f * (w1.y + w2.y), 0.5f * (w2.x - w1.x));
      if (MULTI) {
        const float2 twc = conjf2(cis_fast((k * b) & (P.M - 1u), P.M));
        p0 = cmul(twc, p0);
        p1 = cmul(twc, p1);
        if (b) {  // this thread's own running sums, scaled to the new maximum
          const float2 a0 = o0[i];
          p0 = make_float2(a0.x * f.x + p0.x, a0.y * f.x + p0.y);
          if (has1) {
            const float2 a1 = o1[i];
            p1 = make_float2(a1.x * f.y + p1.x, a1.y * f.y + p1.y);
          }
        }
      }
      o0[i] = p0;
      if (has1) o1[i] = p1;
    }
    __syncthreads();
  }

  const float inv_M = P.gain / (float)P.M;
  const float iz0 = inv_M / Z.x, iz1 = has1 ? inv_M / Z.y : 0.f;
  for (int i = tid; i < L.Bp; i += kFftThreads) {  // padding entries are written as zeros: kernel C reads whole rows
    float2 r0 = make_float2(0.f, 0.f), r1 = r0;
    if (i < L.nb) {
      const float w = wts[i];
      const float2 a0 = o0[i];
      r0 = make_float2(a0.x * (w * iz0), -a0.y * (w * iz0));
      if (has1) {
        const float2 a1 = o1[i];
        r1 = make_float2(a1.x * (w * iz1), -a1.y * (w * iz1));
      }
    }
    o0[i] = r0;
    if (has1) o1[i] = r1;
  }
  for (int e = tid; e < E; e += kFftThreads) {  // raw scores -> weights p_e / Z (same thread, same entry)
    pe0[e] = __builtin_amdgcn_exp2f(pe0[e] * escale - mx.x) / Z.x;
    if (has1) pe1[e] = __builtin_amdgcn_exp2f(pe1[e] * escale - mx.y) / Z.y;
  }
}

// ----------------------------------------------------------------------------------- A + B
// Kernel-A blocks of one group of slices and kernel-B blocks of ANOTHER group in one launch, dealt to the CUs
// side by side: B's transforms run on the vector ALU while A's blocks wait on HBM.  Nothing inside a launch
// depends on anything else inside it -- the host walks the groups as a pipeline, launch i = A(group i) next to
// B(group i - 1), so B always reads qc rows that an earlier launch on the same stream completed.
// Hardware block ids go round-robin to the 8 XCDs; the role is a function of the per-XCD sequence number, so
// every XCD sees the same even mix (nA8 / nB8 = blocks of either role per XCD, rounded up).
// A runs in its read-only form with 512 threads (1024 bins per block).
template <bool BF16, int GT, int LOGQ, int NBT, bool MULTI>
__global__ __launch_bounds__(kFftThreads, (MULTI && NBT > 4) ? 2 : 4) void attn_ab_kernel(
    Params P, const void* __restrict__ q, float2* __restrict__ qc, float* __restrict__ pe, int chunks, StepUpdate up,
    float2* __restrict__ Pn, float scale, int pairs, int np, float* __restrict__ ps, uint32_t baseA, uint32_t nA,
    uint32_t nA8, uint32_t baseB, uint32_t nB, uint32_t nB8) {
  extern __shared__ float2 smem[];
  const uint32_t seq = blockIdx.x >> 3, xcd = blockIdx.x & 7u, tot = nA8 + nB8;
  const uint32_t cb = (uint32_t)(((uint64_t)seq * nB8) / tot), cb1 = (uint32_t)(((uint64_t)(seq + 1) * nB8) / tot);
  if (cb1 > cb) {
    const uint32_t id = (uint32_t)__builtin_amdgcn_readfirstlane((int)(cb * 8 + xcd));
    if (id < nB) fft_body<LOGQ, NBT, MULTI>(P, qc, Pn, pe, scale, pairs, np, up.tsh, ps, baseB + id, smem);
  } else {
    const uint32_t id = (uint32_t)__builtin_amdgcn_readfirstlane((int)((seq - cb) * 8 + xcd));
    if (id < nA) qc_body<BF16, GT, kPlain, kFftThreads>(P, q, qc, pe, chunks, 1, up, baseA + id, (float*)smem);
  }
}

// ------------------------------------------------------------------------------------ B (chirp)
// The same two transforms for M that is not a power of two (e.g. M = context - sink - recent, Sec. 4.2.1, which is a
// power of two only by arrangement), through the chirp-z identity  k a = (k^2 + a^2 - (a - k)^2) / 2:
//   sum_k Z[k] e^{+j 2 pi k a / Qc} = c[a] * sum_k (Z[k] c[k]) h[a - k],   c[n] = e^{+j pi n^2 / Qc},  h = conj c,
// a linear convolution with the chirp h, run as a circular one of length N = 2^LOGN >= 2 Qc - 1 in LDS: transform,
// multiply by the transform of h (host-made table, already divided by N, stored in the digit-reversed order the
// first transform leaves), transform back.  The forward transform of the softmax weights is the conjugate chain.
// Qc = M up to 8192.  Longer M run Pb = M / Qc blocks (Pb the smallest divisor of M that brings Qc down to 8192):
// time index a = Pb a' + b, block b comes from the spectrum folded modulo Qc with twiddle e^{j 2 pi k b / M}, softmax
// runs online across the blocks and the running sums of the weights live in the output rows (every bin belongs to one
// thread, which reads back its own earlier store).  Four N-point transforms per block and pair of query heads instead
// of two Qc-point ones: O(M log M) as well, ~8x the work of the power-of-two kernel, against O(M |B|) of the direct
// sums.  One workgroup per (slice, head pair); LOGN even.  No pending tokens (the deferred write-back needs the
// power-of-two kernel).
template <int LOGN>
__global__ __launch_bounds__(kFftThreads, 2) void attn_chirp_kernel(Params P, const float2* __restrict__ qc,
                                                                   float2* __restrict__ Pn, float* __restrict__ pe,
                                                                   float scale, int pairs) {
  static_assert((LOGN & 1) == 0, "even transform lengths only: no radix-2 stage between the passes");
  extern __shared__ float2 smem[];
  __shared__ float2 scratch[2 * (kFftThreads / 64)];
  const int tid = threadIdx.x;
  constexpr int N = 1 << LOGN;
  float2* buf = smem;
  float2* tab = smem + N + (N >> 5);
  const int pair = blockIdx.x % pairs;
  const int slice = blockIdx.x / pairs;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const int g0 = pair * 2;
  const bool has1 = (g0 + 1) < P.G;
  const uint32_t M = P.M, Qc = P.chirp_Q, Pb = M / Qc;
  const float2* q0 = qc + L.ws_off + ((int64_t)s * P.G + g0) * L.Bp;
  const float2* q1 = has1 ? q0 + L.Bp : q0;
  float2* o0 = Pn + L.ws_off + ((int64_t)s * P.G + g0) * L.Bp;
  float2* o1 = o0 + L.Bp;  // written only if has1
  const int32_t* bins = P.bins + L.bin_off;
  const float* wts = P.weights + L.bin_off;
  const uint16_t* fold = P.fold + L.bin_off;
  const float2* __restrict__ chirp = P.chirp;    // c[a], a < Qc
  const float2* __restrict__ Hd = P.chirpH;      // transform of h / N, digit-reversed positions
  const float gain = 0.5f * 1.44269504088896341f * scale * P.gain / (float)M;  // log2 units; 0.5: bin + mirror
  const float inv_Mf = 1.0f / (float)M;

  for (int m = tid; m <= (N >> 3); m += kFftThreads) tab[m] = cis((uint32_t)m, (uint32_t)N);

  // Exact tokens open the softmax (raw scores q . k_e from kernel A), as in the power-of-two kernel.
  float2 mx = make_float2(-INFINITY, -INFINITY), Z = make_float2(0.f, 0.f);
  const int E = P.S + P.R;
  float* pe0 = pe + ((int64_t)s_global_head(slice, P.G, g0)) * E;
  float* pe1 = pe0 + E;
  const float escale = 1.44269504088896341f * scale;
  if (E > 0) {
    float2 lm = make_float2(-INFINITY, -INFINITY);
    for (int e = tid; e < E; e += kFftThreads) {
      lm.x = fmaxf(lm.x, pe0[e] * escale);
      if (has1) lm.y = fmaxf(lm.y, pe1[e] * escale);
    }
    mx = block_max2(lm, scratch, tid);
    float2 ls = make_float2(0.f, 0.f);
    for (int e = tid; e < E; e += kFftThreads) {
      ls.x += __builtin_amdgcn_exp2f(pe0[e] * escale - mx.x);
      if (has1) ls.y += __builtin_amdgcn_exp2f(pe1[e] * escale - mx.y);
    }
    Z = block_sum2(ls, scratch, tid);
  }

  for (uint32_t b = 0; b < Pb; ++b) {
    // block twiddle e^{j 2 pi k b / M} through the hardware sine / cosine (the phase k b mod M is reduced exactly,
    // its quotient by M is rounded once: ~1e-7 revolutions)
    auto block_tw = [&](uint32_t k) {
      if (Pb == 1) return make_float2(1.f, 0.f);
      const float ph = (float)mulmod(k, b, M, P.Mmask) * inv_Mf;
      return make_float2(__builtin_amdgcn_cosf(ph), __builtin_amdgcn_sinf(ph));
    };
    for (int e = tid; e < N + (N >> 5); e += kFftThreads) buf[e] = make_float2(0.f, 0.f);
    __syncthreads();
    // Hermitian spectrum of both heads (head g0 real, head g0 + 1 imaginary in time), folded modulo Qc, times the
    // chirp.  A slot can receive several terms: successive rounds (host-made schedule).
    for (int round = 0; round < L.fold_rounds; ++round) {
      for (int i = tid; i < L.nb; i += kFftThreads) {
        const uint32_t fr = fold[i];
        const bool direct = (fr & 0xffu) == (uint32_t)round, mirror = (fr >> 8) == (uint32_t)round;
        if (!direct && !mirror) continue;
        const uint32_t k = (uint32_t)bins[i];
        const float w = wts[i] * gain;
        const float2 y0 = q0[i], y1 = q1[i];
        const float2 tw = block_tw(k);
        const float2 z0 = cmul(make_float2(y0.x * w, y0.y * w), tw);
        const float2 z1 = has1 ? cmul(make_float2(y1.x * w, y1.y * w), tw) : make_float2(0.f, 0.f);
        const uint32_t r = k % Qc, rm = r ? Qc - r : 0u;
        if (direct) {  //      z0  + j z1
          float2 v = make_float2(z0.x - z1.y, z0.y + z1.x);
          if (r == rm) v = make_float2(2.f * z0.x, 2.f * z1.x);  // ... plus the mirror term, same slot
          v = cmul(v, chirp[r]);
          if (round) v = cadd(v, buf[pad(r)]);
          buf[pad(r)] = v;
        }
        if (mirror) {  // conj z0  + j conj z1
          float2 v = cmul(make_float2(z0.x + z1.y, z1.x - z0.y), chirp[rm]);
          if (round) v = cadd(v, buf[pad(rm)]);
          buf[pad(rm)] = v;
        }
      }
      __syncthreads();
    }
    ifft_dif<LOGN>(buf, tab, tid);
    for (int p = tid; p < N; p += kFftThreads) buf[pad(p)] = cmul(buf[pad(p)], Hd[p]);
    __syncthreads();
    fft_dit<LOGN>(buf, tab, tid);

    // scores of slot a < Qc of this block: real part head g0, imaginary part head g0 + 1
    float2 lm = make_float2(-INFINITY, -INFINITY);
    for (uint32_t a = tid; a < Qc; a += kFftThreads) {
      const float2 z = cmul(buf[pad(a)], chirp[a]);
      buf[pad(a)] = z;
      lm.x = fmaxf(lm.x, z.x);
      lm.y = fmaxf(lm.y, z.y);
    }
    const float2 bm = block_max2(lm, scratch, tid);
    const float2 mn = make_float2(fmaxf(mx.x, bm.x), fmaxf(mx.y, bm.y));
    const float2 f = make_float2(__builtin_amdgcn_exp2f(mx.x - mn.x), __builtin_amdgcn_exp2f(mx.y - mn.y));
    mx = mn;
    float2 ls = make_float2(0.f, 0.f);
    for (uint32_t a = tid; a < (uint32_t)N; a += kFftThreads) {
      float2 v = make_float2(0.f, 0.f);
      if (a < Qc) {
        const float2 z = buf[pad(a)];
        const float2 p = make_float2(__builtin_amdgcn_exp2f(z.x - mn.x), has1 ? __builtin_amdgcn_exp2f(z.y - mn.y) : 0.f);
        ls.x += p.x;
        ls.y += p.y;
        v = cmul(p, conjf2(chirp[a]));
      }
      buf[pad(a)] = v;
    }
    const float2 bs = block_sum2(ls, scratch, tid);  // its barrier also publishes the writes above
    Z = make_float2(Z.x * f.x + bs.x, Z.y * f.y + bs.y);
    ifft_dif<LOGN>(buf, tab, tid);
    for (int p = tid; p < N; p += kFftThreads) buf[pad(p)] = cmul(buf[pad(p)], conjf2(Hd[p]));
    __syncthreads();
    fft_dit<LOGN>(buf, tab, tid);

    for (int i = tid; i < L.nb; i += kFftThreads) {
      const uint32_t k = (uint32_t)bins[i];
      const uint32_t r = k % Qc, rm = r ? Qc - r : 0u;
      const float2 w1 = cmul(buf[pad(r)], conjf2(chirp[r])), w2 = cmul(buf[pad(rm)], conjf2(chirp[rm]));
      float2 p0 = make_float2(0.5f * (w1.x + w2.x), 0.5f * (w1.y - w2.y));
      float2 p1 = make_float2(0.5f * (w1.y + w2.y), 0.5f * (w2.x - w1.x));
      if (Pb > 1) {
        const float2 twc = conjf2(block_tw(k));
        p0 = cmul(twc, p0);
        p1 = cmul(twc, p1);
        if (b) {  // this thread's own running sums, scaled to the new maximum
          const float2 a0 = o0[i];
          p0 = make_float2(a0.x * f.x + p0.x, a0.y * f.x + p0.y);
          if (has1) {
            const float2 a1 = o1[i];
            p1 = make_float2(a1.x * f.y + p1.x, a1.y * f.y + p1.y);
          }
        }
      }
      o0[i] = p0;
      if (has1) o1[i] = p1;
    }
    __syncthreads();
  }

  const float inv_M = P.gain / (float)M;
  const float iz0 = inv_M / Z.x, iz1 = has1 ? inv_M / Z.y : 0.f;
  for (int i = tid; i < L.Bp; i += kFftThreads) {  // padding entries are written as zeros: kernel C reads whole rows
    float2 r0 = make_float2(0.f, 0.f), r1 = r0;
    if (i < L.nb) {
      const float w = wts[i];
      const float2 a0 = o0[i];
      r0 = make_float2(a0.x * (w * iz0), -a0.y * (w * iz0));
      if (has1) {
        const float2 a1 = o1[i];
        r1 = make_float2(a1.x * (w * iz1), -a1.y * (w * iz1));
      }
    }
    o0[i] = r0;
    if (has1) o1[i] = r1;
  }
  for (int e = tid; e < E; e += kFftThreads) {  // raw scores -> weights p_e / Z
    pe0[e] = __builtin_amdgcn_exp2f(pe0[e] * escale - mx.x) / Z.x;
    if (has1) pe1[e] = __builtin_amdgcn_exp2f(pe1[e] * escale - mx.y) / Z.y;
  }
}

// ---------------------------------------------------------------------------------- B (direct)
constexpr int kDirThreads = 256;
constexpr int kDirStage = 1024;

// grid: slice * G + g.  Evaluates the score and weight sums term by term; O(M |B|) per head.
__global__ __launch_bounds__(kDirThreads) void attn_direct_kernel(Params P, const float2* __restrict__ qc,
                                                                 float2* __restrict__ Pn, float* __restrict__ pe,
                                                                 float scale, float* __restrict__ scores) {
  __shared__ float2 Ys[kDirStage];
  __shared__ uint32_t ks[kDirStage];
  __shared__ float redf[kDirThreads / 64];
  const int tid = threadIdx.x;
  const int g = blockIdx.x % P.G;
  const int slice = blockIdx.x / P.G;
  const int spl = P.batch * P.n_kv;
  const int layer = slice / spl;
  const int s = slice - layer * spl;
  const LayerInfo L = P.layers[layer];
  const float2* qrow = qc + L.ws_off + ((int64_t)s * P.G + g) * L.Bp;
  float* sc = scores + (int64_t)blockIdx.x * P.M;
  const float gain = scale * P.gain / (float)P.M;

  for (int c0 = 0; c0 < L.nb; c0 += kDirStage) {
    const int cn = min(kDirStage, L.nb - c0);
    __syncthreads();
    for (int e = tid; e < cn; e += kDirThreads) {
      const float w = P.weights[L.bin_off + c0 + e] * gain;
      const float2 a = qrow[c0 + e];
      Ys[e] = make_float2(a.x * w, a.y * w);
      ks[e] = (uint32_t)P.bins[L.bin_off + c0 + e];
    }
    __syncthreads();
    for (uint32_t a = tid; a < P.M; a += kDirThreads) {
      float acc = c0 ? sc[a] : 0.f;
      for (int e = 0; e < cn; ++e) {
        const float2 w = cis(mulmod(ks[e], a, P.M, P.Mmask), P.M);
        acc += Ys[e].x * w.x - Ys[e].y * w.y;
      }
      sc[a] = acc;
    }
  }
  __syncthreads();
  const int E = P.S + P.R;
  float* per = pe + ((int64_t)slice * P.G + g) * E;  // raw q . k_e from kernel A
  float lm = -INFINITY;
  for (uint32_t a = tid; a < P.M; a += kDirThreads) lm = fmaxf(lm, sc[a]);
  for (int e = tid; e < E; e += kDirThreads) lm = fmaxf(lm, per[e] * scale);
  lm = wave_max(lm);
  if ((tid & 63) == 0) redf[tid >> 6] = lm;
  __syncthreads();
  float mx = redf[0];
  for (int w = 1; w < kDirThreads / 64; ++w) mx = fmaxf(mx, redf[w]);
  __syncthreads();
  float lsum = 0.f;
  for (uint32_t a = tid; a < P.M; a += kDirThreads) {
    const float p = expf(sc[a] - mx);
    sc[a] = p;
    lsum += p;
  }
  for (int e = tid; e < E; e += kDirThreads) lsum += expf(per[e] * scale - mx);
  lsum = wave_sum(lsum);
  if ((tid & 63) == 0) redf[tid >> 6] = lsum;
  __syncthreads();
  float Z = 0.f;
  for (int w = 0; w < kDirThreads / 64; ++w) Z += redf[w];

  for (int e = tid; e < E; e += kDirThreads) per[e] = expf(per[e] * scale - mx) / Z;  // weights p_e / Z
  float2* orow = Pn + L.ws_off + ((int64_t)s * P.G + g) * L.Bp;
  const float inv_M = P.gain / (float)P.M;
  for (int i = tid; i < L.Bp; i += kDirThreads) {
    float2 r = make_float2(0.f, 0.f);
    if (i < L.nb) {
      const uint32_t k = (uint32_t)P.bins[L.bin_off + i];
      float re = 0.f, im = 0.f;
      uint32_t ph = 0;
      for (uint32_t a = 0; a < P.M; ++a) {
        const float2 w = cis(ph, P.M);
        const float p = sc[a];
        re += p * w.x;
        im += p * w.y;  // conj of sum p e^{-j..} = sum p e^{+j..}
        ph += k;
        if (ph >= P.M) ph -= P.M;
      }
      const float c = P.weights[L.bin_off + i] * inv_M / Z;
      r = make_float2(re * c, im * c);
    }
    orow[i] = r;
  }
}

// --------------------------------------------------------------------------------------- host
constexpr uint32_t kAbMinB = 1024, kAbMaxGroups = 8;  // fewest B blocks per group of slices, most groups
static int heads_per_pass(int G);
bool attn_pipelines(const Params& P, bool use_fft) {
  const int GT = heads_per_pass(P.G);
  const int per_thread = (P.max_Bp + kFftThreads - 1) / kFftThreads;
  return use_fft && P.G <= GT && (GT == 4 || GT == 8) && P.M >= 16384u && per_thread > 2 && per_thread <= kFftNBT &&
         (uint64_t)P.n_slices * ((P.G + 1) / 2) >= 2 * kAbMinB && !P.serial_phases;
}
static int heads_per_pass(int G) { return G <= 2 ? G : (G <= 4 ? 4 : 8); }  // 1, 2, 4 or 8; heads beyond G are masked

// up / mode: the fused decode step's pending tokens and what kernels A and C do with them (see StepUpdate).
template <bool BF16>
static hipError_t launch_attn_t(const Params& P, const void* q, void* out, float scale, float2* qc,
                                float2* Pn, float* pe, float* direct_scratch, bool use_fft,
                                const StepUpdate* up, int mode, const PhaseEvents* marks, hipStream_t st) {
  const int GT = heads_per_pass(P.G);
  const int passes = (P.G + GT - 1) / GT;
  const StepUpdate u = up ? *up : StepUpdate{nullptr, nullptr, 0, 0, 0, nullptr, nullptr, nullptr, -1};
  const int kQcThreads = qc_threads(mode != kPlain), kQcBins = qc_bins(mode != kPlain);
  const int chunks = (P.max_Bp + kQcBins - 1) / kQcBins;
  const uint64_t gridA = (uint64_t)P.n_slices * chunks * passes;
  const int dcC = out_dc(GT, mode == kPlain && u.np > 0 ? kPlainStream : mode);
  const uint64_t gridC = (uint64_t)P.n_slices * (kHeadDim / dcC) * passes;
  const uint64_t gridBd = (uint64_t)P.n_slices * P.G;
  if (gridA > 0x7fffffffull || gridC > 0x7fffffffull || gridBd > 0x7fffffffull)
    return hipErrorInvalidConfiguration;

#define IWDFT_GT_SWITCH1(KERNEL, MODE, GRID, THREADS, ...)                                               \
  switch (GT) {                                                                                          \
    case 1: KERNEL<BF16, 1, MODE><<<dim3((uint32_t)(GRID)), dim3(THREADS), 0, st>>>(__VA_ARGS__); break;  \
    case 2: KERNEL<BF16, 2, MODE><<<dim3((uint32_t)(GRID)), dim3(THREADS), 0, st>>>(__VA_ARGS__); break;  \
    case 4: KERNEL<BF16, 4, MODE><<<dim3((uint32_t)(GRID)), dim3(THREADS), 0, st>>>(__VA_ARGS__); break;  \
    default: KERNEL<BF16, 8, MODE><<<dim3((uint32_t)(GRID)), dim3(THREADS), 0, st>>>(__VA_ARGS__); break; \
  }
#define IWDFT_GT_SWITCH(KERNEL, GRID, THREADS, ...)                                              \
  if (mode == kUpdate1) { IWDFT_GT_SWITCH1(KERNEL, kUpdate1, GRID, THREADS, __VA_ARGS__) }       \
  else if (mode == kUpdateN) { IWDFT_GT_SWITCH1(KERNEL, kUpdateN, GRID, THREADS, __VA_ARGS__) }  \
  else { IWDFT_GT_SWITCH1(KERNEL, kPlain, GRID, THREADS, __VA_ARGS__) }

  if (u.np > 0 && passes != 1) return hipErrorInvalidValue;  // the fused step needs all heads in one pass
  if (u.np > kMaxPend || (mode == kUpdate1 && u.np != 1) || (mode != kPlain && u.np < 1) ||
      (u.np > 0 && mode == kPlain && (!use_fft || !u.ps)))
    return hipErrorInvalidValue;
  const int np_plain = mode == kPlain ? u.np : 0;  // pending tokens kernel B has to weigh
  hipError_t e = hipSuccess;
#define IWDFT_MARK(I)                                            \
  if (marks && (e = hipEventRecord(marks->ev[I], st)) != hipSuccess) return e;
  // Long contexts with many slices: A and B run as a pipeline over groups of slices, each launch holding the
  // A blocks of one group next to the B blocks of the group before (attn_ab_kernel).  Worth it when B is a
  // large share of the step and a group still fills the chip: M >= 16384 and at least kAbMinB B blocks per group;
  // measured (A + B, all slices, ms): 2048 slices x 4096 bins, M = 32768: 2.36 -> 1.9; 10240 x 1638, M = 16384:
  // 6.3 -> 5.5; no gain at M = 8192 (B is 30 us) or with 512 B blocks in all (M = 131072, 256 slices).
  const int pairsB = (P.G + 1) / 2;
  const int per_thread_ab = (P.max_Bp + kFftThreads - 1) / kFftThreads;
  const uint64_t nB_all = (uint64_t)P.n_slices * pairsB;
  const bool pipeline_ab = mode == kPlain && attn_pipelines(P, use_fft);
  if (pipeline_ab) {
    IWDFT_MARK(0)
    const size_t lds = sizeof(float2) * (size_t)fft_lds_float2(kFftMaxLogQ);
    const int chunksA = (P.max_Bp + 2 * kFftThreads - 1) / (2 * kFftThreads);
    uint32_t groups = (uint32_t)(nB_all / kAbMinB);
    if (groups > kAbMaxGroups) groups = kAbMaxGroups;
    const uint32_t spg = ((uint32_t)P.n_slices + groups - 1) / groups;  // slices per group
    for (uint32_t i = 0; i <= groups; ++i) {
      // A: group i, B: group i - 1
      const uint32_t a0 = i * spg, a1 = i < groups ? (a0 + spg < (uint32_t)P.n_slices ? a0 + spg : (uint32_t)P.n_slices) : a0;
      const uint32_t b0 = i ? (i - 1) * spg : 0, b1 = i ? (b0 + spg < (uint32_t)P.n_slices ? b0 + spg : (uint32_t)P.n_slices) : 0;
      const uint32_t sa = a1 > a0 ? a1 - a0 : 0, sb = b1 > b0 ? b1 - b0 : 0;
      const uint32_t nA = sa * chunksA, nB = sb * pairsB;
      if (nA + nB == 0) continue;
      const uint32_t nA8 = (nA + 7) / 8, nB8 = (nB + 7) / 8;
      const uint32_t grid = (nA8 + nB8) * 8;
#define IWDFT_AB_CASE(GTV, NBT, MULTI)                                                                          \
  {                                                                                                             \
    static LdsLimit lim;                                                                                        \
    e = lim.ensure((const void*)attn_ab_kernel<BF16, GTV, kFftMaxLogQ, NBT, MULTI>, (int)lds);                  \
    if (e != hipSuccess) return e;                                                                              \
    attn_ab_kernel<BF16, GTV, kFftMaxLogQ, NBT, MULTI><<<dim3(grid), dim3(kFftThreads), lds, st>>>(             \
        P, q, qc, pe, chunksA, u, Pn, scale, pairsB, np_plain, u.ps, a0 * chunksA, nA, nA8, b0 * pairsB, nB,    \
        nB8);                                                                                                   \
  }
      if (GT == 4) {
        if (per_thread_ab <= 4) IWDFT_AB_CASE(4, 4, true) else IWDFT_AB_CASE(4, 8, true)
      } else {
        if (per_thread_ab <= 4) IWDFT_AB_CASE(8, 4, true) else IWDFT_AB_CASE(8, 8, true)
      }
#undef IWDFT_AB_CASE
      e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    IWDFT_MARK(1)  // the marks cannot separate A from B here: phase A = the pipeline, phase B = nothing
    IWDFT_MARK(2)
  } else {
  IWDFT_MARK(0)
  IWDFT_GT_SWITCH(attn_qc_kernel, gridA, kQcThreads, P, q, qc, pe, chunks, passes, u)
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  IWDFT_MARK(1)
  }

  if (pipeline_ab) {
  } else if (use_fft) {
    int logM = 0;
    while ((1u << logM) < P.M) ++logM;
    const int logQ = logM < kFftMaxLogQ ? logM : kFftMaxLogQ;
    const int pairs = (P.G + 1) / 2;
    const size_t lds = sizeof(float2) * (size_t)fft_lds_float2(logQ);
    const uint32_t gridB = (uint32_t)((uint64_t)P.n_slices * pairs);
    const int per_thread = (P.max_Bp + kFftThreads - 1) / kFftThreads;  // <= 8 (checked at create)
#define IWDFT_FFT_CASE(LQ, NBT, MULTI)                                                                   \
  {                                                                                                      \
    static LdsLimit lim;                                                                                 \
    e = lim.ensure((const void*)attn_fft_kernel<LQ, NBT, MULTI>, (int)lds);                              \
    if (e != hipSuccess) return e;                                                                       \
    attn_fft_kernel<LQ, NBT, MULTI><<<dim3(gridB), dim3(kFftThreads), lds, st>>>(P, qc, Pn, pe, scale,   \
                                                                                pairs, np_plain, u.tsh,  \
                                                                                u.ps);                   \
  }
#define IWDFT_FFT_NBT(LQ, MULTI)                                                                         \
  {                                                                                                      \
    if (per_thread <= 2) IWDFT_FFT_CASE(LQ, 2, MULTI)                                                    \
    else if (per_thread <= 4) IWDFT_FFT_CASE(LQ, 4, MULTI)                                               \
    else IWDFT_FFT_CASE(LQ, 8, MULTI)                                                                    \
  }
    if (per_thread > kFftNBT) {  // more than 4096 kept bins in some layer (so M > 4096): nothing per bin in registers
      if (np_plain > 0) return hipErrorInvalidValue;  // no pending tokens on this path (the plan takes write_every as 1)
#define IWDFT_FFT_BIG(MULTI)                                                                             \
  {                                                                                                      \
    static LdsLimit lim;                                                                                 \
    e = lim.ensure((const void*)attn_fft_big_kernel<kFftMaxLogQ, MULTI>, (int)lds);                      \
    if (e != hipSuccess) return e;                                                                       \
    attn_fft_big_kernel<kFftMaxLogQ, MULTI><<<dim3(gridB), dim3(kFftThreads), lds, st>>>(P, qc, Pn, pe,  \
                                                                                        scale, pairs);  \
  }
      if (logM > logQ) IWDFT_FFT_BIG(true) else IWDFT_FFT_BIG(false)
#undef IWDFT_FFT_BIG
    } else if (logM > logQ) IWDFT_FFT_NBT(kFftMaxLogQ, true)
    else switch (logQ) {
      case 8: IWDFT_FFT_CASE(8, 8, false) break;
      case 9: IWDFT_FFT_CASE(9, 8, false) break;
      case 10: IWDFT_FFT_CASE(10, 8, false) break;
      case 11: IWDFT_FFT_CASE(11, 8, false) break;
      case 12: IWDFT_FFT_CASE(12, 8, false) break;
      default: IWDFT_FFT_NBT(13, false) break;
    }
#undef IWDFT_FFT_NBT
#undef IWDFT_FFT_CASE
  } else if (P.chirp) {
    const int pairs = (P.G + 1) / 2;
    const size_t lds = sizeof(float2) * (size_t)fft_lds_float2(P.chirp_logN);
    const uint32_t gridB = (uint32_t)((uint64_t)P.n_slices * pairs);
#define IWDFT_CHIRP_CASE(LN)                                                                             \
  {                                                                                                      \
    static LdsLimit lim;                                                                                 \
    e = lim.ensure((const void*)attn_chirp_kernel<LN>, (int)lds);                                        \
    if (e != hipSuccess) return e;                                                                       \
    attn_chirp_kernel<LN><<<dim3(gridB), dim3(kFftThreads), lds, st>>>(P, qc, Pn, pe, scale, pairs);     \
  }
    switch (P.chirp_logN) {
      case 8: IWDFT_CHIRP_CASE(8) break;
      case 10: IWDFT_CHIRP_CASE(10) break;
      case 12: IWDFT_CHIRP_CASE(12) break;
      case 14: IWDFT_CHIRP_CASE(14) break;
      default: return hipErrorInvalidValue;
    }
#undef IWDFT_CHIRP_CASE
  } else {
    attn_direct_kernel<<<dim3((uint32_t)gridBd), dim3(kDirThreads), 0, st>>>(P, qc, Pn, pe, scale, direct_scratch);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (!pipeline_ab) { IWDFT_MARK(2) }

  const int per_xcd = (int)((gridC + 7) / 8);
  if (mode == kPlain && u.np > 0) {  // deferred write-back: no append follows that could reuse cached V state
    IWDFT_GT_SWITCH1(attn_out_kernel, kPlainStream, (uint64_t)per_xcd * 8, kOutThreads, P, Pn, out, pe, passes, per_xcd,
                     (int)gridC, u)
  } else {
    IWDFT_GT_SWITCH(attn_out_kernel, (uint64_t)per_xcd * 8, kOutThreads, P, Pn, out, pe, passes, per_xcd, (int)gridC, u)
  }
#undef IWDFT_GT_SWITCH
#undef IWDFT_GT_SWITCH1
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  IWDFT_MARK(3)
#undef IWDFT_MARK
  return hipSuccess;
}

hipError_t launch_attn(const Params& P, const void* q, void* out, float scale, float2* qc, float2* Pn,
                       float* pe, float* direct_scratch, bool use_fft, const PhaseEvents* marks,
                       hipStream_t st) {
  return P.kv_dtype == 1
             ? launch_attn_t<true>(P, q, out, scale, qc, Pn, pe, direct_scratch, use_fft, nullptr, kPlain, marks, st)
             : launch_attn_t<false>(P, q, out, scale, qc, Pn, pe, direct_scratch, use_fft, nullptr, kPlain, marks, st);
}

bool heads_fit_one_pass(int G) { return (G + heads_per_pass(G) - 1) / heads_per_pass(G) == 1; }
bool step_can_fuse(const Params& P) { return heads_fit_one_pass(P.G); }

hipError_t launch_step(const Params& P, const void* tok_k, const void* tok_v, const void* q, void* out,
                       float scale, float2* qc, float2* Pn, float* pe, void* pend_k, void* pend_v, float* ps,
                       float* direct_scratch, bool use_fft, uint32_t tsh0, uint32_t ring_pos, int pend_before,
                       int write_every, const PhaseEvents* marks, hipStream_t st) {
  if (write_every < 1 || write_every > kMaxPend || pend_before < 0 || pend_before >= write_every)
    return hipErrorInvalidValue;
  StepUpdate up{tok_k, tok_v, kHeadDim, tsh0, pend_before + 1, ps, nullptr, nullptr, -1};
  if (P.R > 0 || write_every > 1) {  // the kernels file the step's token themselves (see StepUpdate)
    up.xk = pend_k;
    up.xv = pend_v;
    up.stride = (int64_t)write_every * kHeadDim;
    up.nk = tok_k;
    up.nv = tok_v;
    up.ring_slot = P.R > 0 ? (int)ring_pos : -1;
  }
  const int mode = up.np < write_every ? kPlain : (write_every == 1 ? kUpdate1 : kUpdateN);
  return P.kv_dtype == 1
             ? launch_attn_t<true>(P, q, out, scale, qc, Pn, pe, direct_scratch, use_fft, &up, mode, marks, st)
             : launch_attn_t<false>(P, q, out, scale, qc, Pn, pe, direct_scratch, use_fft, &up, mode, marks, st);
}

}  // namespace iwdft
