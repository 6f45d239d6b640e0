// Shared device-side definitions of libiwdft: state layout, exact phase arithmetic,
// dtype conversion.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>

#include <vector>
#include <stdint.h>

namespace iwdft {

constexpr int kHeadDim = 128;  // channels per head the kernels are written for
constexpr int kRowPad = 32;    // a coefficient row is padded to a multiple of this many bins

// Per-layer geometry, one entry per layer in device memory.
struct LayerInfo {
  int32_t bin_off;   // first entry of this layer in the bins / weights arrays
  int32_t nb;        // number of kept bins |B_l|
  int32_t Bp;        // nb rounded up to kRowPad: length of one coefficient row (in float2)
  int32_t fold_rounds;  // largest number of spectrum entries that fold onto one FFT slot (FFT attention)
  int64_t coef_off;  // float2 offset of the layer's first slice plane inside FK / FV
  int64_t ws_off;    // float2 offset of the layer's first (slice, query-head) row in qc / Pn
};

// Everything a kernel needs to find its data.  Passed by value.
//
// Coefficient storage ("fixed frame"): for tensor X in {K, V}, slice s of layer l, channel c,
// kept-bin index i (bin k = bins[bin_off + i]):
//     F[coef_off + (s * 128 + c) * Bp + i] = F_T[k] = exp(+j 2 pi k (T-M) / M) * U_T[k]
// where U_T = T * S_T is the un-normalised accumulator of the IWDFT recursion (Sec. 4.1).
// In this frame one recursion step is F_{T+1}[k] = F_T[k] + x_T * exp(+j 2 pi k (T-M) / M):
// the rotation by W_k and the factors (N-1)/N, 1/N of Eq. infi-dft are folded into the phase
// of the added term and into the 1/T applied whenever S_T is read out, so the stored numbers
// never pass through a rounded rotation and old tokens keep exactly their weight.
// Row entries with i >= nb are padding and stay zero.
struct Params {
  int32_t n_layers, batch, n_kv, G, n_slices;  // n_slices = n_layers * batch * n_kv
  int32_t kv_dtype;                            // IWDFT_F32 / IWDFT_BF16
  uint32_t M;                                  // DFT length
  uint32_t Mmask;                              // M-1 when M is a power of two, else 0
  int32_t max_nb, max_Bp;
  const LayerInfo* layers;
  const int32_t* bins;
  const float* weights;
  const uint16_t* fold;  // per kept bin: low byte = round of its direct slot, high byte = round of its mirror slot
                         // (0xff: the mirror falls on the direct slot and is added in the same write)
  // Chirp-z attention (M that is not a power of two; null otherwise): transforms of chirp_Q = M / Pb points, Pb the
  // smallest divisor of M with M / Pb <= 8192 (1 for M <= 8192).  chirp[a] = exp(+j pi a^2 / chirp_Q), a < chirp_Q;
  // chirpH: 2^chirp_logN entries, the transform of the conjugate chirp divided by its length, in the digit-reversed
  // order of the in-LDS transform.
  const float2* chirp;
  const float2* chirpH;
  int32_t chirp_logN;
  uint32_t chirp_Q;
  // Twiddle octant of the in-LDS power-of-two transforms: tw8[m] = exp(+j 2 pi m / Q), m = 0 .. Q/8, with
  // Q = min(M, 8192); made on the host in double precision (null unless M = 2^m >= 256).
  const float2* tw8;
  float2* FK;
  float2* FV;
  // Exact tokens (Sec. 4.2.1): S sink tokens and a ring of R recent tokens per slice, kv_dtype,
  // [slice][S][128] and [slice][R][128].  Null / 0 when the windows are not used.
  // 1 except with IWDFT_FLAG_SHORTCUT (Sec. 4.1, (N-1)/N taken as 1), where the host sets them per call: an
  // absorbed token enters scaled by x_scale = M / (T + 1), and everything that reads the coefficients as the
  // paper's S_T (reconstruction, scores, outputs) applies the extra gain = T / M.
  float gain, x_scale;
  int32_t serial_phases;  // IWDFT_FLAG_SERIAL_PHASES: never pipeline kernels A and B over groups of slices
  int32_t S, R;
  void* sinkK;
  void* sinkV;
  void* ringK;
  void* ringV;
};

// (a * b) mod M, exact.
__device__ __forceinline__ uint32_t mulmod(uint32_t a, uint32_t b, uint32_t M, uint32_t Mmask) {
  uint64_t p = (uint64_t)a * (uint64_t)b;
  return Mmask ? ((uint32_t)p & Mmask) : (uint32_t)(p % M);
}

// exp(+j 2 pi p / M) for an already reduced phase 0 <= p < M.  For power-of-two M the
// argument handed to sincospi is exact, so the result is correct to ~1 ulp at any M.
__device__ __forceinline__ float2 cis(uint32_t p, uint32_t M) {
  float x = 2.0f * (float)p / (float)M;
  float s, c;
  sincospif(x, &s, &c);
  return make_float2(c, s);
}

// Same value, branch-free (straight-line code that can sit inside a software-pipelined loop):
// octant reduction in exact arithmetic (p/M and q/8 are exact for power-of-two M), degree-7/8
// Taylor polynomials on |theta| <= pi/8 (truncation < 1e-9), then a rotation by q * 45 degrees.
__device__ __forceinline__ float2 cis_poly_x(float x);
__device__ __forceinline__ float2 cis_poly(uint32_t p, uint32_t M) { return cis_poly_x((float)p / (float)M); }
// 1 / M for M = 2^m, exact (exponent negated), without the division sequence.
__device__ __forceinline__ float rcp_pow2(uint32_t M) { return __uint_as_float(0x7f000000u - __float_as_uint((float)M)); }
// cis_poly for M = 2^m.
__device__ __forceinline__ float2 cis_poly2(uint32_t p, uint32_t M) { return cis_poly_x((float)p * rcp_pow2(M)); }
// x = p / M in [0, 1).
__device__ __forceinline__ float2 cis_poly_x(float x) {
  const float qf = rintf(x * 8.0f);               // nearest octant boundary, 0..8
  const float th = (x - qf * 0.125f) * 6.283185307179586f;  // |th| <= pi/8
  const float t2 = th * th;
  float sn = th * (1.0f + t2 * (-1.0f / 6.0f + t2 * (1.0f / 120.0f + t2 * (-1.0f / 5040.0f))));
  float cs = 1.0f + t2 * (-0.5f + t2 * (1.0f / 24.0f + t2 * (-1.0f / 720.0f + t2 * (1.0f / 40320.0f))));
  const int q = (int)qf;
  if (q & 1) {  // + 45 degrees (compiles to selects)
    const float c2 = (cs - sn) * 0.70710678118654752f, s2 = (cs + sn) * 0.70710678118654752f;
    cs = c2;
    sn = s2;
  }
  if (q & 2) {  // + 90 degrees
    const float c2 = -sn;
    sn = cs;
    cs = c2;
  }
  if (q & 4) {  // + 180 degrees
    cs = -cs;
    sn = -sn;
  }
  return make_float2(cs, sn);
}

__device__ __forceinline__ float2 cmul(float2 a, float2 b) {
  return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <bool BF16>
__device__ __forceinline__ float load_kv(const void* p, int64_t i) {
  if constexpr (BF16) return bf16_to_f32(((const uint16_t*)p)[i]);
  else return ((const float*)p)[i];
}

template <bool BF16>
__device__ __forceinline__ void store_kv(void* p, int64_t i, float v) {
  if constexpr (BF16) ((uint16_t*)p)[i] = f32_to_bf16(v);
  else ((float*)p)[i] = v;
}

// Host-side launchers (defined next to their kernels).  Each validates nothing: the C ABI
// layer has already checked every shape.  They return the hipError_t of the launch.
hipError_t launch_prefill(const Params& P, const void* K, const void* V, hipStream_t st);
// The same transform through in-LDS FFTs; prefill_fft_ok: M is a power of two >= 256 and no layer
// keeps more than 4096 bins.  launch_prefill_edges copies the sink / recent tokens (both prefills).
bool prefill_fft_ok(const Params& P);
hipError_t launch_prefill_fft(const Params& P, const void* K, const void* V, hipStream_t st);
hipError_t launch_prefill_edges(const Params& P, const void* K, const void* V, hipStream_t st);
// ring_pos: slot of the recent ring that holds the oldest token (ignored when R == 0).
hipError_t launch_append(const Params& P, const void* tok_k, const void* tok_v, uint32_t t_shift,
                         uint32_t ring_pos, hipStream_t st);
hipError_t launch_export(const Params& P, int layer, float* SK, float* SV, uint32_t t_shift,
                         float inv_T, hipStream_t st);
// use_fft: the fold schedule (Params::fold) is valid, so long slot ranges may go through inverse FFTs.
// Slots a0, a0 + stride, ..., n_slots of them (stride >= 1; the FFT kernel serves stride 1 only).
hipError_t launch_reconstruct(const Params& P, int layer, uint32_t a0, uint32_t stride, uint32_t n_slots, void* Kt,
                              void* Vt, uint32_t t_shift, bool use_fft, hipStream_t st);
// Optional timing marks of the three attention phases: ev[0] before A, ev[1] after A (q against
// the K coefficients), ev[2] after B (softmax through the transforms), ev[3] after C (output from
// the V coefficients).
struct PhaseEvents {
  hipEvent_t ev[4];
};
// pe: [slice][query head][S + R] normalised softmax weights of the exact tokens (workspace).
// marks may be null.
hipError_t launch_attn(const Params& P, const void* q, void* out, float scale, float2* qc,
                       float2* Pn, float* pe, float* direct_scratch, bool use_fft,
                       const PhaseEvents* marks, hipStream_t st);

// One decode step = append + attention with the update fused into the attention kernels.
// write_every = 1: every coefficient is read once and written once per step.  write_every = J > 1: the
// coefficients are written back only on every J-th step; in between the tokens they do not hold yet
// (pend_before of them before this call, kept in pend_k / pend_v, [slice][J][128] kv_dtype) enter the
// attention through rank-one corrections, so every step returns the same result (up to rounding order).
// t_shift0: slot shift of the oldest pending token (of this step's token if none is pending);
// ps: [slice][query head][kMaxPend] floats.  step_can_fuse: all query heads fit one pass.
constexpr int kMaxPend = 16;
bool heads_fit_one_pass(int G);
// Whether decode attention on this context walks the slices in groups (kernels A and B pipelined, see attn_ab_kernel).
bool attn_pipelines(const Params& P, bool use_fft);
bool step_can_fuse(const Params& P);
hipError_t launch_step(const Params& P, const void* tok_k, const void* tok_v, const void* q, void* out,
                       float scale, float2* qc, float2* Pn, float* pe, void* pend_k, void* pend_v, float* ps,
                       float* direct_scratch, bool use_fft, uint32_t t_shift0, uint32_t ring_pos,
                       int pend_before, int write_every, const PhaseEvents* marks, hipStream_t st);
// The streaming update alone for one row per slice, x[slice * x_slice_stride + channel] (no ring hand-over).
hipError_t launch_absorb(const Params& P, const void* xk, const void* xv, int64_t x_slice_stride,
                         uint32_t t_shift, hipStream_t st);

// Frequency-ablation tools (Sec. 3.2).  launch_ablate: x, out [n_slices][M][128], M = 2^8 .. 2^13, the bins
// [lo, hi) zeroed.  select_chunks: the floor(r C + 1/2) (clamped to 1 .. C) chunks with the largest delta,
// lower index first among equals, ascending; -1 if a delta is NaN.
hipError_t launch_ablate(const void* x, void* out, int n_slices, uint32_t M, int kv_dtype, int lo, int hi,
                         hipStream_t st);
int64_t chunk_edge(int64_t c, int64_t M, int64_t C);
int select_chunks(const float* delta, int n_chunks, double r, std::vector<int>* keep);

// Raises a kernel's dynamic-LDS limit once per (kernel, device); one static instance per kernel.
struct LdsLimit {
  unsigned long long done = 0;  // bit per device; a race only repeats the idempotent call
  hipError_t ensure(const void* fn, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (dev & 63);
    if (done & bit) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done |= bit;
    return e;
  }
};

}  // namespace iwdft
