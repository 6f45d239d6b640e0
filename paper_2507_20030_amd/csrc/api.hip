// C ABI of libiwdft: descriptor validation, buffer layout, call ordering, error reporting.
// All arithmetic lives in the kernels; this file only decides what to launch.
#include <algorithm>
#include <cmath>
#include <complex>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/iwdft.h"
#include "common.h"

using namespace iwdft;

// Library-owned scratch of compressed_decode_attn_static: one copy per GPU, allocated by the loader with the
// code object and held until the process ends.  Host code never uses this name as an address (it is a host-side
// stand-in); the per-device address comes from hipGetSymbolAddress, see static_scratch().
constexpr size_t kStaticScratchBytes = (size_t)IWDFT_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
// Token, query and output tensors are read and written with 16-byte accesses.
bool misaligned16(const void* p) { return ((uintptr_t)p & 15u) != 0; }
const char kAlignMsg[] = "a device tensor is not 16-byte aligned";

struct Plan {  // byte offsets inside the two caller buffers, derived from a descriptor
  std::vector<LayerInfo> layers;
  std::vector<uint16_t> fold;  // see Params::fold
  int64_t n_bins_total = 0;
  int64_t coef_total = 0;  // float2 per tensor
  int64_t ws_total = 0;    // float2 per workspace array
  int32_t G = 1, max_nb = 0, max_Bp = 0;
  bool use_fft = false;          // decode attention through power-of-two FFTs
  bool use_chirp = false;        // ... through chirp-z transforms (any M up to kChirpMaxM when use_fft is false)
  int chirp_logN = 0;            // length of its circular convolutions
  int64_t chirp_Q = 0;           // points per chirp-z transform: M / Pb (M itself up to 8192)
  size_t off_chirp = 0, off_chirpH = 0;
  int64_t tw_Q = 0;              // length of the power-of-two in-LDS transforms (0: none), table at off_tw
  size_t off_tw = 0;
  bool use_fft_prefill = false;  // prefill through FFTs (else the dense MFMA contraction)
  int write_every = 1;           // fused decode step: coefficients written back every this many tokens
  size_t off_layers = 0, off_bins = 0, off_weights = 0, off_fold = 0, off_FK = 0, off_FV = 0, state_bytes = 0;
  size_t off_sinkK = 0, off_sinkV = 0, off_ringK = 0, off_ringV = 0;
  size_t off_qc = 0, off_Pn = 0, off_pe = 0, off_pendK = 0, off_pendV = 0, off_ps = 0, off_direct = 0, ws_bytes = 0;
};

// Most kept bins per layer the FFT kernels keep in registers (prefill, reconstruction, the deferred write-back);
// decode attention itself takes any number through its bin-strided kernel.
constexpr int kFftMaxBins = 4096;
constexpr int kFftPrefillMinBins = 384;  // fewer kept bins per layer: the dense contraction is faster
constexpr int kMaxExact = 1024;  // most sink + recent tokens (their scores sit in LDS)
constexpr uint32_t kFftMinM = 256;
constexpr int64_t kFftMaxQ = 8192;  // longest transform the FFT attention kernel holds in LDS
constexpr int64_t kChirpMinM = 32, kChirpMaxM = 8192;  // chirp-z transforms: 2 Q - 1 <= 16384 points fit in LDS
constexpr int64_t kChirpMaxBlocks = 256;  // most decimated blocks M / Q of the chirp-z attention
constexpr uint64_t kDirectMaxTerms = 1ull << 30;  // most M * |B| the direct sums are chosen for without being asked

int make_plan(const iwdft_desc* d, Plan* pl) {
  if (!d) return fail(IWDFT_ERR_ARG, "desc is NULL");
  if (d->n_layers <= 0 || d->batch <= 0 || d->n_kv_heads <= 0 || d->n_q_heads <= 0)
    return fail(IWDFT_ERR_ARG, "n_layers, batch, n_kv_heads, n_q_heads must be positive");
  if (d->n_q_heads % d->n_kv_heads != 0)
    return fail(IWDFT_ERR_ARG, "n_q_heads (%d) is not a multiple of n_kv_heads (%d)", d->n_q_heads,
                d->n_kv_heads);
  if (d->kv_dtype != IWDFT_F32 && d->kv_dtype != IWDFT_BF16)
    return fail(IWDFT_ERR_ARG, "kv_dtype %d is neither IWDFT_F32 nor IWDFT_BF16", d->kv_dtype);
  if (d->write_every > (uint32_t)kMaxPend)
    return fail(IWDFT_ERR_ARG, "write_every = %u exceeds %d", d->write_every, kMaxPend);
  if (d->flags & ~(uint32_t)(IWDFT_FLAG_DIRECT_SYNTHESIS | IWDFT_FLAG_DENSE_PREFILL | IWDFT_FLAG_FFT_PREFILL |
                             IWDFT_FLAG_SHORTCUT | IWDFT_FLAG_SERIAL_PHASES))
    return fail(IWDFT_ERR_ARG, "unknown bits in flags: 0x%x", d->flags);
  if ((d->flags & IWDFT_FLAG_DENSE_PREFILL) && (d->flags & IWDFT_FLAG_FFT_PREFILL))
    return fail(IWDFT_ERR_ARG, "flags ask for both the dense and the FFT prefill");
  if (d->M < 1 || d->M > ((int64_t)1 << 30))
    return fail(IWDFT_ERR_ARG, "M = %lld outside [1, 2^30]", (long long)d->M);
  if (d->n_sink < 0 || d->n_recent < 0) return fail(IWDFT_ERR_ARG, "n_sink / n_recent is negative");
  if ((int64_t)d->n_sink + d->n_recent > kMaxExact)
    return fail(IWDFT_ERR_UNSUPPORTED, "n_sink + n_recent = %lld exceeds %d", (long long)d->n_sink + d->n_recent,
                kMaxExact);
  if (d->head_dim <= 0) return fail(IWDFT_ERR_ARG, "head_dim must be positive");
  if (d->head_dim != kHeadDim)
    return fail(IWDFT_ERR_UNSUPPORTED, "head_dim %d: this build has kernels for head_dim 128 only",
                d->head_dim);
  pl->G = d->n_q_heads / d->n_kv_heads;
  if (pl->G > 64) return fail(IWDFT_ERR_UNSUPPORTED, "more than 64 query heads per KV head");
  if ((int64_t)d->n_layers * d->batch * d->n_kv_heads > ((int64_t)1 << 24))
    return fail(IWDFT_ERR_UNSUPPORTED, "more than 2^24 slices");
  if (!d->bin_offsets || !d->bins) return fail(IWDFT_ERR_ARG, "bin_offsets / bins is NULL");
  if (d->bin_offsets[0] != 0) return fail(IWDFT_ERR_BINS, "bin_offsets[0] must be 0");

  const int64_t slices_per_layer = (int64_t)d->batch * d->n_kv_heads;
  pl->layers.resize(d->n_layers);
  int64_t coef = 0, ws = 0;
  for (int l = 0; l < d->n_layers; ++l) {
    int64_t b0 = d->bin_offsets[l], b1 = d->bin_offsets[l + 1];
    if (b1 <= b0) return fail(IWDFT_ERR_BINS, "layer %d keeps no bins (or offsets decrease)", l);
    if (b1 - b0 > d->M) return fail(IWDFT_ERR_BINS, "layer %d keeps more than M bins", l);
    if (b1 > ((int64_t)1 << 30)) return fail(IWDFT_ERR_UNSUPPORTED, "more than 2^30 bins in total");
    int64_t prev = -1;
    for (int64_t i = b0; i < b1; ++i) {
      int64_t k = d->bins[i];
      if (k < 0 || k >= d->M)
        return fail(IWDFT_ERR_BINS, "layer %d: bin %lld outside [0, M)", l, (long long)k);
      if (k <= prev)
        return fail(IWDFT_ERR_BINS, "layer %d: bins not strictly increasing at entry %lld", l,
                    (long long)(i - b0));
      prev = k;
      if (d->bin_weights && !std::isfinite(d->bin_weights[i]))
        return fail(IWDFT_ERR_BINS, "layer %d: non-finite bin weight", l);
    }
    LayerInfo& L = pl->layers[l];
    L.bin_off = (int32_t)b0;
    L.nb = (int32_t)(b1 - b0);
    L.Bp = (L.nb + kRowPad - 1) / kRowPad * kRowPad;
    L.fold_rounds = 0;
    L.coef_off = coef;
    L.ws_off = ws;
    coef += slices_per_layer * kHeadDim * L.Bp;
    ws += slices_per_layer * pl->G * L.Bp;
    if (L.nb > pl->max_nb) pl->max_nb = L.nb;
    if (L.Bp > pl->max_Bp) pl->max_Bp = L.Bp;
  }
  pl->n_bins_total = d->bin_offsets[d->n_layers];
  pl->coef_total = coef;
  pl->ws_total = ws;

  const bool pow2 = (d->M & (d->M - 1)) == 0;
  pl->use_fft = pow2 && (uint64_t)d->M >= kFftMinM && !(d->flags & IWDFT_FLAG_DIRECT_SYNTHESIS);
  // Prefill: the FFT costs the same whatever the number of kept bins, the dense contraction grows
  // with it; measured break-even on MI355X: about 300 kept bins per layer at M = 8192, 430 at M = 131072.
  const bool fft_pf_ok = pow2 && (uint64_t)d->M >= kFftMinM;
  if (d->flags & IWDFT_FLAG_FFT_PREFILL) {
    if (!fft_pf_ok)
      return fail(IWDFT_ERR_UNSUPPORTED, "FFT prefill needs M = 2^m >= %d", (int)kFftMinM);
    pl->use_fft_prefill = true;
  } else {
    pl->use_fft_prefill = fft_pf_ok && !(d->flags & IWDFT_FLAG_DENSE_PREFILL) && pl->max_nb >= kFftPrefillMinBins;
  }
  // Chirp-z attention for M that is not a power of two: M itself up to 8192 points; longer M in Pb decimated blocks
  // of M / Pb points, Pb the smallest divisor of M that brings the block down to 8192 (none: the direct sums).
  pl->use_chirp = false;
  if (!pl->use_fft && !(d->flags & IWDFT_FLAG_DIRECT_SYNTHESIS) && d->M >= kChirpMinM) {
    for (int64_t pb = (d->M + kChirpMaxM - 1) / kChirpMaxM; pb <= kChirpMaxBlocks && d->M / pb >= kChirpMinM; ++pb) {
      if (d->M % pb == 0) {
        pl->use_chirp = true;
        pl->chirp_Q = d->M / pb;
        break;
      }
    }
  }
  if (pl->use_chirp) {
    pl->chirp_logN = 8;
    while (((int64_t)1 << pl->chirp_logN) < 2 * pl->chirp_Q - 1) pl->chirp_logN += 2;  // even lengths only
  }
  pl->fold.assign((size_t)pl->n_bins_total, 0);
  if (pl->use_fft || pl->use_chirp) {
    // The FFT attention kernels place the sparse spectrum (each bin k and its mirror -k) into an LDS array:
    // folded modulo the transform length Q (power-of-two kernel) or at k and M - k (chirp-z kernel).  Entries that
    // land on the same slot are added in separate rounds, so the kernels need no atomics and sum in a fixed order:
    // round = how many earlier entries of the layer already use that slot.
    const int64_t Q = pl->use_chirp ? pl->chirp_Q : (d->M < kFftMaxQ ? d->M : kFftMaxQ);
    std::vector<uint16_t> cnt((size_t)Q);
    for (int l = 0; l < d->n_layers && (pl->use_fft || pl->use_chirp); ++l) {
      std::fill(cnt.begin(), cnt.end(), 0);
      LayerInfo& L = pl->layers[l];
      int rounds = 0;
      for (int i = 0; i < L.nb; ++i) {
        const int64_t k = d->bins[L.bin_off + i];
        const int64_t r = k % Q, rm = (Q - r) % Q;
        const int fd = cnt[r]++;
        // a bin whose mirror falls on its own slot (k = 0 or Q/2 mod Q) adds both halves in one write:
        // its mirror byte is 0xff, "no round"
        const int fm = r == rm ? 0xff : cnt[rm]++;
        if (fd > 254 || (r != rm && fm > 254)) { pl->use_fft = pl->use_chirp = false; break; }
        pl->fold[L.bin_off + i] = (uint16_t)(fd | (fm << 8));
        if (fd + 1 > rounds) rounds = fd + 1;
        if (r != rm && fm + 1 > rounds) rounds = fm + 1;
      }
      L.fold_rounds = rounds;
    }
  }

  // What is left takes the direct O(M |B|) sums: fine for short or sparse states, useless beyond -- refuse instead of
  // running for minutes per step (a prime M of 2^20 with 4096 kept bins is 2^32 sine / cosine pairs per query head).
  if (!pl->use_fft && !pl->use_chirp && !(d->flags & IWDFT_FLAG_DIRECT_SYNTHESIS) &&
      (uint64_t)d->M * (uint64_t)pl->max_nb > kDirectMaxTerms)
    return fail(IWDFT_ERR_UNSUPPORTED,
                "M = %lld with %d kept bins in a layer has no O(M log M) decode attention (M is neither a power of two nor "
                "has a divisor Pb <= %d with 32 <= M / Pb <= %d) and is too large for the direct sums; pick M with such a "
                "divisor (e.g. move tokens to the sink / recent windows) or pass IWDFT_FLAG_DIRECT_SYNTHESIS to insist",
                (long long)d->M, pl->max_nb, (int)kChirpMaxBlocks, (int)kChirpMaxM);

  size_t o = 0;
  pl->off_layers = o;  o = align256(o + sizeof(LayerInfo) * (size_t)d->n_layers);
  pl->off_bins = o;    o = align256(o + sizeof(int32_t) * (size_t)pl->n_bins_total);
  pl->off_weights = o; o = align256(o + sizeof(float) * (size_t)pl->n_bins_total);
  pl->off_fold = o;    o = align256(o + sizeof(uint16_t) * (size_t)pl->n_bins_total);
  pl->off_chirp = o;   o = align256(o + (pl->use_chirp ? sizeof(float2) * (size_t)pl->chirp_Q : 0));
  pl->off_chirpH = o;  o = align256(o + (pl->use_chirp ? sizeof(float2) * ((size_t)1 << pl->chirp_logN) : 0));
  pl->tw_Q = (pow2 && (uint64_t)d->M >= kFftMinM) ? (d->M < kFftMaxQ ? d->M : kFftMaxQ) : 0;
  pl->off_tw = o;      o = align256(o + (pl->tw_Q ? sizeof(float2) * (size_t)(pl->tw_Q / 8 + 1) : 0));
  pl->off_FK = o;      o = align256(o + sizeof(float2) * (size_t)coef);
  pl->off_FV = o;      o = align256(o + sizeof(float2) * (size_t)coef);
  const size_t esz = d->kv_dtype == IWDFT_BF16 ? 2 : 4;
  const size_t n_sl = (size_t)d->n_layers * (size_t)slices_per_layer;
  pl->off_sinkK = o;   o = align256(o + esz * n_sl * (size_t)d->n_sink * kHeadDim);
  pl->off_sinkV = o;   o = align256(o + esz * n_sl * (size_t)d->n_sink * kHeadDim);
  pl->off_ringK = o;   o = align256(o + esz * n_sl * (size_t)d->n_recent * kHeadDim);
  pl->off_ringV = o;   o = align256(o + esz * n_sl * (size_t)d->n_recent * kHeadDim);
  pl->state_bytes = o;

  o = 0;
  pl->off_qc = o; o = align256(o + sizeof(float2) * (size_t)ws);
  pl->off_Pn = o; o = align256(o + sizeof(float2) * (size_t)ws);
  pl->off_pe = o; o = align256(o + sizeof(float) * n_sl * (size_t)pl->G * (size_t)(d->n_sink + d->n_recent));
  // Deferred write-back needs the FFT attention kernels (they weigh the pending tokens) and all
  // query heads of a KV head in one pass; otherwise every step writes back.
  pl->write_every = (d->write_every > 1 && pl->use_fft && pl->max_nb <= kFftMaxBins && heads_fit_one_pass(pl->G) &&
                     !(d->flags & IWDFT_FLAG_SHORTCUT))
                        ? (int)d->write_every
                        : 1;
  const size_t pend_rows = (d->n_recent || pl->write_every > 1) ? (size_t)pl->write_every : 0;
  pl->off_pendK = o; o = align256(o + esz * n_sl * pend_rows * kHeadDim);
  pl->off_pendV = o; o = align256(o + esz * n_sl * pend_rows * kHeadDim);
  pl->off_ps = o;    o = align256(o + (pl->write_every > 1 ? sizeof(float) * n_sl * (size_t)pl->G * kMaxPend : 0));
  pl->off_direct = o;
  if (!pl->use_fft && !pl->use_chirp)
    o = align256(o + sizeof(float) * (size_t)d->n_layers * (size_t)slices_per_layer *
                         (size_t)pl->G * (size_t)d->M);
  pl->ws_bytes = o;
  return IWDFT_OK;
}

// Tables of the chirp-z attention kernel, in double precision: c[a] = exp(+j pi a^2 / M) and the length-N
// transform (sign +) of h[n] = exp(-j pi n^2 / M), |n| < M, wrapped modulo N, divided by N and stored where the
// kernel's first in-LDS transform leaves entry m: base-4 digit-reversed position.
void make_chirp_tables(int64_t M, int logN, std::vector<float2>* chirp, std::vector<float2>* H) {
  const double kPi = 3.14159265358979323846;
  const int64_t N = (int64_t)1 << logN;
  chirp->resize((size_t)M);
  std::vector<std::complex<double>> h((size_t)N, 0.0);
  for (int64_t n = 0; n < M; ++n) {
    const double ph = kPi * (double)((n * n) % (2 * M)) / (double)M;  // exact phase reduction
    (*chirp)[(size_t)n] = make_float2((float)std::cos(ph), (float)std::sin(ph));
    const std::complex<double> v(std::cos(ph), -std::sin(ph));
    h[(size_t)n] = v;
    if (n) h[(size_t)(N - n)] = v;
  }
  // iterative radix-2 transform, sign +
  for (int64_t i = 1, j = 0; i < N; ++i) {
    int64_t bit = N >> 1;
    for (; j & bit; bit >>= 1) j ^= bit;
    j ^= bit;
    if (i < j) std::swap(h[(size_t)i], h[(size_t)j]);
  }
  for (int64_t len = 2; len <= N; len <<= 1) {
    for (int64_t i = 0; i < N; i += len)
      for (int64_t j = 0; j < len / 2; ++j) {
        const double a = 2.0 * kPi * (double)j / (double)len;
        const std::complex<double> w(std::cos(a), std::sin(a));
        const std::complex<double> u = h[(size_t)(i + j)], v = h[(size_t)(i + j + len / 2)] * w;
        h[(size_t)(i + j)] = u + v;
        h[(size_t)(i + j + len / 2)] = u - v;
      }
  }
  H->resize((size_t)N);
  for (int64_t m = 0; m < N; ++m) {
    int64_t p = 0;
    for (int t = 0; t < logN / 2; ++t) p |= ((m >> (2 * t)) & 3) << (logN - 2 * t - 2);
    (*H)[(size_t)p] = make_float2((float)(h[(size_t)m].real() / (double)N), (float)(h[(size_t)m].imag() / (double)N));
  }
}

}  // namespace

struct iwdft_ctx {
  iwdft_desc desc;  // host pointers inside are cleared after create
  Plan plan;
  Params P;
  int device = 0;
  int64_t T = 0;
  char* state = nullptr;
  char* ws = nullptr;
  int pend = 0;  // tokens counted in T that only the pending rows hold (deferred write-back), < write_every
  // phase timing (iwdft_phase_timing): events of the calls since the last read-out
  bool timing = false;
  std::vector<iwdft::PhaseEvents> marks;  // pool, reused after every read-out
  size_t marks_used = 0;
};

namespace {

int check_ctx(const iwdft_ctx* c) {
  if (!c) return fail(IWDFT_ERR_ARG, "ctx is NULL");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return fail(IWDFT_ERR_HIP, "hipGetDevice failed");
  if (dev != c->device)
    return fail(IWDFT_ERR_STATE, "context belongs to device %d but device %d is current", c->device,
                dev);
  return IWDFT_OK;
}

int launched(hipError_t e, const char* what) {
  if (e != hipSuccess) return fail(IWDFT_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return IWDFT_OK;
}

// Device address of this GPU's copy of `scratch`, looked up once per device with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(int dev, char** out) {
  if (dev < 0 || dev >= kMaxDevices) return fail(IWDFT_ERR_UNSUPPORTED, "device index %d beyond %d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return fail(IWDFT_ERR_HIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = (char*)g_scratch_ptr[dev];
  return IWDFT_OK;
}

// Next set of phase events of a timed call (created on demand), or null when timing is off.
int next_marks(iwdft_ctx* c, const PhaseEvents** out) {
  try {
    *out = nullptr;
    if (!c->timing) return IWDFT_OK;
    if (c->marks_used == c->marks.size()) {
      PhaseEvents m;
      for (int i = 0; i < 4; ++i) {
        hipError_t e = hipEventCreate(&m.ev[i]);
        if (e != hipSuccess) {
          for (int j = 0; j < i; ++j) (void)hipEventDestroy(m.ev[j]);
          return fail(IWDFT_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
        }
      }
      c->marks.push_back(m);
    }
    *out = &c->marks[c->marks_used++];
    return IWDFT_OK;

  } catch (...) {  // std::bad_alloc from the host-side containers: nothing may cross the C ABI
    return fail(IWDFT_ERR_ARG, "out of host memory");
  }
}

bool shortcut(const iwdft_ctx* c) { return (c->desc.flags & IWDFT_FLAG_SHORTCUT) != 0; }

// Readers of the coefficients: gain T / M with the Sec. 4.1 shortcut (the stored state is then M S_T, not T S_T).
void set_read_gain(iwdft_ctx* c) {
  c->P.gain = shortcut(c) ? (float)((double)c->T / (double)c->desc.M) : 1.0f;
}

uint32_t t_shift(const iwdft_ctx* c) {  // (T - M) mod M
  return (uint32_t)((c->T - c->desc.M) % c->desc.M);
}

// Writes the tokens that the fused decode step has deferred into the coefficients, oldest first, one
// streaming update each (the rare path: a call other than the fused step arrived in between).
int flush_pending(iwdft_ctx* c, hipStream_t st) {
  if (c->pend == 0) return IWDFT_OK;
  const Plan& pl = c->plan;
  const size_t esz = c->desc.kv_dtype == IWDFT_BF16 ? 2 : 4;
  for (int j = 0; j < c->pend; ++j) {
    const uint32_t tsh = (uint32_t)((c->T - c->pend + j - c->desc.M) % c->desc.M);
    hipError_t e = launch_absorb(c->P, c->ws + pl.off_pendK + (size_t)j * kHeadDim * esz,
                                 c->ws + pl.off_pendV + (size_t)j * kHeadDim * esz,
                                 (int64_t)pl.write_every * kHeadDim, tsh, st);
    if (e != hipSuccess) return fail(IWDFT_ERR_HIP, "write-back of deferred tokens: %s", hipGetErrorString(e));
  }
  c->pend = 0;
  return IWDFT_OK;
}

}  // namespace

extern "C" {

const char* iwdft_last_error(void) { return g_err; }

int iwdft_query_bytes(const iwdft_desc* desc, size_t* state_bytes, size_t* workspace_bytes) {
  try {
    if (!state_bytes || !workspace_bytes) return fail(IWDFT_ERR_ARG, "output pointer is NULL");
    Plan pl;
    int rc = make_plan(desc, &pl);
    if (rc != IWDFT_OK) return rc;
    *state_bytes = pl.state_bytes;
    *workspace_bytes = pl.ws_bytes < 256 ? 256 : pl.ws_bytes;
    return IWDFT_OK;

  } catch (...) {  // std::bad_alloc from the host-side containers: nothing may cross the C ABI
    return fail(IWDFT_ERR_ARG, "out of host memory");
  }
}

int iwdft_create(const iwdft_desc* desc, void* d_state, size_t state_bytes, void* d_workspace,
                 size_t workspace_bytes, iwdft_ctx** out) {
  try {
    if (!out) return fail(IWDFT_ERR_ARG, "out is NULL");
    *out = nullptr;
    std::unique_ptr<iwdft_ctx> c(new iwdft_ctx());  // freed on every early return and on exceptions
    int rc = make_plan(desc, &c->plan);
    if (rc != IWDFT_OK) return rc;
    const Plan& pl = c->plan;
    size_t need_ws = pl.ws_bytes < 256 ? 256 : pl.ws_bytes;
    if (!d_state || !d_workspace) { return fail(IWDFT_ERR_ARG, "d_state / d_workspace is NULL"); }
    if (((uintptr_t)d_state & 255) || ((uintptr_t)d_workspace & 255)) {
      return fail(IWDFT_ERR_ARG, "d_state and d_workspace must be 256-byte aligned");
    }
    if (state_bytes < pl.state_bytes) {
      return fail(IWDFT_ERR_SIZE, "state buffer has %zu bytes, %zu needed", state_bytes, pl.state_bytes);
    }
    if (workspace_bytes < need_ws) {
      return fail(IWDFT_ERR_SIZE, "workspace has %zu bytes, %zu needed", workspace_bytes, need_ws);
    }
    c->desc = *desc;
    c->state = (char*)d_state;
    c->ws = (char*)d_workspace;
    if (hipGetDevice(&c->device) != hipSuccess) { return fail(IWDFT_ERR_HIP, "hipGetDevice failed"); }
    {  // set-up of compressed_decode_attn_static: this device's scratch address (a failure is reported by that call)
      char* unused = nullptr;
      (void)static_scratch(c->device, &unused);
    }

    // Device copies of geometry, bins and weights live at the head of the state buffer.
    std::vector<float> w((size_t)pl.n_bins_total, 1.0f);
    if (desc->bin_weights) memcpy(w.data(), desc->bin_weights, sizeof(float) * w.size());
    hipError_t e = hipMemset(c->state, 0, pl.state_bytes);
    if (e == hipSuccess)
      e = hipMemcpy(c->state + pl.off_layers, pl.layers.data(), sizeof(LayerInfo) * pl.layers.size(),
                    hipMemcpyHostToDevice);
    if (e == hipSuccess)
      e = hipMemcpy(c->state + pl.off_bins, desc->bins, sizeof(int32_t) * (size_t)pl.n_bins_total,
                    hipMemcpyHostToDevice);
    if (e == hipSuccess)
      e = hipMemcpy(c->state + pl.off_weights, w.data(), sizeof(float) * w.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess)
      e = hipMemcpy(c->state + pl.off_fold, pl.fold.data(), sizeof(uint16_t) * pl.fold.size(),
                    hipMemcpyHostToDevice);
    if (e == hipSuccess && pl.use_chirp) {
      std::vector<float2> chirp, H;
      make_chirp_tables(pl.chirp_Q, pl.chirp_logN, &chirp, &H);
      e = hipMemcpy(c->state + pl.off_chirp, chirp.data(), sizeof(float2) * chirp.size(), hipMemcpyHostToDevice);
      if (e == hipSuccess)
        e = hipMemcpy(c->state + pl.off_chirpH, H.data(), sizeof(float2) * H.size(), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess && pl.tw_Q) {
      const double kTwoPi = 6.28318530717958647692;
      std::vector<float2> tw((size_t)(pl.tw_Q / 8 + 1));
      for (size_t m = 0; m < tw.size(); ++m) {
        const double ph = kTwoPi * (double)m / (double)pl.tw_Q;
        tw[m] = make_float2((float)std::cos(ph), (float)std::sin(ph));
      }
      e = hipMemcpy(c->state + pl.off_tw, tw.data(), sizeof(float2) * tw.size(), hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
      return fail(IWDFT_ERR_HIP, "initialising the state buffer: %s", hipGetErrorString(e));
    }
    c->desc.bin_offsets = nullptr;
    c->desc.bins = nullptr;
    c->desc.bin_weights = nullptr;

    Params& P = c->P;
    P.n_layers = desc->n_layers;
    P.batch = desc->batch;
    P.n_kv = desc->n_kv_heads;
    P.G = pl.G;
    P.n_slices = desc->n_layers * desc->batch * desc->n_kv_heads;
    P.kv_dtype = desc->kv_dtype;
    P.M = (uint32_t)desc->M;
    P.Mmask = ((desc->M & (desc->M - 1)) == 0) ? (uint32_t)(desc->M - 1) : 0u;
    if (desc->M == 1) P.Mmask = 0;  // M = 1: "mod 1" through the generic path
    P.max_nb = pl.max_nb;
    P.max_Bp = pl.max_Bp;
    P.layers = (const LayerInfo*)(c->state + pl.off_layers);
    P.bins = (const int32_t*)(c->state + pl.off_bins);
    P.weights = (const float*)(c->state + pl.off_weights);
    P.fold = (const uint16_t*)(c->state + pl.off_fold);
    P.chirp = pl.use_chirp ? (const float2*)(c->state + pl.off_chirp) : nullptr;
    P.chirpH = pl.use_chirp ? (const float2*)(c->state + pl.off_chirpH) : nullptr;
    P.chirp_logN = pl.chirp_logN;
    P.chirp_Q = (uint32_t)pl.chirp_Q;
    P.tw8 = pl.tw_Q ? (const float2*)(c->state + pl.off_tw) : nullptr;
    P.FK = (float2*)(c->state + pl.off_FK);
    P.FV = (float2*)(c->state + pl.off_FV);
    P.gain = 1.0f;
    P.x_scale = 1.0f;
    P.serial_phases = (desc->flags & IWDFT_FLAG_SERIAL_PHASES) ? 1 : 0;
    P.S = desc->n_sink;
    P.R = desc->n_recent;
    P.sinkK = c->state + pl.off_sinkK;
    P.sinkV = c->state + pl.off_sinkV;
    P.ringK = c->state + pl.off_ringK;
    P.ringV = c->state + pl.off_ringV;
    c->T = 0;
    *out = c.release();
    return IWDFT_OK;

  } catch (...) {  // std::bad_alloc from the host-side containers: nothing may cross the C ABI
    return fail(IWDFT_ERR_ARG, "out of host memory");
  }
}

int iwdft_destroy(iwdft_ctx* ctx) {
  if (ctx)
    for (auto& m : ctx->marks)
      for (int i = 0; i < 4; ++i) (void)hipEventDestroy(m.ev[i]);
  delete ctx;
  return IWDFT_OK;
}

int iwdft_phase_timing(iwdft_ctx* ctx, int enable) {
  int rc = check_ctx(ctx);
  if (rc != IWDFT_OK) return rc;
  ctx->timing = enable != 0;
  return IWDFT_OK;
}

int iwdft_phase_times(iwdft_ctx* ctx, double* ms, int64_t* n_calls) {
  int rc = check_ctx(ctx);
  if (rc != IWDFT_OK) return rc;
  if (!ms || !n_calls) return fail(IWDFT_ERR_ARG, "ms / n_calls is NULL");
  ms[0] = ms[1] = ms[2] = 0.0;
  *n_calls = 0;
  for (size_t i = 0; i < ctx->marks_used; ++i) {
    const PhaseEvents& m = ctx->marks[i];
    hipError_t e = hipEventSynchronize(m.ev[3]);
    for (int p = 0; p < 3 && e == hipSuccess; ++p) {
      float t = 0.f;
      e = hipEventElapsedTime(&t, m.ev[p], m.ev[p + 1]);
      ms[p] += t;
    }
    if (e != hipSuccess) {
      ctx->marks_used = 0;
      return fail(IWDFT_ERR_HIP, "reading phase events: %s", hipGetErrorString(e));
    }
  }
  *n_calls = (int64_t)ctx->marks_used;
  ctx->marks_used = 0;
  return IWDFT_OK;
}

int64_t iwdft_num_tokens(const iwdft_ctx* ctx) { return ctx ? ctx->T : -1; }

int iwdft_prefill_kind(const iwdft_ctx* ctx) { return ctx ? (ctx->plan.use_fft_prefill ? 1 : 0) : -1; }

int iwdft_attn_pipelined(const iwdft_ctx* ctx) { return ctx ? (attn_pipelines(ctx->P, ctx->plan.use_fft) ? 1 : 0) : -1; }

int iwdft_attn_kind(const iwdft_ctx* ctx) { return ctx ? (ctx->plan.use_fft ? 1 : (ctx->plan.use_chirp ? 2 : 0)) : -1; }

int iwdft_set_num_tokens(iwdft_ctx* ctx, int64_t T) {
  if (!ctx) return fail(IWDFT_ERR_ARG, "ctx is NULL");
  if (T < ctx->desc.M) return fail(IWDFT_ERR_ARG, "T = %lld is below M", (long long)T);
  ctx->T = T;
  ctx->pend = 0;  // the restored buffer is taken as complete
  return IWDFT_OK;
}

int iwdft_prefill(iwdft_ctx* ctx, const void* d_K, const void* d_V, void* hip_stream) {
  int rc = check_ctx(ctx);
  if (rc != IWDFT_OK) return rc;
  if (!d_K || !d_V) return fail(IWDFT_ERR_ARG, "d_K / d_V is NULL");
  {
    // the FFT prefill without sink / recent windows falls back to narrower loads; it still needs whole channel pairs
    const bool narrow_ok = ctx->plan.use_fft_prefill && ctx->desc.n_sink == 0 && ctx->desc.n_recent == 0;
    const uintptr_t mask = narrow_ok ? (ctx->desc.kv_dtype == IWDFT_BF16 ? 3u : 7u) : 15u;
    if ((((uintptr_t)d_K | (uintptr_t)d_V) & mask) != 0)
      return fail(IWDFT_ERR_ARG, "d_K / d_V must be %u-byte aligned for this prefill", (unsigned)mask + 1);
  }
  ctx->pend = 0;  // the prefill overwrites the whole state
  rc = launched(ctx->plan.use_fft_prefill ? launch_prefill_fft(ctx->P, d_K, d_V, (hipStream_t)hip_stream)
                                          : launch_prefill(ctx->P, d_K, d_V, (hipStream_t)hip_stream),
                "prefill launch");
  if (rc != IWDFT_OK) return rc;
  ctx->T = ctx->desc.M;
  return IWDFT_OK;
}

int iwdft_append(iwdft_ctx* ctx, const void* d_tok_k, const void* d_tok_v, void* hip_stream) {
  int rc = check_ctx(ctx);
  if (rc != IWDFT_OK) return rc;
  if (!d_tok_k || !d_tok_v) return fail(IWDFT_ERR_ARG, "d_tok_k / d_tok_v is NULL");
  if (misaligned16(d_tok_k) || misaligned16(d_tok_v)) return fail(IWDFT_ERR_ARG, kAlignMsg);
  if (ctx->T < ctx->desc.M) return fail(IWDFT_ERR_STATE, "iwdft_append before iwdft_prefill");
  if ((rc = flush_pending(ctx, (hipStream_t)hip_stream)) != IWDFT_OK) return rc;
  // The recent ring was filled oldest-first at prefill, so after T - M appends the oldest token
  // sits in slot (T - M) mod R.
  const uint32_t ring_pos = ctx->P.R ? (uint32_t)((ctx->T - ctx->desc.M) % ctx->P.R) : 0u;
  // Sec. 4.1 shortcut: S <- W (S + x / (T + 1)); on the stored M S_T that is the exact update of x M / (T + 1).
  ctx->P.x_scale = shortcut(ctx) ? (float)((double)ctx->desc.M / (double)(ctx->T + 1)) : 1.0f;
  rc = launched(launch_append(ctx->P, d_tok_k, d_tok_v, t_shift(ctx), ring_pos, (hipStream_t)hip_stream),
                "append launch");
  ctx->P.x_scale = 1.0f;
  if (rc != IWDFT_OK) return rc;
  ctx->T += 1;
  return IWDFT_OK;
}

int iwdft_export_coeffs(iwdft_ctx* ctx, int32_t layer, float* d_SK, float* d_SV, void* hip_stream) {
  int rc = check_ctx(ctx);
  if (rc != IWDFT_OK) return rc;
  if (layer < 0 || layer >= ctx->desc.n_layers) return fail(IWDFT_ERR_ARG, "layer %d out of range", layer);
  if (ctx->T < ctx->desc.M) return fail(IWDFT_ERR_STATE, "iwdft_export_coeffs before iwdft_prefill");
  if (!d_SK && !d_SV) return IWDFT_OK;
  if ((rc = flush_pending(ctx, (hipStream_t)hip_stream)) != IWDFT_OK) return rc;
  return launched(launch_export(ctx->P, layer, d_SK, d_SV, t_shift(ctx),
                                (float)(1.0 / (double)(shortcut(ctx) ? ctx->desc.M : ctx->T)),
                                (hipStream_t)hip_stream),
                  "export launch");
}

int iwdft_export_bins(iwdft_ctx* ctx, int32_t layer, int32_t* d_bins, void* hip_stream) {
  int rc = check_ctx(ctx);
  if (rc != IWDFT_OK) return rc;
  if (layer < 0 || layer >= ctx->desc.n_layers) return fail(IWDFT_ERR_ARG, "layer %d out of range", layer);
  if (!d_bins) return fail(IWDFT_ERR_ARG, "d_bins is NULL");
  const LayerInfo& L = ctx->plan.layers[layer];
  return launched(hipMemcpyAsync(d_bins, ctx->P.bins + L.bin_off, sizeof(int32_t) * (size_t)L.nb,
                                 hipMemcpyDeviceToDevice, (hipStream_t)hip_stream),
                  "export bins");
}

int iwdft_reconstruct_grid(iwdft_ctx* ctx, int32_t layer, int64_t a0, int64_t stride, int64_t n_slots, void* d_Kt,
                           void* d_Vt, void* hip_stream) {
  int rc = check_ctx(ctx);
  if (rc != IWDFT_OK) return rc;
  if (layer < 0 || layer >= ctx->desc.n_layers) return fail(IWDFT_ERR_ARG, "layer %d out of range", layer);
  if (stride < 1 || stride > ctx->desc.M) return fail(IWDFT_ERR_ARG, "stride %lld outside [1, M]", (long long)stride);
  if (a0 < 0 || n_slots < 0 || a0 > ctx->desc.M || (n_slots > 0 && a0 + (n_slots - 1) * stride >= ctx->desc.M))
    return fail(IWDFT_ERR_ARG, "slots %lld + %lld * [0, %lld) outside [0, M)", (long long)a0, (long long)stride,
                (long long)n_slots);
  if (ctx->T < ctx->desc.M) return fail(IWDFT_ERR_STATE, "iwdft_reconstruct before iwdft_prefill");
  if (n_slots == 0 || (!d_Kt && !d_Vt)) return IWDFT_OK;
  if ((rc = flush_pending(ctx, (hipStream_t)hip_stream)) != IWDFT_OK) return rc;
  set_read_gain(ctx);
  return launched(launch_reconstruct(ctx->P, layer, (uint32_t)a0, (uint32_t)stride, (uint32_t)n_slots, d_Kt, d_Vt,
                                     t_shift(ctx), ctx->plan.use_fft, (hipStream_t)hip_stream),
                  "reconstruct launch");
}

int iwdft_reconstruct(iwdft_ctx* ctx, int32_t layer, int64_t a0, int64_t n_slots, void* d_Kt, void* d_Vt,
                      void* hip_stream) {
  if (ctx && (a0 < 0 || n_slots < 0 || a0 + n_slots > ctx->desc.M))
    return fail(IWDFT_ERR_ARG, "slots [%lld, %lld) outside [0, M)", (long long)a0, (long long)(a0 + n_slots));
  return iwdft_reconstruct_grid(ctx, layer, a0, 1, n_slots, d_Kt, d_Vt, hip_stream);
}

int compressed_decode_attn(iwdft_ctx* ctx, const void* d_q, void* d_out, float scale, void* hip_stream) {
  int rc = check_ctx(ctx);
  if (rc != IWDFT_OK) return rc;
  if (!d_q || !d_out) return fail(IWDFT_ERR_ARG, "d_q / d_out is NULL");
  if (misaligned16(d_q) || misaligned16(d_out)) return fail(IWDFT_ERR_ARG, kAlignMsg);
  if (ctx->T < ctx->desc.M) return fail(IWDFT_ERR_STATE, "compressed_decode_attn before iwdft_prefill");
  if (!std::isfinite(scale)) return fail(IWDFT_ERR_ARG, "scale is not finite");
  if (scale <= 0.0f) scale = 1.0f / std::sqrt((float)ctx->desc.head_dim);
  if ((rc = flush_pending(ctx, (hipStream_t)hip_stream)) != IWDFT_OK) return rc;
  const Plan& pl = ctx->plan;
  const PhaseEvents* marks = nullptr;
  if ((rc = next_marks(ctx, &marks)) != IWDFT_OK) return rc;
  set_read_gain(ctx);
  return launched(launch_attn(ctx->P, d_q, d_out, scale, (float2*)(ctx->ws + pl.off_qc),
                              (float2*)(ctx->ws + pl.off_Pn), (float*)(ctx->ws + pl.off_pe),
                              (float*)(ctx->ws + pl.off_direct),
                              pl.use_fft, marks, (hipStream_t)hip_stream),
                  "decode attention launch");
}

int compressed_decode_attn_static(iwdft_ctx* ctx, const void* d_q, void* d_out, float scale, void* hip_stream) {
  int rc = check_ctx(ctx);
  if (rc != IWDFT_OK) return rc;
  if (!d_q || !d_out) return fail(IWDFT_ERR_ARG, "d_q / d_out is NULL");
  if (misaligned16(d_q) || misaligned16(d_out)) return fail(IWDFT_ERR_ARG, kAlignMsg);
  if (ctx->T < ctx->desc.M) return fail(IWDFT_ERR_STATE, "compressed_decode_attn_static before iwdft_prefill");
  if (!std::isfinite(scale)) return fail(IWDFT_ERR_ARG, "scale is not finite");
  if (scale <= 0.0f) scale = 1.0f / std::sqrt((float)ctx->desc.head_dim);
  const Plan& pl = ctx->plan;
  // Same arrays as the workspace form, laid out inside the library's scratch: qc | Pn | pe | direct scores.
  const size_t n_heads = (size_t)ctx->P.n_slices * (size_t)pl.G;
  const size_t rows = align256(sizeof(float2) * (size_t)pl.ws_total);
  const size_t pe_bytes = align256(sizeof(float) * n_heads * (size_t)(ctx->P.S + ctx->P.R));
  const size_t direct_bytes = (pl.use_fft || pl.use_chirp) ? 0 : align256(sizeof(float) * n_heads * (size_t)ctx->desc.M);
  const size_t need = 2 * rows + pe_bytes + direct_bytes;
  if (need > kStaticScratchBytes)
    return fail(IWDFT_ERR_SIZE, "compressed_decode_attn_static needs %zu bytes of scratch, the library holds %zu", need,
                kStaticScratchBytes);
  char* sc = nullptr;
  if ((rc = static_scratch(ctx->device, &sc)) != IWDFT_OK) return rc;
  if ((rc = flush_pending(ctx, (hipStream_t)hip_stream)) != IWDFT_OK) return rc;
  set_read_gain(ctx);
  // Every entry of the four arrays is written by the kernels before it is read, so nothing needs clearing
  // although the scratch still holds the previous call's contents.
  return launched(launch_attn(ctx->P, d_q, d_out, scale, (float2*)sc, (float2*)(sc + rows), (float*)(sc + 2 * rows),
                              (float*)(sc + 2 * rows + pe_bytes), pl.use_fft, nullptr, (hipStream_t)hip_stream),
                  "decode attention launch (static scratch)");
}

int iwdft_append_attn(iwdft_ctx* ctx, const void* d_tok_k, const void* d_tok_v, const void* d_q, void* d_out,
                      float scale, void* hip_stream) {
  int rc = check_ctx(ctx);
  if (rc != IWDFT_OK) return rc;
  if (!d_tok_k || !d_tok_v || !d_q || !d_out) return fail(IWDFT_ERR_ARG, "a token / query / output pointer is NULL");
  if (misaligned16(d_tok_k) || misaligned16(d_tok_v) || misaligned16(d_q) || misaligned16(d_out))
    return fail(IWDFT_ERR_ARG, kAlignMsg);
  if (ctx->T < ctx->desc.M) return fail(IWDFT_ERR_STATE, "iwdft_append_attn before iwdft_prefill");
  if (!std::isfinite(scale)) return fail(IWDFT_ERR_ARG, "scale is not finite");
  if (scale <= 0.0f) scale = 1.0f / std::sqrt((float)ctx->desc.head_dim);
  if (!step_can_fuse(ctx->P) || shortcut(ctx)) {  // more query heads per KV head than one pass holds, or the
                                                  // shortcut's per-token scale: plain sequence
    rc = iwdft_append(ctx, d_tok_k, d_tok_v, hip_stream);
    if (rc != IWDFT_OK) return rc;
    return compressed_decode_attn(ctx, d_q, d_out, scale, hip_stream);
  }
  const Plan& pl = ctx->plan;
  const uint32_t ring_pos = ctx->P.R ? (uint32_t)((ctx->T - ctx->desc.M) % ctx->P.R) : 0u;
  const PhaseEvents* marks = nullptr;
  if ((rc = next_marks(ctx, &marks)) != IWDFT_OK) return rc;
  const uint32_t tsh0 = (uint32_t)((ctx->T - ctx->pend - ctx->desc.M) % ctx->desc.M);  // oldest pending token
  rc = launched(launch_step(ctx->P, d_tok_k, d_tok_v, d_q, d_out, scale, (float2*)(ctx->ws + pl.off_qc),
                            (float2*)(ctx->ws + pl.off_Pn), (float*)(ctx->ws + pl.off_pe),
                            ctx->ws + pl.off_pendK, ctx->ws + pl.off_pendV, (float*)(ctx->ws + pl.off_ps),
                            (float*)(ctx->ws + pl.off_direct), pl.use_fft, tsh0, ring_pos, ctx->pend,
                            pl.write_every, marks, (hipStream_t)hip_stream),
                "fused decode step launch");
  if (rc != IWDFT_OK) return rc;
  ctx->pend = (ctx->pend + 1) % pl.write_every;  // back to 0: this step wrote the coefficients
  ctx->T += 1;
  return IWDFT_OK;
}

int iwdft_flush(iwdft_ctx* ctx, void* hip_stream) {
  int rc = check_ctx(ctx);
  if (rc != IWDFT_OK) return rc;
  return flush_pending(ctx, (hipStream_t)hip_stream);
}

int iwdft_select_bins(const float* delta, int32_t n_layers, int32_t n_chunks, int64_t M, double r,
                      int64_t* bin_offsets, int32_t* bins, int64_t bins_capacity) {
  try {
    if (!delta || !bin_offsets) return fail(IWDFT_ERR_ARG, "delta / bin_offsets is NULL");
    if (n_layers <= 0 || n_chunks <= 0) return fail(IWDFT_ERR_ARG, "n_layers and n_chunks must be positive");
    if (M < 1 || M > ((int64_t)1 << 30)) return fail(IWDFT_ERR_ARG, "M = %lld outside [1, 2^30]", (long long)M);
    if (!(r >= 0.0) || !std::isfinite(r)) return fail(IWDFT_ERR_ARG, "retention ratio must be finite and >= 0");
    if (bins_capacity < 0 || (bins_capacity > 0 && !bins)) return fail(IWDFT_ERR_ARG, "bins is NULL");
    std::vector<int> keep;
    int64_t total = 0;
    bin_offsets[0] = 0;
    for (int l = 0; l < n_layers; ++l) {
      if (select_chunks(delta + (size_t)l * n_chunks, n_chunks, r, &keep) != 0)
        return fail(IWDFT_ERR_ARG, "delta of layer %d holds a NaN", l);
      for (int c : keep) {
        const int64_t a = chunk_edge(c, M, n_chunks), b = chunk_edge(c + 1, M, n_chunks);
        for (int64_t k = a; k < b; ++k, ++total)
          if (total < bins_capacity) bins[total] = (int32_t)k;
      }
      bin_offsets[l + 1] = total;
    }
    if (total > bins_capacity)
      return fail(IWDFT_ERR_SIZE, "bins holds %lld entries, %lld needed", (long long)bins_capacity, (long long)total);
    for (int l = 0; l < n_layers; ++l)
      if (bin_offsets[l + 1] == bin_offsets[l])
        return fail(IWDFT_ERR_BINS, "layer %d keeps no bin (M smaller than the number of chunks)", l);
    return IWDFT_OK;

  } catch (...) {  // std::bad_alloc from the host-side containers: nothing may cross the C ABI
    return fail(IWDFT_ERR_ARG, "out of host memory");
  }
}

int iwdft_ablate_chunk(const void* d_x, void* d_out, int64_t n_slices, int64_t M, int32_t head_dim,
                       int32_t kv_dtype, int32_t n_chunks, int32_t chunk, void* hip_stream) {
  if (!d_x || !d_out) return fail(IWDFT_ERR_ARG, "d_x / d_out is NULL");
  if (n_slices < 0 || n_slices > 0x3fffff) return fail(IWDFT_ERR_ARG, "n_slices = %lld out of range", (long long)n_slices);
  if (kv_dtype != IWDFT_F32 && kv_dtype != IWDFT_BF16) return fail(IWDFT_ERR_ARG, "bad kv_dtype %d", kv_dtype);
  if (n_chunks <= 0 || chunk < 0 || chunk >= n_chunks)
    return fail(IWDFT_ERR_ARG, "chunk %d outside [0, %d)", chunk, n_chunks);
  if (M < 1) return fail(IWDFT_ERR_ARG, "M must be positive");
  if (head_dim != kHeadDim) return fail(IWDFT_ERR_UNSUPPORTED, "head_dim %d: this build handles 128", head_dim);
  if ((M & (M - 1)) != 0 || M < (int64_t)kFftMinM || M > ((int64_t)1 << 24))
    return fail(IWDFT_ERR_UNSUPPORTED, "iwdft_ablate_chunk needs M = 2^m with 256 <= M <= 2^24 (got %lld)",
                (long long)M);
  const size_t esz = kv_dtype == IWDFT_BF16 ? 2 : 4;
  const size_t bytes = (size_t)n_slices * (size_t)M * kHeadDim * esz;
  const char *a = (const char*)d_x, *b = (const char*)d_out;
  if (a < b + bytes && b < a + bytes && bytes) return fail(IWDFT_ERR_ARG, "d_x and d_out overlap");
  if (n_slices == 0) return IWDFT_OK;
  return launched(launch_ablate(d_x, d_out, (int)n_slices, (uint32_t)M, kv_dtype,
                                (int)chunk_edge(chunk, M, n_chunks), (int)chunk_edge(chunk + 1, M, n_chunks),
                                (hipStream_t)hip_stream),
                  "ablation launch");
}

}  // extern "C"
