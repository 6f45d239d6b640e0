/*
 * libiwdft -- the Infinite-Window DFT (IWDFT) K/V-cache hot path of FAEDKV
 * (arxiv 2507.20030) for AMD MI355X (gfx950).  C ABI, plain pointers and sizes.
 *
 * One *slice* is one (layer, sequence, KV head).  Along the token axis every
 * channel of K and of V is a real signal x[n].  With M the DFT length fixed at
 * prefill, T the number of tokens absorbed so far and W_k = exp(-j 2 pi k / M),
 * the library keeps, for every kept bin k of the layer, the coefficient
 *
 *     S_T[k] = (1/T) * U_T[k],
 *     U_M[k]     = sum_{n<M} x[n] W_k^n                  (Sec. 3.1.2, Eq. dft-full;
 *                                                        Sec. 4.2.1, Eq. prefill-dft)
 *     S_{T+1}[k] = W_k ( T/(T+1) S_T[k] + x_T/(T+1) )    (Sec. 4.1, Eq. infi-dft)
 *
 * so every token ever seen contributes with weight exactly 1/T.  Only kept
 * bins are computed or stored (Sec. 3.2 Eq. freq-zero; Sec. 4.2.2 "Updating
 * Cache").  The state is reconstructed with the inverse DFT over the kept bins
 * (Sec. 3.1.2 Eq. inverse-swdft; Sec. 4.2.2 Eq. reconstruct-idft) and consumed
 * by softmax attention (Sec. 3.1.1 Eq. kv-attn; Sec. 4.2.2 Eq. kv-concat, middle
 * segment).
 *
 * Memory: every d_* pointer is DEVICE memory owned by the caller; the library
 * never allocates or frees device memory.  Pointers inside iwdft_desc are HOST
 * memory and are copied by iwdft_create.  Hot calls (prefill, append,
 * reconstruct, attention, export) only enqueue kernels on the given HIP stream
 * (a hipStream_t passed as void*, NULL = default stream) and never synchronise;
 * T advances when the call is enqueued.  Calls on one context from several host
 * threads, or on different streams without caller-side ordering, race.
 * Alignment: token, query, attention-output and prefill tensors must be 16-byte
 * aligned (IWDFT_ERR_ARG otherwise); the FFT prefill of a context without sink /
 * recent windows also takes K, V aligned to one channel pair (4 bytes bf16, 8 fp32).
 *
 * Errors: every call returns IWDFT_OK or a negative code, validates all
 * arguments before launching anything, and never throws or aborts.
 * iwdft_last_error() returns a thread-local description of the last failure.
 *
 * Dtypes: K, V, appended tokens, queries, attention output and reconstruction
 * output share desc.kv_dtype (fp32 or bf16, round-to-nearest-even on output);
 * coefficients are complex fp32 and all arithmetic accumulates in fp32.
 */
#ifndef IWDFT_H_
#define IWDFT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct iwdft_ctx iwdft_ctx; /* opaque, host memory, owned by the library */

enum {
  IWDFT_OK = 0,
  IWDFT_ERR_ARG = -1,         /* null pointer, non-positive dimension, bad dtype ...   */
  IWDFT_ERR_BINS = -2,        /* bins not strictly increasing / out of [0,M) / empty   */
  IWDFT_ERR_SIZE = -3,        /* state or workspace buffer smaller than queried        */
  IWDFT_ERR_STATE = -4,       /* call out of order (e.g. append before prefill)        */
  IWDFT_ERR_HIP = -5,         /* a HIP runtime call or kernel launch failed            */
  IWDFT_ERR_UNSUPPORTED = -6  /* valid request this build has no kernel for            */
};

enum { IWDFT_F32 = 0, IWDFT_BF16 = 1 };

/* desc.flags */
enum {
  IWDFT_FLAG_DIRECT_SYNTHESIS = 1u, /* decode attention evaluates the O(M*|B|) sums
                                       directly instead of through FFTs (see
                                       iwdft_attn_kind for what runs otherwise)    */
  IWDFT_FLAG_DENSE_PREFILL = 2u,    /* iwdft_prefill always runs the dense contraction
                                       at the kept bins (matrix cores).  Its operands
                                       are fp16 pairs: inputs must lie within +-65504,
                                       bf16 inputs below 2^-14 in magnitude lose bits
                                       (below 2^-24 they count as 0), fp32 inputs keep
                                       ~21 bits down to 2^-14 and an absolute 2^-25
                                       below.  The FFT prefill has no such limits.   */
  IWDFT_FLAG_FFT_PREFILL = 4u,      /* iwdft_prefill always runs FFTs + pruning; needs
                                       M = 2^m >= 256, else IWDFT_ERR_UNSUPPORTED (layers
                                       with more than 4096 kept bins take a form that
                                       keeps nothing per bin in registers).  With neither flag
                                       the library picks: FFT when it applies and some
                                       layer keeps >= 384 bins                     */
  IWDFT_FLAG_SHORTCUT = 8u,         /* the variant of the update that Sec. 4.1 mentions for long
                                       contexts, the factor (N-1)/N of Eq. infi-dft taken as 1:
                                       S_{T+1}[k] = W_k ( S_T[k] + x_T / (T+1) ).  Tokens no longer
                                       weigh the same (prefill tokens keep 1/M, token n enters with
                                       1/(n+1)); reconstruction and attention read the state as they
                                       read S_T otherwise (gain T/M).  iwdft_append_attn then runs
                                       its two calls in sequence and write_every is taken as 1.    */
  IWDFT_FLAG_SERIAL_PHASES = 16u    /* decode attention (Sec. 4.2.2 "Calculating Attention") always runs
                                       its three kernels one after the other.  Without the flag, long
                                       contexts with many slices (M >= 16384, >= 2048 pairs of query
                                       heads in all, more than 1024 kept bins in some layer, 4 or 8 query
                                       heads per pass) walk the slices in groups and put the transforms
                                       of one group into the same launches as the K-coefficient stream of
                                       the next.  Same arithmetic, same results bit for bit.          */
};

typedef struct {
  int32_t n_layers;
  int32_t batch;
  int32_t n_kv_heads;
  int32_t n_q_heads;          /* multiple of n_kv_heads; query head hq reads KV head
                                 hq / (n_q_heads / n_kv_heads)                      */
  int32_t head_dim;           /* this build: 128                                    */
  int32_t kv_dtype;           /* IWDFT_F32 or IWDFT_BF16                            */
  int64_t M;                  /* DFT length = tokens given to iwdft_prefill,
                                 1 <= M <= 2^30                                     */
  const int64_t* bin_offsets; /* HOST [n_layers+1], bin_offsets[0] = 0; layer l keeps
                                 bins[bin_offsets[l] .. bin_offsets[l+1])           */
  const int32_t* bins;        /* HOST, per layer strictly increasing, each in [0,M) */
  const float* bin_weights;   /* HOST, same indexing as bins, or NULL (= all 1).
                                 w_k multiplies bin k in every inverse transform;
                                 w = 2 for 0 < k < M/2 with bins <= M/2 gives the
                                 one-sided (real-signal) synthesis                  */
  uint32_t flags;
  int32_t n_sink;             /* S >= 0: first S prefill tokens kept exact (attention sinks) */
  int32_t n_recent;           /* R >= 0: the R newest tokens kept exact (recent window);
                                 S + R <= 1024                                         */
  uint32_t write_every;       /* J: iwdft_append_attn writes the coefficients back on every J-th call only
                                 (0 or 1: on every call; at most 16); see iwdft_append_attn         */
} iwdft_desc;

/* Sizes of the two caller-provided device buffers for this descriptor. */
int iwdft_query_bytes(const iwdft_desc* desc, size_t* state_bytes, size_t* workspace_bytes);

/* Validates desc, copies the bin lists into d_state and zeroes the coefficients
 * (synchronous; not a hot call).  Both buffers must be 256-byte aligned and stay
 * alive and untouched by the caller until iwdft_destroy.  The HIP device that is
 * current at this call owns the context. */
int iwdft_create(const iwdft_desc* desc, void* d_state, size_t state_bytes, void* d_workspace,
                 size_t workspace_bytes, iwdft_ctx** out);

int iwdft_destroy(iwdft_ctx* ctx); /* frees host memory only; NULL is accepted */

/* Prefill transform (Eq. dft-full at the kept bins, Eq. prefill-dft, Eq. freq-zero), either as a
 * dense contraction with an on-chip basis or as FFTs followed by pruning (see desc.flags).
 * d_K, d_V: [n_layers][batch][n_kv_heads][S + M + R][head_dim] contiguous, kv_dtype.
 * Per slice the first S tokens are copied to the sink store, the last R to the recent
 * window, and the middle M tokens are transformed (Sec. 4.2.1).  Overwrites the state;
 * T becomes M. */
int iwdft_prefill(iwdft_ctx* ctx, const void* d_K, const void* d_V, void* hip_stream);

/* Which transform iwdft_prefill runs for this context: 0 = dense contraction, 1 = FFTs + pruning;
 * -1 if ctx is NULL. */
int iwdft_prefill_kind(const iwdft_ctx* ctx);

/* Which synthesis compressed_decode_attn / iwdft_append_attn run for this context: 1 = scores and softmax
 * weights through in-LDS FFTs (M = 2^m >= 256: O(M log M) per query head, the HBM-bound path; layers with more than
 * 4096 kept bins run a form of it that keeps nothing per bin in registers); 2 = through chirp-z transforms (any
 * other M >= 32 that is at most 8192 or has a divisor Pb <= 256 with 32 <= M / Pb <= 8192, e.g. M = context - sink -
 * recent = 16384 - 60 = 2 * 8162: O(M log M) as well, about 8 times the arithmetic of 1); 0 = the direct O(M |B|)
 * sums (arithmetic-bound; chosen by IWDFT_FLAG_DIRECT_SYNTHESIS, for M < 32, and for M > 8192 without such a divisor,
 * e.g. a prime -- there only while M * (most kept bins of a layer) <= 2^30, beyond that iwdft_query_bytes /
 * iwdft_create return IWDFT_ERR_UNSUPPORTED unless the flag insists); -1 if ctx is NULL.
 * With 0 or 2, or when some layer keeps more than 4096 bins, desc.write_every is taken as 1. */
int iwdft_attn_kind(const iwdft_ctx* ctx);

/* Whether decode attention on this context (Sec. 4.2.2 "Calculating Attention") walks the slices in groups, with
 * the transforms of one group in the same launches as the K-coefficient stream of the next (see
 * IWDFT_FLAG_SERIAL_PHASES for the conditions): 1 = yes, 0 = the three kernels run one after the other;
 * -1 if ctx is NULL.  Results are identical either way; with 1 the marks of iwdft_phase_timing cannot separate
 * the first two kernels (their time is reported as phase 0, phase 1 reads ~0). */
int iwdft_attn_pipelined(const iwdft_ctx* ctx);

/* Streaming update with one new token per sequence (Eq. infi-dft, Eq. update-iwdft).
 * d_tok_k, d_tok_v: [n_layers][batch][n_kv_heads][head_dim], kv_dtype.  T -> T+1.
 * With R > 0 the new token joins the recent window and the token that ages out of it is
 * the one absorbed into the coefficients ("Updating Cache", Sec. 4.2.2); with R = 0 the
 * new token itself is absorbed.  Requires a prior prefill (IWDFT_ERR_STATE otherwise). */
int iwdft_append(iwdft_ctx* ctx, const void* d_tok_k, const void* d_tok_v, void* hip_stream);

/* Reconstruction of time slots a0 .. a0+n_slots-1 of one layer (Eq. inverse-swdft over
 * the kept bins, real part, gain T/M on S_T; Eq. reconstruct-idft):
 *   x~[a] = (1/M) Re sum_{k in B} w_k T S_T[k] exp(+j 2 pi k a / M).
 * d_Kt, d_Vt: [batch][n_kv_heads][n_slots][head_dim], kv_dtype; either may be NULL.
 * 0 <= a0, a0 + n_slots <= M. */
int iwdft_reconstruct(iwdft_ctx* ctx, int32_t layer, int64_t a0, int64_t n_slots, void* d_Kt,
                      void* d_Vt, void* hip_stream);

/* The same reconstruction on a strided grid of time slots: a0, a0 + stride, ..., n_slots of them
 * (stride >= 1, a0 + (n_slots - 1) * stride < M) -- a compressed token set of n_slots < M rows instead of the
 * original length that Sec. 4.2.2 reconstructs to (an extension; stride 1 is iwdft_reconstruct).
 * d_Kt, d_Vt: [batch][n_kv_heads][n_slots][head_dim], kv_dtype; either may be NULL. */
int iwdft_reconstruct_grid(iwdft_ctx* ctx, int32_t layer, int64_t a0, int64_t stride, int64_t n_slots,
                           void* d_Kt, void* d_Vt, void* hip_stream);

/* Decode attention over the assembled cache of every layer (Eq. kv-attn over Eq. kv-concat:
 * the S sink tokens, the M reconstructed slots, the R recent tokens, one softmax):
 * o = softmax(q [K_sink; K~; K_recent]^T * scale) [V_sink; V~; V_recent] without writing
 * K~, V~ to memory.  d_q, d_out: [n_layers][batch][n_q_heads][head_dim], kv_dtype.
 * scale <= 0 selects 1/sqrt(head_dim). */
int compressed_decode_attn(iwdft_ctx* ctx, const void* d_q, void* d_out, float scale,
                           void* hip_stream);

/* compressed_decode_attn for callers that cannot allocate device memory or hand over a workspace at the time
 * of the call (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels and the same result, but the intermediate arrays (the q.F_K rows, the softmax-weight rows, the scores
 * of the exact tokens; the score rows of the direct synthesis) live in a scratch array that is part of the
 * library's code object -- IWDFT_STATIC_SCRATCH_BYTES per GPU, held until the process ends -- instead of the
 * context's workspace.  Calls no hipMalloc / hipFree or any other allocating routine.  Returns IWDFT_ERR_SIZE
 * when the context needs more than the scratch holds: 16 * sum over layers of batch * n_q_heads * Bp_l bytes
 * (Bp_l = kept bins of layer l rounded up to 32) + 4 * n_layers * batch * n_q_heads * (S + R) bytes, each part
 * rounded up to 256 (+ 4 * M bytes per query head with the direct synthesis).  All calls on one GPU share that
 * GPU's array: calls that overlap in time on one GPU (different streams or contexts) race; calls ordered on one
 * stream do not.  Nothing in the array needs to survive between calls. */
#define IWDFT_STATIC_SCRATCH_BYTES (64u << 20)
int compressed_decode_attn_static(iwdft_ctx* ctx, const void* d_q, void* d_out, float scale,
                                  void* hip_stream);

/* One decode step: iwdft_append(tok) followed by compressed_decode_attn(q) (the three operations
 * of the decoding stage, Sec. 4.2.2), fused: each K coefficient is updated (Eq. infi-dft) on its
 * way into the scores and each V coefficient on its way into the output, so every coefficient is
 * read once and written once per step instead of read twice and written once.  Same arguments,
 * same result (up to rounding order) and same errors as the two calls in sequence.  T -> T+1.
 *
 * desc.write_every = J > 1 (J <= 16) defers the write-back: the step's token (the one leaving the recent window
 * when R > 0) is kept in the workspace, and until J of them have gathered the coefficients are only
 * read -- the tokens they do not hold yet enter scores and output through the exact rank-one terms
 * F + x e^{j theta} contributes -- so every call still returns the attention over all T tokens, and the
 * coefficients are written once per J steps.  Every other call on the context (append, attention,
 * reconstruct, export) first writes the deferred tokens back, so results never depend on J beyond
 * rounding order; only a caller that copies the state buffer itself (checkpoint) must call iwdft_flush
 * first.  Deferral needs the FFT attention path and at most 8 query heads per KV head; without them
 * J is taken as 1. */
int iwdft_append_attn(iwdft_ctx* ctx, const void* d_tok_k, const void* d_tok_v, const void* d_q,
                      void* d_out, float scale, void* hip_stream);

/* Profiling aid (no paper operation).  While enabled, every compressed_decode_attn and fused
 * iwdft_append_attn call records HIP events around its three phases -- A: the query against the K
 * coefficients (Eq. kv-attn scores in the frequency domain; with the K update in the fused step),
 * B: inverse transform + softmax + forward transform, C: the output from the V coefficients (with
 * the V update in the fused step) -- on the call's stream.  Events are host objects the context
 * owns; no device memory is allocated.  A fused call that falls back to append + attention marks
 * its attention part only. */
int iwdft_phase_timing(iwdft_ctx* ctx, int enable);

/* Waits for the marked calls made since the last read-out, then returns the summed duration of each
 * phase in milliseconds (ms[0..2] = A, B, C; HOST) and the number of calls, and clears the list. */
int iwdft_phase_times(iwdft_ctx* ctx, double* ms, int64_t* n_calls);

/* Writes tokens deferred by iwdft_append_attn (desc.write_every > 1) into the coefficients; afterwards the
 * state buffer alone describes the cache.  No-op when nothing is deferred. */
int iwdft_flush(iwdft_ctx* ctx, void* hip_stream);

/* The paper-convention coefficients S_T of one layer, for inspection and parity:
 * d_SK, d_SV: [batch][n_kv_heads][|B_layer|][head_dim][2] (re, im) fp32; either may be NULL. */
int iwdft_export_coeffs(iwdft_ctx* ctx, int32_t layer, float* d_SK, float* d_SV,
                        void* hip_stream);

/* Device copy of the kept bins of one layer, int32 [|B_layer|] (for bit-exact mask checks). */
int iwdft_export_bins(iwdft_ctx* ctx, int32_t layer, int32_t* d_bins, void* hip_stream);

int64_t iwdft_num_tokens(const iwdft_ctx* ctx); /* T = tokens inside the coefficients (the sink and
                                                    recent tokens are not counted); 0 before prefill;
                                                    -1 if ctx is NULL */

/* Sets T after the caller restored a saved copy of the state buffer (checkpoint / resume; the copy
 * must have been taken after iwdft_flush if write-back is deferred).  T >= M. */
int iwdft_set_num_tokens(iwdft_ctx* ctx, int64_t T);

/* Greedy frequency mask of the ablation study (Sec. 3.2): the M bins are cut into n_chunks contiguous
 * chunks, chunk c = bins [floor(c M / n_chunks), floor((c+1) M / n_chunks)); per layer the
 * clamp(floor(r * n_chunks + 1/2), 1, n_chunks) chunks with the largest importance delta (Eq. delta-ppl)
 * are kept, the lower chunk index first among equal values.  All pointers are HOST memory:
 * delta [n_layers][n_chunks] (no NaN), bin_offsets [n_layers + 1] (out), bins [bins_capacity] (out,
 * per layer ascending -- the lists iwdft_desc takes).  bin_offsets is always filled, so a call with
 * bins_capacity = 0 sizes the list (returns IWDFT_ERR_SIZE).  No GPU work. */
int iwdft_select_bins(const float* delta, int32_t n_layers, int32_t n_chunks, int64_t M, double r,
                      int64_t* bin_offsets, int32_t* bins, int64_t bins_capacity);

/* Frequency ablation of one chunk (Sec. 3.2, Eq. freq-zero): per slice and channel the DFT along the token
 * axis, the coefficients of the chunk's bins set to zero, the inverse DFT, real part.
 * d_x, d_out: DEVICE [n_slices][M][head_dim], kv_dtype, must not overlap.  This build: head_dim 128 and
 * M = 2^m, 256 <= M <= 2^24 (IWDFT_ERR_UNSUPPORTED otherwise).  For M > 8192 the chunk's part is taken off the
 * input 4096 bins at a time through d_out, so a bf16 result carries one more rounding per such piece.
 * Needs no context; enqueues on hip_stream. */
int iwdft_ablate_chunk(const void* d_x, void* d_out, int64_t n_slices, int64_t M, int32_t head_dim,
                       int32_t kv_dtype, int32_t n_chunks, int32_t chunk, void* hip_stream);

const char* iwdft_last_error(void); /* thread-local, static storage, never NULL */

#ifdef __cplusplus
}
#endif
#endif /* IWDFT_H_ */
