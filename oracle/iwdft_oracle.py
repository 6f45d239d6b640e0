"""Float64 CPU oracle of the FAEDKV / IWDFT hot path (arxiv 2507.20030).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition the GPU
library is checked against.  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import it; the product package never does, and this
module imports nothing from the product package.  It shares no code, tables or
constants with the HIP path.

Everything works on ONE slice (one layer, one sequence, one KV head): ``x`` is a
``[tokens, channels]`` float64 array, K and V are treated identically.

Notation (paper, Sec. 3.1.2 and Sec. 4.1):
    M        DFT length = number of tokens transformed at prefill
    T        number of tokens absorbed so far (T == M right after prefill)
    W_k      exp(-j 2 pi k / M)                               (Eq. sliding-dft)
    S_T[k]   normalised coefficient the IWDFT recursion carries (Eq. infi-dft)
    U_T[k]   T * S_T[k], the un-normalised accumulator
    B        sorted kept bins of the layer                     (Sec. 3.2, 4.2)

Readings of the paper this oracle fixes (the paper leaves them open):
  * hand-over prefill -> streaming: the state after prefill is Eq. dft-full
    divided by M, every later token applies Eq. infi-dft exactly as printed,
    with N = token count after the append.
  * reconstruction takes the real part of the masked inverse DFT of the
    UN-normalised spectrum U_T (gain T/M on S_T), output length M.
  * tokens beyond M alias onto the M slots (W_k^M = 1).
  * frequency chunks (Sec. 3.2): chunk c of C holds the bins
    floor(c M / C) .. floor((c+1) M / C) - 1 (M need not divide by C); "the top
    r*C chunks" means n_c = clamp(floor(r C + 1/2), 1, C) chunks, largest
    Delta first, equal Delta -> lower chunk index first.
Parity unpinned: the choice among those readings (slot map, real part, gain)
is not fixed by anything the paper prints; every function below is pinned by
identities in tests/test_oracle_pins.py.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "W", "prefill", "append", "append_many", "slot", "fold_to_slots",
    "closed_form", "reconstruct", "reconstruct_grid", "attention", "decode_attention",
    "stream_decode", "windowed_attention", "windowed_stream_decode",
    "chunk_bounds", "ablate_chunk", "select_bins",
    "append_shortcut", "closed_form_shortcut",
]


def W(bins, M):
    """Twiddle W_k = exp(-j 2 pi k / M) for each kept bin (Eq. sliding-dft)."""
    k = np.asarray(bins, dtype=np.int64) % M
    return np.exp(-2j * np.pi * k.astype(np.float64) / float(M))


def prefill(x, bins):
    """Normalised prefill state S_M[k] = (1/M) sum_n x[n] W_k^n, k in B.

    Eq. dft-full applied to the M prefill tokens (Eq. prefill-dft), kept bins
    only (Eq. freq-zero), divided by M so that Eq. infi-dft can carry it on.
    x: [M, d] float64.  Returns [|B|, d] complex128.
    """
    x = np.asarray(x, dtype=np.float64)
    M = x.shape[0]
    bins = np.asarray(bins, dtype=np.int64)
    return np.fft.fft(x, axis=0)[bins] / M


def append(S, x_new, T, bins, M):
    """One IWDFT update, Eq. infi-dft, literally.

    S: state after T tokens, [|B|, d] complex.  x_new: [d], token number T
    (0-based).  N = T + 1 is the sequence length after the append.
    Returns S_{T+1} = W_k * ((N-1)/N * S_T + x_new / N).
    """
    N = float(T + 1)
    w = W(bins, M)[:, None]
    x_new = np.asarray(x_new, dtype=np.float64)
    return w * (((N - 1.0) / N) * S + x_new[None, :] / N)


def append_many(S, xs, T, bins, M):
    """Apply `append` for every row of xs in order. Returns (S, T)."""
    for row in np.asarray(xs, dtype=np.float64):
        S = append(S, row, T, bins, M)
        T += 1
    return S, T


def slot(n, T, M):
    """Time slot (0..M-1) token n occupies once T tokens have been absorbed.

    Follows from unrolling Eq. infi-dft from the Eq. dft-full prefill state:
    each update multiplies the whole state by W_k (one slot later) and the new
    token enters with a single factor W_k (slot 1).
    """
    n = np.asarray(n, dtype=np.int64)
    return np.where(n < M, (n + (T - M)) % M, (T - n) % M)


def fold_to_slots(xs, M):
    """y[a] = sum of all tokens currently sitting in slot a.  xs: [T, d]."""
    xs = np.asarray(xs, dtype=np.float64)
    T = xs.shape[0]
    y = np.zeros((M, xs.shape[1]), dtype=np.float64)
    np.add.at(y, slot(np.arange(T), T, M), xs)
    return y


def closed_form(xs, M, bins):
    """From-scratch recompute of S_T from all T >= M tokens seen so far.

    U_T[k] = sum_a y[a] W_k^a with y = fold_to_slots(xs), S_T = U_T / T:
    every token enters with weight exactly 1/T.
    """
    xs = np.asarray(xs, dtype=np.float64)
    T = xs.shape[0]
    assert T >= M
    bins = np.asarray(bins, dtype=np.int64)
    return np.fft.fft(fold_to_slots(xs, M), axis=0)[bins] / T


def reconstruct(S, T, M, bins, weights=None):
    """Time-domain reconstruction, Eq. inverse-swdft on the masked spectrum.

    x~[a] = (1/M) Re sum_{k in B} w_k U_T[k] exp(+j 2 pi k a / M), U_T = T S_T,
    a = 0..M-1.  Returns [M, d] float64.
    """
    bins = np.asarray(bins, dtype=np.int64)
    w = np.ones(len(bins)) if weights is None else np.asarray(weights, np.float64)
    full = np.zeros((M, S.shape[1]), dtype=np.complex128)
    full[bins] = (w[:, None] * float(T)) * S
    return np.fft.ifft(full, axis=0).real


def reconstruct_grid(S, T, M, bins, a0, stride, n_out, weights=None):
    """The reconstruction of Eq. inverse-swdft evaluated on a strided grid of time slots only,
    a_j = a0 + j * stride, j < n_out (a compressed token set; an extension of Sec. 4.2.2, which
    reconstructs all M slots), as the sum it is:
    x~[a_j] = (T/M) Re sum_{k in B} w_k S_T[k] exp(+j 2 pi k a_j / M).  Returns [n_out, d]."""
    bins = np.asarray(bins, dtype=np.int64)
    w = np.ones(len(bins)) if weights is None else np.asarray(weights, np.float64)
    a = a0 + stride * np.arange(n_out, dtype=np.int64)
    assert n_out == 0 or (a0 >= 0 and a[-1] < M and stride >= 1)
    basis = np.exp(2j * np.pi * ((a[:, None] * bins[None, :]) % M) / float(M))      # [n_out, |B|]
    return (basis @ (w[:, None] * np.asarray(S, dtype=np.complex128))).real * (float(T) / float(M))


def attention(q, K, V, scale=None):
    """Softmax attention of Eq. kv-attn for a group of query heads.

    q: [G, d]; K, V: [n, d].  o = softmax(q K^T * scale) V, scale = 1/sqrt(d).
    """
    q = np.asarray(q, dtype=np.float64)
    d = q.shape[-1]
    if scale is None or scale <= 0:
        scale = 1.0 / np.sqrt(d)
    logits = (q @ K.T) * scale
    logits = logits - logits.max(axis=-1, keepdims=True)
    p = np.exp(logits)
    p /= p.sum(axis=-1, keepdims=True)
    return p @ V


def decode_attention(q, SK, SV, T, M, bins, weights=None, scale=None):
    """Attention over the reconstructed segment (Eq. kv-concat with S = R = 0)."""
    Kt = reconstruct(SK, T, M, bins, weights)
    Vt = reconstruct(SV, T, M, bins, weights)
    return attention(q, Kt, Vt, scale)


def stream_decode(K0, V0, bins, k_new, v_new, q_new, weights=None, scale=None):
    """Prefill, then per step: append (k_i, v_i), attend with q_i.

    K0, V0: [M, d]; k_new, v_new: [steps, d]; q_new: [steps, G, d].
    Returns (outs [steps, G, d], SK, SV, T).
    """
    M = K0.shape[0]
    SK, SV, T = prefill(K0, bins), prefill(V0, bins), M
    outs = []
    for i in range(len(k_new)):
        SK = append(SK, k_new[i], T, bins, M)
        SV = append(SV, v_new[i], T, bins, M)
        T += 1
        outs.append(decode_attention(q_new[i], SK, SV, T, M, bins, weights, scale))
    return np.stack(outs) if outs else np.zeros((0,) + q_new.shape[1:]), SK, SV, T


def windowed_attention(q, sinkK, sinkV, SK, SV, T, M, bins, recK, recV, weights=None, scale=None):
    """Attention over the assembled cache of Eq. kv-concat: [sink tokens, reconstructed
    middle segment, recent tokens] (the V line of that equation prints K~ where V~ is meant)."""
    Kt = reconstruct(SK, T, M, bins, weights)
    Vt = reconstruct(SV, T, M, bins, weights)
    K = np.concatenate([sinkK, Kt, recK], axis=0)
    V = np.concatenate([sinkV, Vt, recV], axis=0)
    return attention(q, K, V, scale)


def windowed_stream_decode(K0, V0, S, R, bins, k_new, v_new, q_new, weights=None, scale=None):
    """The decoding stage of Sec. 4.2.2 with S sink and R recent tokens kept exact.

    K0, V0: [N, d] prefill cache, N = S + M + R; the middle M tokens are transformed
    (Eq. prefill-dft).  Per step: the new token (k_i, v_i) joins the recent window, the
    token that ages out of it is absorbed by the IWDFT update (Eq. update-iwdft), and the
    query attends over [sink, reconstruction, recent] (Eq. kv-concat, Eq. kv-attn), so
    that every token seen so far sits in exactly one of the three parts.
    Returns (outs [steps, G, d], SK, SV, T, recent_K [R, d], recent_V [R, d]).
    """
    K0, V0 = np.asarray(K0, np.float64), np.asarray(V0, np.float64)
    N = K0.shape[0]
    M = N - S - R
    assert M >= 1
    sinkK, sinkV = K0[:S], V0[:S]
    SK, SV, T = prefill(K0[S:S + M], bins), prefill(V0[S:S + M], bins), M
    recK, recV = [r for r in K0[S + M:]], [r for r in V0[S + M:]]
    outs = []
    for i in range(len(k_new)):
        recK.append(np.asarray(k_new[i], np.float64))
        recV.append(np.asarray(v_new[i], np.float64))
        if len(recK) > R:                      # the oldest recent token ages out
            SK = append(SK, recK.pop(0), T, bins, M)
            SV = append(SV, recV.pop(0), T, bins, M)
            T += 1
        rk = np.stack(recK) if recK else np.zeros((0, K0.shape[1]))
        rv = np.stack(recV) if recV else np.zeros((0, K0.shape[1]))
        outs.append(windowed_attention(q_new[i], sinkK, sinkV, SK, SV, T, M, bins, rk, rv, weights, scale))
    rk = np.stack(recK) if recK else np.zeros((0, K0.shape[1]))
    rv = np.stack(recV) if recV else np.zeros((0, K0.shape[1]))
    return (np.stack(outs) if outs else np.zeros((0,) + np.shape(q_new)[1:])), SK, SV, T, rk, rv


def chunk_bounds(M, C):
    """Edges of the C contiguous frequency chunks of an M-bin spectrum (Sec. 3.2):
    chunk c = bins [edges[c], edges[c+1])."""
    return np.array([(c * int(M)) // int(C) for c in range(int(C) + 1)], dtype=np.int64)


def ablate_chunk(x, C, c):
    """Frequency ablation of one chunk (Sec. 3.2, Eq. freq-zero): DFT of x along the
    token axis, the coefficients of chunk c set to zero, inverse DFT, real part.
    x: [M, d] float64.  Returns [M, d] float64."""
    x = np.asarray(x, dtype=np.float64)
    M = x.shape[0]
    e = chunk_bounds(M, C)
    X = np.fft.fft(x, axis=0)
    X[e[c]:e[c + 1]] = 0.0
    return np.fft.ifft(X, axis=0).real


def select_bins(delta, M, r):
    """Greedy mask of Sec. 3.2: per layer keep the n_c chunks with the largest
    Delta (Eq. delta-ppl) and return their bins, sorted.
    delta: [layers, C].  n_c = clamp(floor(r C + 1/2), 1, C) in float64;
    equal Delta: the lower chunk index wins.  Returns a list of int32 arrays."""
    delta = np.asarray(delta)
    n_layers, C = delta.shape
    n_c = int(min(max(np.floor(np.float64(r) * np.float64(C) + np.float64(0.5)), 1), C))
    e = chunk_bounds(M, C)
    out = []
    for l in range(n_layers):
        order = sorted(range(C), key=lambda c: (-float(delta[l, c]), c))
        keep = sorted(order[:n_c])
        b = [np.arange(e[c], e[c + 1], dtype=np.int64) for c in keep]
        out.append(np.concatenate(b).astype(np.int32) if b else np.zeros(0, np.int32))
    return out


def append_shortcut(S, x_new, T, bins, M):
    """The variant of Eq. infi-dft that Sec. 4.1 mentions for long contexts, with the factor
    (N-1)/N of the old state taken as 1:  S_{T+1}[k] = W_k ( S_T[k] + x_T / (T+1) ).
    Not what the hot path computes (old tokens keep their weight, so weights are no longer
    equal); kept to measure how far the shortcut drifts from the exact rule."""
    S = np.asarray(S, dtype=np.complex128)
    x_new = np.asarray(x_new, dtype=np.float64)
    return W(bins, M)[:, None] * (S + x_new[None, :] / float(T + 1))


def closed_form_shortcut(xs, M, bins):
    """What append_shortcut reaches after T - M steps, written out: the prefill tokens keep
    weight 1/M for ever, token n >= M enters with weight 1/(n+1):
    S_T[k] = W_k^(T-M) S_M[k] + sum_{n=M}^{T-1} x[n] W_k^(T-n) / (n+1).   xs: [T, d]."""
    xs = np.asarray(xs, dtype=np.float64)
    T = xs.shape[0]
    k = np.asarray(bins, dtype=np.int64)
    out = np.exp(-2j * np.pi * ((k * (T - M)) % M) / float(M))[:, None] * prefill(xs[:M], bins)
    for n in range(M, T):
        ph = np.exp(-2j * np.pi * ((k * (T - n)) % M) / float(M))
        out = out + ph[:, None] * xs[n][None, :] / float(n + 1)
    return out
