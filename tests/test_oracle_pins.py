"""Pins for the float64 oracle: every function is checked against something
other than itself -- brute-force sums written out here with cmath, textbook
closed forms, exact inversion, library routines, invariants.  CPU only.
"""
import cmath
import math

import numpy as np
import pytest
import torch

from oracle import iwdft_oracle as orc


def rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- brute force
def brute_prefill(x, bins):
    """(1/M) sum_n x[n] exp(-j 2 pi k n / M), plain loops (Eq. dft-full)."""
    M, d = len(x), len(x[0])
    out = [[0j] * d for _ in bins]
    for i, k in enumerate(bins):
        for c in range(d):
            acc = 0j
            for n in range(M):
                acc += x[n][c] * cmath.exp(-2j * math.pi * k * n / M)
            out[i][c] = acc / M
    return np.array(out)


def brute_stream(xs, M, bins):
    """Eq. infi-dft run token by token with Python complex scalars."""
    d = len(xs[0])
    S = brute_prefill([list(r) for r in xs[:M]], bins)
    S = [[complex(S[i][c]) for c in range(d)] for i in range(len(bins))]
    T = M
    for row in xs[M:]:
        N = T + 1
        for i, k in enumerate(bins):
            wk = cmath.exp(-2j * math.pi * k / M)
            for c in range(d):
                S[i][c] = wk * ((N - 1) / N * S[i][c] + row[c] / N)
        T = N
    return np.array(S), T


def brute_reconstruct(S, T, M, bins, weights=None):
    d = S.shape[1]
    out = np.zeros((M, d))
    for a in range(M):
        for c in range(d):
            acc = 0j
            for i, k in enumerate(bins):
                w = 1.0 if weights is None else weights[i]
                acc += w * T * S[i, c] * cmath.exp(2j * math.pi * k * a / M)
            out[a, c] = (acc / M).real
    return out


# -------------------------------------------------------------------- prefill
@pytest.mark.parametrize("M,bins", [(8, [0, 1, 2, 7]), (12, [0, 3, 5, 6, 11]), (16, list(range(16)))])
def test_prefill_matches_brute_force(M, bins):
    x = rng(1).normal(size=(M, 3))
    np.testing.assert_allclose(orc.prefill(x, bins), brute_prefill(x.tolist(), bins), atol=1e-13)


def test_prefill_textbook_cases():
    M, bins = 32, np.arange(32)
    const = np.full((M, 1), 2.5)
    S = orc.prefill(const, bins)[:, 0]
    assert abs(S[0] - 2.5) < 1e-14 and np.abs(S[1:]).max() < 1e-14
    n0 = 5
    imp = np.zeros((M, 1)); imp[n0] = 1.0
    np.testing.assert_allclose(orc.prefill(imp, bins)[:, 0],
                               np.exp(-2j * np.pi * bins * n0 / M) / M, atol=1e-15)
    k0 = 3
    cosx = np.cos(2 * np.pi * k0 * np.arange(M) / M)[:, None]
    S = orc.prefill(cosx, bins)[:, 0]
    expect = np.zeros(M, complex); expect[k0] = expect[M - k0] = 0.5
    np.testing.assert_allclose(S, expect, atol=1e-14)
    # a sine has a purely imaginary coefficient of sign -j/2 at +k0 (fixes the sign of W_k)
    sinx = np.sin(2 * np.pi * k0 * np.arange(M) / M)[:, None]
    S = orc.prefill(sinx, bins)[:, 0]
    assert abs(S[k0] - (-0.5j)) < 1e-14 and abs(S[M - k0] - 0.5j) < 1e-14


def test_prefill_keeps_only_requested_bins_in_order():
    x = rng(2).normal(size=(16, 2))
    full = orc.prefill(x, np.arange(16))
    bins = [1, 4, 9, 15]
    np.testing.assert_array_equal(orc.prefill(x, bins), full[bins])


# ------------------------------------------------------------------ streaming
@pytest.mark.parametrize("M,extra", [(8, 1), (8, 5), (8, 8), (8, 27), (12, 30)])
def test_recursion_matches_brute_and_closed_form(M, extra):
    bins = sorted(rng(3).choice(M, size=M // 2 + 1, replace=False).tolist())
    xs = rng(4).normal(size=(M + extra, 2))
    S, T = orc.append_many(orc.prefill(xs[:M], bins), xs[M:], M, bins, M)
    Sb, Tb = brute_stream(xs.tolist(), M, bins)
    assert T == Tb == M + extra
    np.testing.assert_allclose(S, Sb, atol=1e-13)
    np.testing.assert_allclose(S, orc.closed_form(xs, M, bins), atol=1e-12)


def test_closed_form_is_the_explicit_slot_sum():
    M, T = 8, 21
    bins = [0, 1, 3, 6]
    xs = rng(5).normal(size=(T, 2))
    # U_T[k] = sum_n x[n] W_k^{e(n)}, e = n+T-M for prefill tokens, T-n after
    U = np.zeros((len(bins), 2), complex)
    for n in range(T):
        e = n + T - M if n < M else T - n
        for i, k in enumerate(bins):
            U[i] += xs[n] * cmath.exp(-2j * math.pi * k * e / M)
    np.testing.assert_allclose(orc.closed_form(xs, M, bins), U / T, atol=1e-13)
    assert list(orc.slot(np.arange(T), T, M)) == [
        (n + T - M) % M if n < M else (T - n) % M for n in range(T)]


def test_dc_bin_is_running_mean():
    M = 16
    xs = rng(6).normal(size=(M + 40, 3))
    S, T = orc.append_many(orc.prefill(xs[:M], [0, 5]), xs[M:], M, [0, 5], M)
    np.testing.assert_allclose(S[0], xs.mean(axis=0), atol=1e-13)


def test_every_token_has_weight_one_over_T():
    # perturbing any single token by delta moves |S_T[k]| by exactly delta/T
    M, T, bins = 8, 19, [1, 2, 5]
    xs = rng(7).normal(size=(T, 1))
    base = orc.closed_form(xs, M, bins)
    for n in (0, 3, 7, 8, 13, 18):
        ys = xs.copy(); ys[n] += 1.0
        S, _ = orc.append_many(orc.prefill(ys[:M], bins), ys[M:], M, bins, M)
        np.testing.assert_allclose(np.abs(S - base), 1.0 / T, atol=1e-13)


def test_linearity():
    M, bins = 8, [0, 2, 3]
    xa, xb = rng(8).normal(size=(M + 9, 2)), rng(9).normal(size=(M + 9, 2))
    f = lambda x: orc.append_many(orc.prefill(x[:M], bins), x[M:], M, bins, M)[0]
    np.testing.assert_allclose(f(2.0 * xa - 0.75 * xb), 2.0 * f(xa) - 0.75 * f(xb), atol=1e-13)


@pytest.mark.parametrize("j,i", [(0, 0), (2, 3), (1, 11)])
def test_appended_impulse_lands_in_slot_i_plus_one(j, i):
    M, bins = 8, np.arange(8)
    zeros = np.zeros((M, 1))
    S, T = orc.prefill(zeros, bins), M
    S, T = orc.append_many(S, np.zeros((j, 1)), T, bins, M)
    S, T = orc.append_many(S, np.ones((1, 1)), T, bins, M)
    S, T = orc.append_many(S, np.zeros((i, 1)), T, bins, M)
    np.testing.assert_allclose(S[:, 0], np.exp(-2j * np.pi * bins * (i + 1) / M) / T, atol=1e-14)


# ------------------------------------------------------------- reconstruction
def test_reconstruct_matches_brute_force():
    M, bins = 8, [0, 1, 3, 6]
    xs = rng(10).normal(size=(M + 3, 2))
    S, T = orc.append_many(orc.prefill(xs[:M], bins), xs[M:], M, bins, M)
    w = [1.0, 2.0, 0.5, 1.5]
    np.testing.assert_allclose(orc.reconstruct(S, T, M, bins), brute_reconstruct(S, T, M, bins), atol=1e-13)
    np.testing.assert_allclose(orc.reconstruct(S, T, M, bins, w), brute_reconstruct(S, T, M, bins, w), atol=1e-13)


def test_all_bins_exact_inverse_at_prefill():
    x = rng(11).normal(size=(32, 4))
    bins = np.arange(32)
    np.testing.assert_allclose(orc.reconstruct(orc.prefill(x, bins), 32, 32, bins), x, atol=1e-13)


def test_all_bins_after_appends_gives_folded_sums():
    M, T = 8, 8 + 13
    xs = rng(12).normal(size=(T, 2))
    bins = np.arange(M)
    S, _ = orc.append_many(orc.prefill(xs[:M], bins), xs[M:], M, bins, M)
    expect = np.zeros((M, 2))
    for n in range(T):
        a = (n + T - M) % M if n < M else (T - n) % M
        expect[a] += xs[n]
    np.testing.assert_allclose(orc.reconstruct(S, T, M, bins), expect, atol=1e-12)


def test_hermitian_closed_mask_is_a_projection():
    M = 16
    bins = [0, 1, 2, 5, 8, 11, 14, 15]           # closed under k -> M-k
    x = rng(13).normal(size=(M, 2))
    S = orc.prefill(x, bins)
    np.testing.assert_allclose(orc.prefill(orc.reconstruct(S, M, M, bins), bins), S, atol=1e-14)


def test_unmirrored_bin_reconstructs_at_half_amplitude():
    M, k0 = 16, 3
    x = np.cos(2 * np.pi * k0 * np.arange(M) / M)[:, None]
    np.testing.assert_allclose(orc.reconstruct(orc.prefill(x, [k0]), M, M, [k0]), 0.5 * x, atol=1e-14)


def test_one_sided_weights_give_exact_inverse():
    M = 16
    bins = np.arange(M // 2 + 1)
    w = np.where((bins == 0) | (bins == M // 2), 1.0, 2.0)
    x = rng(14).normal(size=(M, 3))
    np.testing.assert_allclose(orc.reconstruct(orc.prefill(x, bins), M, M, bins, w), x, atol=1e-13)


# ------------------------------------------------- reconstruction on a strided grid
def test_reconstruct_grid_matches_brute_force_and_the_subsampled_inverse_transform():
    M, bins = 12, [0, 1, 4, 7, 11]                       # M not a power of two, unmirrored bins
    xs = rng(30).normal(size=(M + 5, 3))
    S, T = orc.append_many(orc.prefill(xs[:M], bins), xs[M:], M, bins, M)
    w = [1.0, 2.0, 0.5, 1.5, 1.0]
    for a0, stride, n in [(0, 1, 12), (1, 3, 4), (5, 2, 3), (11, 1, 1), (0, 12, 1), (2, 5, 2), (3, 4, 0)]:
        for ww in (None, w):
            got = orc.reconstruct_grid(S, T, M, bins, a0, stride, n, ww)
            assert got.shape == (n, 3)
            slots = [a0 + j * stride for j in range(n)]
            # scalar sums with cmath, term by term
            www = [1.0] * len(bins) if ww is None else ww
            for j, a in enumerate(slots):
                for c in range(3):
                    tot = sum(www[i] * T * S[i, c] * cmath.exp(2j * math.pi * k * a / M) for i, k in enumerate(bins))
                    assert abs(got[j, c] - tot.real / M) < 1e-12
            # the zero-filled inverse FFT of the full-length reconstruction, subsampled
            np.testing.assert_allclose(got, orc.reconstruct(S, T, M, bins, ww)[slots], atol=1e-12)


def test_reconstruct_grid_all_bins_returns_the_tokens_on_the_grid():
    M = 32
    x = rng(31).normal(size=(M, 2))
    bins = np.arange(M)
    np.testing.assert_allclose(orc.reconstruct_grid(orc.prefill(x, bins), M, M, bins, 3, 4, 7), x[3::4][:7], atol=1e-12)
    # after appends: the folded sums of the slot map, on the grid
    xs = rng(32).normal(size=(M + 9, 2))
    S, T = orc.append_many(orc.prefill(xs[:M], bins), xs[M:], M, bins, M)
    np.testing.assert_allclose(orc.reconstruct_grid(S, T, M, bins, 1, 5, 6), orc.fold_to_slots(xs, M)[1::5][:6], atol=1e-11)


# ------------------------------------------------------------------ attention
def test_attention_matches_library_sdpa():
    q, K, V = rng(15).normal(size=(4, 16)), rng(16).normal(size=(40, 16)), rng(17).normal(size=(40, 16))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None])[0].numpy()
    np.testing.assert_allclose(orc.attention(q, K, V), ref, atol=1e-12)
    np.testing.assert_allclose(orc.attention(q, K, V, 0.3),
                               torch.softmax(torch.from_numpy(q @ K.T * 0.3), -1).numpy() @ V, atol=1e-12)


def test_attention_large_logits_do_not_overflow():
    q, K, V = np.full((1, 4), 300.0), rng(18).normal(size=(6, 4)), rng(19).normal(size=(6, 4))
    assert np.isfinite(orc.attention(q, K, V)).all()


def test_decode_attention_all_bins_equals_full_attention():
    M, d = 32, 8
    K, V, q = rng(20).normal(size=(M, d)), rng(21).normal(size=(M, d)), rng(22).normal(size=(2, d))
    bins = np.arange(M)
    o = orc.decode_attention(q, orc.prefill(K, bins), orc.prefill(V, bins), M, M, bins)
    np.testing.assert_allclose(o, orc.attention(q, K, V), atol=1e-12)


def test_decode_attention_shift_invariance_and_dc_only():
    M, d = 16, 4
    K, V, q = rng(23).normal(size=(M, d)), rng(24).normal(size=(M, d)), rng(25).normal(size=(3, d))
    bins = [0, 1, 2, 14, 15]
    a = orc.decode_attention(q, orc.prefill(K, bins), orc.prefill(V, bins), M, M, bins)
    Kr, Vr = np.roll(K, 5, axis=0), np.roll(V, 5, axis=0)
    b = orc.decode_attention(q, orc.prefill(Kr, bins), orc.prefill(Vr, bins), M, M, bins)
    np.testing.assert_allclose(a, b, atol=1e-13)
    o = orc.decode_attention(q, orc.prefill(K, [0]), orc.prefill(V, [0]), M, M, [0])
    np.testing.assert_allclose(o, np.broadcast_to(V.mean(axis=0), o.shape), atol=1e-13)


def test_fast_path_identities():
    """Identities a kernel may use instead of materialising K~ and V~."""
    M, d, G = 16, 4, 2
    bins = np.array([0, 1, 3, 9, 15]); w = np.array([1.0, 2.0, 1.0, 0.5, 1.0])
    xs = rng(26).normal(size=(M + 5, d)); vs = rng(27).normal(size=(M + 5, d))
    q = rng(28).normal(size=(G, d))
    SK, T = orc.append_many(orc.prefill(xs[:M], bins), xs[M:], M, bins, M)
    SV, _ = orc.append_many(orc.prefill(vs[:M], bins), vs[M:], M, bins, M)
    Kt, Vt = orc.reconstruct(SK, T, M, bins, w), orc.reconstruct(SV, T, M, bins, w)
    theta = 2 * np.pi * np.outer(bins, np.arange(M)) / M          # [k, a]
    qc = SK @ q.T                                                  # [k, G]
    scores = (T / M) * np.einsum("k,kg,ka->ga", w, qc, np.exp(1j * theta)).real
    np.testing.assert_allclose(scores, q @ Kt.T, atol=1e-12)
    p = rng(29).random(size=(G, M))
    P = p @ np.exp(-1j * theta).T                                  # [G, k]
    o = (T / M) * np.einsum("k,kd,gk->gd", w, SV, np.conj(P)).real
    np.testing.assert_allclose(o, p @ Vt, atol=1e-12)


def test_stream_decode_order_append_then_attend():
    M, d, steps = 8, 4, 3
    bins = [0, 1, 2, 7]
    r = rng(30)
    K0, V0 = r.normal(size=(M, d)), r.normal(size=(M, d))
    kn, vn, qn = r.normal(size=(steps, d)), r.normal(size=(steps, d)), r.normal(size=(steps, 2, d))
    outs, SK, SV, T = orc.stream_decode(K0, V0, bins, kn, vn, qn)
    assert T == M + steps
    allK, allV = np.vstack([K0, kn]), np.vstack([V0, vn])
    np.testing.assert_allclose(SK, orc.closed_form(allK, M, bins), atol=1e-13)
    last = orc.decode_attention(qn[-1], orc.closed_form(allK, M, bins), orc.closed_form(allV, M, bins), T, M, bins)
    np.testing.assert_allclose(outs[-1], last, atol=1e-12)
    first = orc.decode_attention(qn[0], orc.closed_form(allK[:M + 1], M, bins),
                                 orc.closed_form(allV[:M + 1], M, bins), M + 1, M, bins)
    np.testing.assert_allclose(outs[0], first, atol=1e-12)


# ------------------------------------------------------------ sink / recent windows
def test_windowed_all_bins_at_prefill_is_full_attention_over_every_token():
    # with every bin kept and nothing absorbed yet the middle segment is exact, so the assembled
    # cache is the whole context (in some order) and softmax attention does not care about order
    S, R, M, d = 3, 5, 16, 4
    r = rng(40)
    K0, V0 = r.normal(size=(S + M + R, d)), r.normal(size=(S + M + R, d))
    q = r.normal(size=(2, d))
    bins = np.arange(M)
    o = orc.windowed_attention(q, K0[:S], V0[:S], orc.prefill(K0[S:S + M], bins), orc.prefill(V0[S:S + M], bins),
                               M, M, bins, K0[S + M:], V0[S + M:])
    np.testing.assert_allclose(o, orc.attention(q, K0, V0), atol=1e-12)


def test_windowed_stream_every_token_sits_in_exactly_one_part():
    S, R, M, d, steps = 2, 3, 8, 3, 7
    r = rng(41)
    N = S + M + R
    K0, V0 = r.normal(size=(N, d)), r.normal(size=(N, d))
    kn, vn, qn = r.normal(size=(steps, d)), r.normal(size=(steps, d)), r.normal(size=(steps, 2, d))
    bins = [0, 1, 2, 6, 7]
    outs, SK, SV, T, rk, rv = orc.windowed_stream_decode(K0, V0, S, R, bins, kn, vn, qn)
    allK, allV = np.vstack([K0, kn]), np.vstack([V0, vn])
    # spectral state = tokens S .. S+T-1 in arrival order, each with weight 1/T; recent = the last R
    assert T == M + steps
    np.testing.assert_allclose(SK, orc.closed_form(allK[S:S + T], M, bins), atol=1e-13)
    np.testing.assert_allclose(SV, orc.closed_form(allV[S:S + T], M, bins), atol=1e-13)
    np.testing.assert_array_equal(rk, allK[-R:])
    np.testing.assert_array_equal(rv, allV[-R:])
    # the newest token is visible at once: the last output is attention over sink + reconstruction + last R
    ref = orc.attention(qn[-1], np.vstack([K0[:S], orc.reconstruct(SK, T, M, bins), allK[-R:]]),
                        np.vstack([V0[:S], orc.reconstruct(SV, T, M, bins), allV[-R:]]))
    np.testing.assert_allclose(outs[-1], ref, atol=1e-12)


def test_windowed_stream_without_windows_is_the_plain_stream():
    M, d, steps = 8, 4, 4
    r = rng(42)
    K0, V0 = r.normal(size=(M, d)), r.normal(size=(M, d))
    kn, vn, qn = r.normal(size=(steps, d)), r.normal(size=(steps, d)), r.normal(size=(steps, 2, d))
    bins = [0, 2, 3, 7]
    a = orc.windowed_stream_decode(K0, V0, 0, 0, bins, kn, vn, qn)
    b = orc.stream_decode(K0, V0, bins, kn, vn, qn)
    np.testing.assert_allclose(a[0], b[0], atol=1e-13)
    np.testing.assert_allclose(a[1], b[1], atol=1e-14)
    assert a[3] == b[3]


def test_windowed_attention_weights_split_between_parts():
    # a sink key aligned with the query and scaled up takes (almost) all the probability mass,
    # so the output tends to that sink token's value: exact tokens enter the same softmax
    S, R, M, d = 2, 2, 8, 4
    r = rng(43)
    K0, V0 = r.normal(size=(S + M + R, d)), r.normal(size=(S + M + R, d))
    q = r.normal(size=(1, d))
    K0[1] = 50.0 * q[0]
    bins = [0, 1, 7]
    o = orc.windowed_attention(q, K0[:S], V0[:S], orc.prefill(K0[S:S + M], bins), orc.prefill(V0[S:S + M], bins),
                               M, M, bins, K0[S + M:], V0[S + M:])
    np.testing.assert_allclose(o[0], V0[1], atol=1e-9)


# ------------------------------------------------------------ frequency chunks (Sec. 3.2)
def test_chunk_bounds_partition_the_spectrum():
    for M, C in [(8192, 22), (1024, 22), (22, 22), (100, 7), (16, 1), (5, 8)]:
        e = orc.chunk_bounds(M, C)
        assert e[0] == 0 and e[-1] == M and len(e) == C + 1 and np.all(np.diff(e) >= 0)
        # every bin lies in exactly one chunk, chunk sizes differ by at most one
        sizes = np.diff(e)
        assert sizes.sum() == M and sizes.max() - sizes.min() <= 1
        for k in range(M):
            assert sum(e[c] <= k < e[c + 1] for c in range(C)) == 1


def test_ablate_chunk_brute_force_tiny():
    M, d, C = 12, 2, 5
    x = rng(50).normal(size=(M, d))
    e = [(c * M) // C for c in range(C + 1)]
    for c in range(C):
        ref = np.zeros((M, d))
        for ch in range(d):
            X = [sum(x[n, ch] * cmath.exp(-2j * math.pi * k * n / M) for n in range(M)) for k in range(M)]
            for k in range(e[c], e[c + 1]):
                X[k] = 0.0
            for n in range(M):
                ref[n, ch] = (sum(X[k] * cmath.exp(2j * math.pi * k * n / M) for k in range(M)) / M).real
        np.testing.assert_allclose(orc.ablate_chunk(x, C, c), ref, atol=1e-12)


def test_ablate_chunks_partition_identity_and_special_cases():
    M, d, C = 64, 3, 22
    x = rng(51).normal(size=(M, d))
    # the chunks partition the spectrum: removing each once removes everything exactly once
    total = sum(x - orc.ablate_chunk(x, C, c) for c in range(C))
    np.testing.assert_allclose(total, x, atol=1e-12)
    # a single chunk is the whole spectrum
    np.testing.assert_allclose(orc.ablate_chunk(x, 1, 0), 0.0, atol=1e-12)
    # M chunks of one bin: chunk 0 is the DC bin, its removal subtracts the mean
    np.testing.assert_allclose(orc.ablate_chunk(x, M, 0), x - x.mean(axis=0), atol=1e-12)
    # a cosine at bin k0 has half of its amplitude in k0 and half in M - k0: removing the chunk that holds
    # only k0 leaves half a cosine (real part of the one-sided remainder).  The real part puts a quarter
    # back into each of the two bins, so removing M - k0 afterwards leaves a quarter of the cosine
    k0 = 5
    n = np.arange(M)
    cosx = np.cos(2 * np.pi * k0 * n / M)[:, None]
    np.testing.assert_allclose(orc.ablate_chunk(cosx, M, k0), 0.5 * cosx, atol=1e-12)
    both = orc.ablate_chunk(orc.ablate_chunk(cosx, M, k0), M, M - k0)
    np.testing.assert_allclose(both, 0.25 * cosx, atol=1e-12)
    # ablation is linear
    y = rng(52).normal(size=(M, d))
    np.testing.assert_allclose(orc.ablate_chunk(2 * x - 3 * y, C, 4),
                               2 * orc.ablate_chunk(x, C, 4) - 3 * orc.ablate_chunk(y, C, 4), atol=1e-12)


def test_ablate_is_what_a_mask_without_the_chunk_reconstructs():
    # zeroing chunk c == reconstructing from every bin outside chunk c (ties Eq. freq-zero to the
    # reconstruction the hot path uses)
    M, d, C, c = 48, 2, 6, 2
    x = rng(53).normal(size=(M, d))
    e = orc.chunk_bounds(M, C)
    keep = np.array([k for k in range(M) if not (e[c] <= k < e[c + 1])])
    np.testing.assert_allclose(orc.ablate_chunk(x, C, c), orc.reconstruct(orc.prefill(x, keep), M, M, keep),
                               atol=1e-12)


def test_select_bins_brute_force_with_ties():
    M, C = 220, 22
    r = rng(54)
    delta = r.normal(size=(6, C))
    delta[1, :] = 0.25                     # all equal: the lowest chunk indices win
    delta[2, [3, 9, 17]] = delta[2].max() + 1.0   # three-way tie at the top
    delta[3, 0] = -np.inf
    for ratio in [0.094, 0.125, 0.25, 0.5, 1.0, 0.0, 0.01]:
        n_c = min(max(int(math.floor(ratio * C + 0.5)), 1), C)
        got = orc.select_bins(delta, M, ratio)
        for l in range(delta.shape[0]):
            # brute force: repeatedly take the best remaining chunk, lower index on ties
            left = list(range(C))
            keep = []
            for _ in range(n_c):
                best = left[0]
                for c in left:
                    if delta[l, c] > delta[l, best]:
                        best = c
                keep.append(best)
                left.remove(best)
            ref = sorted(k for c in keep for k in range((c * M) // C, ((c + 1) * M) // C))
            assert got[l].dtype == np.int32 and list(got[l]) == ref
    assert [len(b) for b in orc.select_bins(delta, M, 0.094)] == [20] * 6     # round(2.07) = 2 chunks of 10
    assert list(orc.select_bins(delta, M, 0.125)[1]) == list(range(30))        # round(2.75) = 3, all-equal layer
    assert len(orc.select_bins(delta, M, 0.25)[0]) == 60                       # 5.5 rounds half up to 6


def test_select_bins_uneven_chunks_and_count_rule():
    # M not divisible by C: floor boundaries; every layer's list is sorted, unique, inside [0, M)
    M, C = 1000, 22
    delta = rng(55).normal(size=(3, C))
    for ratio in [0.1, 0.3]:
        for b in orc.select_bins(delta, M, ratio):
            assert np.all(np.diff(b) > 0) and b[0] >= 0 and b[-1] < M
    top = int(np.argmax(delta[0]))
    one = orc.select_bins(delta, M, 0.0)[0]   # never fewer than one chunk
    assert list(one) == list(range((top * M) // C, ((top + 1) * M) // C))


# ------------------------------------------------------------ the (N-1)/N -> 1 shortcut (Sec. 4.1)
def test_shortcut_recursion_matches_its_closed_form_and_token_weights():
    M, d, extra = 16, 3, 37
    r = rng(60)
    xs = r.normal(size=(M + extra, d))
    bins = [0, 1, 5, 9, 15]
    S = orc.prefill(xs[:M], bins)
    for t in range(extra):
        S = orc.append_shortcut(S, xs[M + t], M + t, bins, M)
    np.testing.assert_allclose(S, orc.closed_form_shortcut(xs, M, bins), atol=1e-13)
    # DC bin (W_0 = 1): mean of the prefill plus sum of x_n / (n + 1) -- old tokens are never scaled down
    dc = xs[:M].mean(axis=0) + sum(xs[n] / (n + 1) for n in range(M, M + extra))
    np.testing.assert_allclose(S[0], dc, atol=1e-13)
    # a unit impulse appended at step n0 and nothing else: weight 1/(n0+1), slot T - n0
    imp = np.zeros((M + extra, 1))
    n0 = M + 4
    imp[n0] = 1.0
    T = M + extra
    k = np.array(bins)
    ref = np.exp(-2j * np.pi * k * (T - n0) / M)[:, None] / (n0 + 1)
    np.testing.assert_allclose(orc.closed_form_shortcut(imp, M, bins), ref, atol=1e-14)


def test_shortcut_differs_from_the_exact_rule_by_the_missing_decay():
    # exact rule: every token weighs 1/T.  Shortcut: prefill tokens 1/M, token n 1/(n+1).  With only
    # prefill tokens non-zero the two states differ exactly by the factor T/M.
    M, d, extra = 8, 2, 5
    xs = np.vstack([rng(61).normal(size=(M, d)), np.zeros((extra, d))])
    bins = np.arange(M)
    T = M + extra
    np.testing.assert_allclose(orc.closed_form_shortcut(xs, M, bins), orc.closed_form(xs, M, bins) * T / M,
                               atol=1e-13)
    # in general the relative distance grows with the number of appended tokens
    r = rng(62)
    xs = r.normal(size=(64 + 64, 4))
    d1 = [np.linalg.norm(orc.closed_form_shortcut(xs[:T], 64, bins) - orc.closed_form(xs[:T], 64, bins)) /
          np.linalg.norm(orc.closed_form(xs[:T], 64, bins)) for T in (65, 80, 128)]
    assert d1[0] < d1[1] < d1[2] and d1[0] < 0.05 and d1[2] > 0.3


# ------------------------------------------------------------ why the coefficients stay fp32
def test_half_precision_coefficient_storage_misses_the_bar():
    # A study, not a pin: the streaming update with the accumulator rounded to fp16 after every
    # token (what half-precision coefficient storage would do) against the float64 stream.  The update adds
    # a term of size |x| to an accumulator of size |x| sqrt(T); fp16 carries 11 bits, so the added term
    # loses most of its own bits and the rel-L2 error ends orders of magnitude above the 1e-4 target.
    M, d, steps = 1024, 8, 256
    r = rng(70)
    xs = r.normal(size=(M + steps, d))
    bins = np.arange(0, 256)
    k = bins[:, None].astype(np.float64)
    U = np.fft.fft(xs[:M], axis=0)[bins]                     # un-normalised state, as stored
    Uh = (U.real.astype(np.float16) + 1j * U.imag.astype(np.float16)).astype(np.complex128)
    err0 = np.linalg.norm(Uh - U) / np.linalg.norm(U)        # storage rounding alone
    for t in range(steps):
        tw = np.exp(2j * np.pi * ((bins * t) % M) / M)[:, None]   # fixed-frame update: F += x e^{+j 2 pi k (T-M)/M}
        U = U + tw * xs[M + t][None, :]
        Uh = Uh + tw * xs[M + t][None, :]
        Uh = (Uh.real.astype(np.float16) + 1j * Uh.imag.astype(np.float16)).astype(np.complex128)
    err = np.linalg.norm(Uh - U) / np.linalg.norm(U)
    assert 1e-4 < err0 < 1e-3          # one rounding: ~3e-4, already above the target
    assert err > 2e-3                  # and it grows with every token
    # fp32 accumulators under the same schedule stay near 1e-7
    U32 = np.fft.fft(xs[:M], axis=0)[bins].astype(np.complex64)
    for t in range(steps):
        tw = np.exp(2j * np.pi * ((bins * t) % M) / M)[:, None].astype(np.complex64)
        U32 = (U32 + tw * xs[M + t][None, :].astype(np.float32)).astype(np.complex64)
    assert np.linalg.norm(U32 - U) / np.linalg.norm(U) < 1e-6
