"""GPU parity: every C-ABI call against the float64 oracle on the same seeded inputs.

Tolerances (relative L2 over the compared tensor):
  coefficients (fp32 complex)            1e-4   (stated target)
  attention output, bf16 storage         2e-2   (stated target)
  attention output, fp32 storage         1e-4   (fp32 arithmetic: FFT + exp of scores of
                                                 magnitude <~ 50 gives ~1e-5; one decade of slack)
  reconstruction, fp32 / bf16 storage    1e-4 / 4e-3 (bf16 rounding alone is 2^-9 per element)
Kept-bin masks read back from the device must be bit-exact.
"""
import numpy as np
import pytest
import torch

from oracle import iwdft_oracle as orc
from paper_2507_20030_amd import binding as B
from paper_2507_20030_amd import workload as wl

pytestmark = pytest.mark.gpu

TOL_COEF = 1e-4
TOL_ATTN = {torch.float32: 1e-4, torch.bfloat16: 2e-2}
TOL_REC = {torch.float32: 1e-4, torch.bfloat16: 4e-3}
DEV = "cuda:0"


def rel_l2(a, ref):
    return float(np.linalg.norm(np.asarray(a) - ref) / max(np.linalg.norm(ref), 1e-300))


def f64(t):
    return t.detach().to("cpu").to(torch.float64).numpy()


def c128(t):
    return t.detach().to("cpu").numpy().astype(np.complex128)


def make_cache(cfg, bins, weights=None, flags=0, write_every=0):
    return B.Cache(cfg.n_layers, cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.torch_dtype,
                   cfg.L, bins, weights, flags, DEV, n_sink=cfg.n_sink, n_recent=cfg.n_recent,
                   write_every=write_every)


class SliceOracle:
    """Float64 state of a few sampled slices, advanced next to the GPU cache: coefficients of the
    transformed middle segment plus the exact sink tokens and the recent window (Sec. 4.2)."""

    def __init__(self, cfg, bins, weights, K, V, slices):
        self.cfg, self.bins, self.weights, self.slices = cfg, bins, weights, slices
        self.M = cfg.L
        self.T = cfg.L
        self.S, self.sink, self.recent = {}, {}, {}
        s0, s1 = cfg.n_sink, cfg.n_sink + cfg.L
        for key in slices:
            l = key[0]
            k, v = f64(K[key]), f64(V[key])
            self.S[key] = [orc.prefill(k[s0:s1], bins[l]), orc.prefill(v[s0:s1], bins[l])]
            self.sink[key] = (k[:s0], v[:s0])
            self.recent[key] = ([r for r in k[s1:]], [r for r in v[s1:]])

    def append(self, tk, tv):
        for key, st in self.S.items():
            l = key[0]
            rk, rv = self.recent[key]
            rk.append(f64(tk[key]))
            rv.append(f64(tv[key]))
            st[0] = orc.append(st[0], rk.pop(0), self.T, self.bins[l], self.M)
            st[1] = orc.append(st[1], rv.pop(0), self.T, self.bins[l], self.M)
        self.T += 1

    def attend(self, q):
        G, d = self.cfg.group, self.cfg.head_dim
        out = {}
        for key, st in self.S.items():
            l, b, h = key
            w = None if self.weights is None else self.weights[l]
            rk, rv = self.recent[key]
            rk = np.stack(rk) if rk else np.zeros((0, d))
            rv = np.stack(rv) if rv else np.zeros((0, d))
            out[key] = orc.windowed_attention(f64(q[l, b, h * G:(h + 1) * G]), self.sink[key][0], self.sink[key][1],
                                              st[0], st[1], self.T, self.M, self.bins[l], rk, rv, w)
        return out

    def reconstruct(self, key, which):
        l = key[0]
        w = None if self.weights is None else self.weights[l]
        return orc.reconstruct(self.S[key][which], self.T, self.M, self.bins[l], w)


def check_coeffs(cache, ora, tag):
    worst = 0.0
    for l in sorted({k[0] for k in ora.S}):
        SK, SV = cache.export_coeffs(l)
        for (ll, b, h), st in ora.S.items():
            if ll != l:
                continue
            worst = max(worst, rel_l2(c128(SK[b, h]), st[0]), rel_l2(c128(SV[b, h]), st[1]))
    assert worst < TOL_COEF, f"{tag}: coefficient rel-L2 {worst:.3e}"
    return worst


def check_attn(cfg, cache, ora, q, tag):
    out = cache.attend(q)
    ref = ora.attend(q)
    G = cfg.group
    worst = 0.0
    for (l, b, h), r in ref.items():
        worst = max(worst, rel_l2(f64(out[l, b, h * G:(h + 1) * G]), r))
    assert worst < TOL_ATTN[cfg.torch_dtype], f"{tag}: attention rel-L2 {worst:.3e}"
    return worst


def check_reconstruct(cfg, cache, ora, a0, n, tag):
    worst = 0.0
    for l in sorted({k[0] for k in ora.S}):
        Kt, Vt = cache.reconstruct(l, a0, n)
        for key in ora.S:
            if key[0] != l:
                continue
            _, b, h = key
            worst = max(worst, rel_l2(f64(Kt[b, h]), ora.reconstruct(key, 0)[a0:a0 + n]),
                        rel_l2(f64(Vt[b, h]), ora.reconstruct(key, 1)[a0:a0 + n]))
    assert worst < TOL_REC[cfg.torch_dtype], f"{tag}: reconstruction rel-L2 {worst:.3e}"
    return worst


def check_masks(cache, bins):
    for l, b in enumerate(bins):
        got = cache.export_bins(l).cpu().numpy()
        assert got.dtype == np.int32 and np.array_equal(got, np.asarray(b, np.int32)), f"mask of layer {l}"


def run_stream(cfg, bins, weights=None, flags=0, steps=None, slices=None, rec=(0, 64), tag="", fused=False,
               write_every=0):
    steps = cfg.steps if steps is None else steps
    slices = wl.sample_slices(cfg) if slices is None else slices
    K, V = wl.prefill_tensors(cfg, DEV)
    cache = make_cache(cfg, bins, weights, flags, write_every)
    check_masks(cache, bins)
    cache.prefill(K, V)
    assert cache.T == cfg.L
    ora = SliceOracle(cfg, bins, weights, K, V, slices)
    del K, V
    stats = {"coef0": check_coeffs(cache, ora, tag + " prefill")}
    stats["rec0"] = check_reconstruct(cfg, cache, ora, rec[0], rec[1], tag + " prefill")
    worst_attn = 0.0
    for i in range(steps):
        tk, tv, q = wl.decode_step(cfg, i, DEV)
        ora.append(tk, tv)
        if fused:  # one call: append, then attend
            out = cache.step(tk, tv, q)
            ref = ora.attend(q)
            G = cfg.group
            w = max(rel_l2(f64(out[l, b, h * G:(h + 1) * G]), r) for (l, b, h), r in ref.items())
            assert w < TOL_ATTN[cfg.torch_dtype], f"{tag} fused step {i}: attention rel-L2 {w:.3e}"
            worst_attn = max(worst_attn, w)
        else:
            cache.append(tk, tv)
            worst_attn = max(worst_attn, check_attn(cfg, cache, ora, q, f"{tag} step {i}"))
    assert cache.T == cfg.L + steps
    stats["attn"] = worst_attn
    stats["coefN"] = check_coeffs(cache, ora, tag + " after appends")
    stats["recN"] = check_reconstruct(cfg, cache, ora, max(0, cfg.L - rec[1]), min(rec[1], cfg.L), tag + " end")
    torch.cuda.synchronize()
    print(f"\n[{tag}] " + " ".join(f"{k}={v:.2e}" for k, v in stats.items()), flush=True)
    cache.close()
    return stats


def small_cfg(**kw):
    base = dict(name="small", n_layers=2, batch=2, n_kv_heads=2, group=2, head_dim=128, L=256, n_bins=40,
                steps=5, dtype="f32", mask="low", seed=3)
    base.update(kw)
    return wl.Config(**base)


def random_bins(cfg, seed):
    rng = np.random.default_rng(seed)
    return [np.sort(rng.choice(cfg.L, size=cfg.n_bins - (l % 2), replace=False)).astype(np.int32)
            for l in range(cfg.n_layers)]


def test_cfg1_full_stream_fft_path():
    cfg = wl.CONFIGS["cfg1"]
    run_stream(cfg, wl.layer_bins(cfg), tag="cfg1")


def test_cfg1_direct_synthesis_path():
    cfg = wl.CONFIGS["cfg1"]
    run_stream(cfg, wl.layer_bins(cfg), flags=B.IWDFT_FLAG_DIRECT_SYNTHESIS, steps=3, tag="cfg1-direct")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,group", [(256, 2), (1024, 3), (96, 1), (160, 2), (2048, 8)])
def test_ragged_random_masks(dtype, L, group):
    # odd bin counts (ragged rows), scattered bins (folding collisions), batch > 1, odd group size,
    # non-power-of-two M (direct synthesis), wrap-around of the slot shift (steps > 0 with small M);
    # 96 and 160 tokens: a ragged last tile and an odd number of 64-token tiles in the dense prefill
    cfg = small_cfg(L=L, group=group, dtype=dtype, n_bins=min(77, L // 2 + 5))
    run_stream(cfg, random_bins(cfg, 11), rec=(3, 50), tag=f"ragged-{dtype}-L{L}-G{group}")


def test_bin_weights_one_sided():
    cfg = small_cfg(L=512, n_bins=257, group=2)
    bins = [np.arange(257, dtype=np.int32) for _ in range(cfg.n_layers)]
    w = [np.where((b == 0) | (b == 256), 1.0, 2.0).astype(np.float32) for b in bins]
    st = run_stream(cfg, bins, weights=w, steps=2, tag="one-sided")
    # the weights also scale the deferred tokens' rank-one terms: fused steps with write-back every 4th
    run_stream(cfg, bins, weights=w, steps=6, fused=True, write_every=4, tag="one-sided-deferred")
    # with every bin of a real signal represented, reconstruction at T = M is the input itself
    K, V = wl.prefill_tensors(cfg, DEV)
    cache = make_cache(cfg, bins, w)
    cache.prefill(K, V)
    Kt, Vt = cache.reconstruct(1, 0, cfg.L)
    assert rel_l2(f64(Kt), f64(K[1])) < 1e-5 and rel_l2(f64(Vt), f64(V[1])) < 1e-5
    cache.close()


@pytest.mark.parametrize("L", [100, 75])
def test_bin_weights_one_sided_any_length(L):
    # the same one-sided synthesis where M is not a power of two (chirp-z attention, dense prefill, direct
    # reconstruction); odd M has no Nyquist bin
    cfg = small_cfg(L=L, n_bins=L // 2 + 1, group=3)
    bins = [np.arange(L // 2 + 1, dtype=np.int32) for _ in range(cfg.n_layers)]
    w = [np.where((b == 0) | (2 * b == L), 1.0, 2.0).astype(np.float32) for b in bins]
    run_stream(cfg, bins, weights=w, steps=3, rec=(0, 32), tag=f"one-sided-{L}")
    run_stream(cfg, bins, weights=w, steps=3, rec=(0, 32), fused=True, tag=f"one-sided-{L}-fused")
    K, V = wl.prefill_tensors(cfg, DEV)
    cache = make_cache(cfg, bins, w)
    assert B.iwdft_attn_kind(cache.ctx) == "chirp"
    cache.prefill(K, V)
    Kt, Vt = cache.reconstruct(1, 0, cfg.L)
    assert rel_l2(f64(Kt), f64(K[1])) < 1e-5 and rel_l2(f64(Vt), f64(V[1])) < 1e-5
    cache.close()


def test_many_wraps_slot_shift():
    # more appends than M: the shift (T - M) mod M wraps several times
    cfg = small_cfg(L=64, n_bins=20, group=1, steps=150, n_layers=1, batch=1)
    run_stream(cfg, random_bins(cfg, 5), rec=(0, 64), tag="wraps")


def test_call_order_and_argument_errors():
    cfg = small_cfg()
    bins = random_bins(cfg, 1)
    cache = make_cache(cfg, bins)
    tk, tv, q = wl.decode_step(cfg, 0, DEV)
    for fn in (lambda: cache.append(tk, tv), lambda: cache.attend(q), lambda: cache.export_coeffs(0),
               lambda: cache.reconstruct(0, 0, 4)):
        with pytest.raises(B.IwdftError) as e:
            fn()
        assert e.value.code == B.IWDFT_ERR_STATE
    K, V = wl.prefill_tensors(cfg, DEV)
    cache.prefill(K, V)
    for fn, code in ((lambda: cache.reconstruct(5, 0, 4), B.IWDFT_ERR_ARG),
                     (lambda: cache.reconstruct(0, cfg.L - 2, 4), B.IWDFT_ERR_ARG),
                     (lambda: cache.export_coeffs(-1), B.IWDFT_ERR_ARG),
                     (lambda: B.iwdft_set_num_tokens(cache.ctx, cfg.L - 1), B.IWDFT_ERR_ARG)):
        with pytest.raises(B.IwdftError) as e:
            fn()
        assert e.value.code == code
    small = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.IwdftError) as e:
        B.iwdft_create(cache.desc, small, cache.workspace)
    assert e.value.code == B.IWDFT_ERR_SIZE
    cache.close()


def test_checkpoint_resume_is_bitwise():
    cfg = small_cfg(steps=6)
    bins = random_bins(cfg, 2)
    K, V = wl.prefill_tensors(cfg, DEV)
    cache = make_cache(cfg, bins)
    cache.prefill(K, V)
    steps = [wl.decode_step(cfg, i, DEV) for i in range(6)]
    for tk, tv, _ in steps[:2]:
        cache.append(tk, tv)
    saved, T = cache.state.clone(), cache.T
    for tk, tv, _ in steps[2:]:
        cache.append(tk, tv)
    a = cache.attend(steps[5][2]).clone()
    end = cache.state.clone()
    cache.state.copy_(saved)
    B.iwdft_set_num_tokens(cache.ctx, T)
    for tk, tv, _ in steps[2:]:
        cache.append(tk, tv)
    assert torch.equal(cache.state, end)
    assert torch.equal(cache.attend(steps[5][2]), a)
    cache.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,S,R,group", [(256, 10, 50, 2), (1024, 3, 1, 3), (96, 4, 7, 1), (512, 0, 5, 4),
                                         (512, 6, 0, 8)])
def test_sink_and_recent_windows(dtype, L, S, R, group):
    # exact sink / recent tokens join the softmax; more appends than R so that the ring wraps and every
    # original recent token and several appended ones have aged into the coefficients
    cfg = small_cfg(L=L, group=group, dtype=dtype, n_bins=41, n_sink=S, n_recent=R, steps=max(6, R + 3) if R < 10 else 7)
    run_stream(cfg, random_bins(cfg, 17), rec=(2, 40), tag=f"windows-{dtype}-L{L}-S{S}-R{R}-G{group}")


def test_windows_all_bins_equals_full_attention_over_the_whole_context():
    # every bin kept, nothing appended beyond the recent hand-over: the assembled cache is the complete
    # context, so the library must reproduce plain softmax attention over all S + M + R tokens
    cfg = small_cfg(L=256, n_bins=256, group=2, dtype="f32", n_sink=5, n_recent=9, n_layers=1, batch=1, steps=0)
    bins = [np.arange(256, dtype=np.int32)]
    K, V = wl.prefill_tensors(cfg, DEV)
    cache = make_cache(cfg, bins)
    cache.prefill(K, V)
    _, _, q = wl.decode_step(cfg, 0, DEV)
    out = cache.attend(q)
    G = cfg.group
    for h in range(cfg.n_kv_heads):
        ref = orc.attention(f64(q[0, 0, h * G:(h + 1) * G]), f64(K[0, 0, h]), f64(V[0, 0, h]))
        assert rel_l2(f64(out[0, 0, h * G:(h + 1) * G]), ref) < 1e-5
    cache.close()


def test_cfg2_with_paper_windows_full_size():
    cfg = wl.CONFIGS["cfg2w"]
    run_stream(cfg, wl.layer_bins(cfg), steps=3, tag="cfg2w")


def test_fused_step_cfg1():
    cfg = wl.CONFIGS["cfg1"]
    run_stream(cfg, wl.layer_bins(cfg), fused=True, tag="cfg1-fused")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,S,R,group", [(256, 0, 0, 2), (1024, 3, 5, 3), (96, 4, 7, 1), (2048, 0, 0, 8),
                                         (512, 2, 3, 16)])
def test_fused_step_ragged_and_windows(dtype, L, S, R, group):
    # the fused call must give what append + attend give; group 16 needs two head passes and takes the
    # unfused sequence inside the library
    cfg = small_cfg(L=L, group=group, dtype=dtype, n_bins=min(77, L // 2 + 5), n_sink=S, n_recent=R, steps=9)
    run_stream(cfg, random_bins(cfg, 23), rec=(3, 50), fused=True, tag=f"fused-{dtype}-L{L}-S{S}-R{R}-G{group}")


def test_fused_step_leaves_the_same_state_as_append():
    cfg = small_cfg(L=512, n_bins=100, group=4, dtype="bf16", n_sink=3, n_recent=4, steps=6)
    bins = random_bins(cfg, 29)
    K, V = wl.prefill_tensors(cfg, DEV)
    a, b = make_cache(cfg, bins), make_cache(cfg, bins)
    a.prefill(K, V)
    b.prefill(K, V)
    for i in range(cfg.steps):
        tk, tv, q = wl.decode_step(cfg, i, DEV)
        a.append(tk, tv)
        oa = a.attend(q)
        ob = b.step(tk, tv, q)
        assert rel_l2(f64(ob), f64(oa)) < 5e-3
    assert a.T == b.T
    for l in range(cfg.n_layers):
        (ka, va), (kb, vb) = a.export_coeffs(l), b.export_coeffs(l)
        assert rel_l2(c128(kb), c128(ka)) < 1e-6 and rel_l2(c128(vb), c128(va)) < 1e-6
    a.close()
    b.close()


def test_phase_timing_marks_calls_without_changing_results():
    cfg = small_cfg(L=1024, n_bins=200, group=4, dtype="bf16", n_sink=2, n_recent=3, steps=4)
    bins = random_bins(cfg, 31)
    K, V = wl.prefill_tensors(cfg, DEV)
    a, b = make_cache(cfg, bins), make_cache(cfg, bins)
    a.prefill(K, V)
    b.prefill(K, V)
    B.iwdft_phase_timing(b.ctx, True)
    for i in range(cfg.steps):
        tk, tv, q = wl.decode_step(cfg, i, DEV)
        oa = a.step(tk, tv, q)
        ob = b.step(tk, tv, q)
        assert torch.equal(oa, ob)
        assert torch.equal(a.attend(q), b.attend(q))
    ms, n = B.iwdft_phase_times(b.ctx)
    assert n == 2 * cfg.steps and all(0.0 < m < 1e3 for m in ms)
    ms, n = B.iwdft_phase_times(b.ctx)       # the read-out cleared the list
    assert n == 0 and ms == [0.0, 0.0, 0.0]
    B.iwdft_phase_timing(b.ctx, False)
    tk, tv, q = wl.decode_step(cfg, 0, DEV)
    b.step(tk, tv, q)
    assert B.iwdft_phase_times(b.ctx)[1] == 0
    a.close()
    b.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,S,R,group,J", [(256, 0, 0, 2, 2), (1024, 3, 5, 3, 8), (512, 0, 4, 1, 3), (2048, 0, 0, 8, 8),
                                           (4096, 2, 0, 4, 5), (16384, 0, 3, 4, 8), (512, 2, 3, 16, 8),
                                           (96, 0, 0, 2, 8), (1024, 2, 3, 4, 16), (8192, 0, 0, 2, 13),
                                           (32768, 0, 2, 4, 16)])
def test_deferred_write_back_stream(dtype, L, S, R, group, J):
    # the coefficients are written back every J-th fused step only; every step's attention still has to
    # match the oracle, and so do the coefficients once the deferred tokens are flushed (19 steps: several
    # write-backs and a partial batch at the end).  group 16 and M = 96 cannot defer and run with J = 1.
    big = L > 8192
    cfg = small_cfg(L=L, group=group, dtype=dtype, n_bins=min(77, L // 2 + 5), n_sink=S, n_recent=R,
                    steps=19 if J <= 8 else 37,
                    n_layers=1 if big else 2)
    run_stream(cfg, random_bins(cfg, 47), rec=(3, 50), fused=True, write_every=J,
               tag=f"defer-{dtype}-L{L}-S{S}-R{R}-G{group}-J{J}")


@pytest.mark.parametrize("L,n_bins", [(16384, 1600), (16384, 3000), (8192, 4096), (32768, 900)])
def test_deferred_write_back_every_fft_kernel_variant(L, n_bins):
    # the pending tokens are weighed in the epilogue of attention kernel B, which exists in several
    # register-budget variants (2, 4 or 8 kept bins per thread, one or many transform blocks): all of
    # them with 16 deferred tokens, windows included
    cfg = small_cfg(L=L, group=4, dtype="bf16", n_bins=n_bins, n_sink=2, n_recent=3, steps=18, n_layers=1, batch=1)
    run_stream(cfg, random_bins(cfg, 79), rec=(3, 50), fused=True, write_every=16, tag=f"defer-variants-L{L}-B{n_bins}")


def test_deferred_write_back_mixed_with_other_calls():
    # any call other than the fused step first writes the deferred tokens back: a random mix of calls
    # gives, step for step, what the oracle gives
    cfg = small_cfg(L=1024, n_bins=150, group=4, dtype="bf16", n_sink=2, n_recent=3, steps=40, n_layers=1)
    bins = random_bins(cfg, 53)
    K, V = wl.prefill_tensors(cfg, DEV)
    cache = make_cache(cfg, bins, write_every=8)
    cache.prefill(K, V)
    slices = wl.sample_slices(cfg, 4)
    ora = SliceOracle(cfg, bins, None, K, V, slices)
    rng = np.random.default_rng(5)
    G = cfg.group
    for i in range(cfg.steps):
        tk, tv, q = wl.decode_step(cfg, i, DEV)
        ora.append(tk, tv)
        op = rng.integers(0, 5)
        if op <= 2:
            out = cache.step(tk, tv, q)
            ref = ora.attend(q)
            w = max(rel_l2(f64(out[l, b, h * G:(h + 1) * G]), r) for (l, b, h), r in ref.items())
            assert w < TOL_ATTN[cfg.torch_dtype], f"mixed step {i}: {w:.3e}"
        else:
            cache.append(tk, tv)
            check_attn(cfg, cache, ora, q, f"mixed append/attend {i}")
        if op == 1:
            check_attn(cfg, cache, ora, q, f"mixed attend after step {i}")      # same state, plain attention
        if op == 2 and i % 3 == 0:
            check_coeffs(cache, ora, f"mixed export {i}")
        if op == 0 and i % 4 == 0:
            check_reconstruct(cfg, cache, ora, 7, 40, f"mixed reconstruct {i}")
        assert cache.T == cfg.L + i + 1
    check_coeffs(cache, ora, "mixed end")
    cache.close()


def test_deferred_write_back_equals_immediate_and_checkpoints_after_flush():
    cfg = small_cfg(L=512, n_bins=100, group=4, dtype="bf16", n_sink=3, n_recent=4, steps=13)
    bins = random_bins(cfg, 59)
    K, V = wl.prefill_tensors(cfg, DEV)
    a, b = make_cache(cfg, bins), make_cache(cfg, bins, write_every=8)
    a.prefill(K, V)
    b.prefill(K, V)
    steps = [wl.decode_step(cfg, i, DEV) for i in range(cfg.steps)]
    for tk, tv, q in steps[:11]:                      # 11 steps: one write-back, three tokens deferred
        oa, ob = a.step(tk, tv, q), b.step(tk, tv, q)
        assert rel_l2(f64(ob), f64(oa)) < 5e-3
    b.flush()
    for l in range(cfg.n_layers):
        (ka, va), (kb, vb) = a.export_coeffs(l), b.export_coeffs(l)
        assert rel_l2(c128(kb), c128(ka)) < 1e-6 and rel_l2(c128(vb), c128(va)) < 1e-6
    saved, T = b.state.clone(), b.T                   # complete after the flush
    tail = [b.step(tk, tv, q).clone() for tk, tv, q in steps[11:]]
    b.state.copy_(saved)
    B.iwdft_set_num_tokens(b.ctx, T)
    again = [b.step(tk, tv, q).clone() for tk, tv, q in steps[11:]]
    assert all(torch.equal(x, y) for x, y in zip(tail, again))
    a.close()
    b.close()


@pytest.mark.parametrize("prefill", ["fft", "dense"])
def test_two_runs_are_bitwise_identical(prefill):
    # no kernel uses atomics or data-dependent orders: the same calls on the same inputs leave the same
    # bytes in the state buffer and return the same outputs (whole-buffer comparison, all slices)
    cfg = small_cfg(L=2048, n_bins=333, group=4, dtype="bf16", n_sink=2, n_recent=5, steps=11, n_layers=3, batch=2)
    bins = random_bins(cfg, 67)
    flags = B.IWDFT_FLAG_FFT_PREFILL if prefill == "fft" else B.IWDFT_FLAG_DENSE_PREFILL
    K, V = wl.prefill_tensors(cfg, DEV)
    states, outs = [], []
    for run in range(2):
        c = make_cache(cfg, bins, flags=flags, write_every=4)
        c.prefill(K, V)
        o = []
        for i in range(cfg.steps):
            tk, tv, q = wl.decode_step(cfg, i, DEV)
            if i % 5 == 3:
                c.append(tk, tv)
                o.append(c.attend(q).clone())
            else:
                o.append(c.step(tk, tv, q).clone())
        c.flush()
        torch.cuda.synchronize()
        states.append(c.state.clone())
        outs.append(o)
        c.close()
    assert torch.equal(states[0], states[1])
    assert all(torch.equal(a, b) for a, b in zip(outs[0], outs[1]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,S,R,group,steps", [(256, 0, 0, 2, 64), (1024, 3, 5, 4, 9), (96, 0, 2, 1, 200)])
def test_shortcut_flag_matches_the_oracle_recursion(dtype, L, S, R, group, steps):
    """IWDFT_FLAG_SHORTCUT: Sec. 4.1's update with (N-1)/N taken as 1, inside the library (the token's scale
    M / (T+1) is applied by the append kernel, the gain T/M by every reader).  Exported coefficients against the
    oracle's shortcut recursion and its closed form, attention and reconstruction against the oracle run on that
    state; both the two calls and iwdft_append_attn (which must fall back to them)."""
    cfg = small_cfg(L=L, n_bins=min(40, L // 2), group=group, dtype=dtype, steps=steps, n_layers=2, batch=1, n_sink=S,
                    n_recent=R)
    bins = random_bins(cfg, 71)
    K, V = wl.prefill_tensors(cfg, DEV)
    cache = B.Cache(cfg.n_layers, cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.torch_dtype, cfg.L,
                    bins, None, B.IWDFT_FLAG_SHORTCUT, DEV, n_sink=S, n_recent=R, write_every=8)
    cache.prefill(K, V)
    key = (1, 0, 1)
    l = key[0]
    k0, v0 = f64(K[key]), f64(V[key])
    SK, SV, T = orc.prefill(k0[S:S + L], bins[l]), orc.prefill(v0[S:S + L], bins[l]), L
    sink = (k0[:S], v0[:S])
    rk, rv = [r for r in k0[S + L:]], [r for r in v0[S + L:]]
    absorbed = [k0[S:S + L]]
    worst = 0.0
    G = cfg.group
    for i in range(cfg.steps):
        tk, tv, q = wl.decode_step(cfg, i, DEV)
        if i % 3 == 2:
            out = cache.step(tk, tv, q)
        else:
            cache.append(tk, tv)
            out = cache.attend(q)
        rk.append(f64(tk[key]))
        rv.append(f64(tv[key]))
        xk, xv = rk.pop(0), rv.pop(0)
        SK, SV = orc.append_shortcut(SK, xk, T, bins[l], L), orc.append_shortcut(SV, xv, T, bins[l], L)
        absorbed.append(xk[None, :])
        T += 1
        ref = orc.windowed_attention(f64(q[l, 0, G:2 * G]), sink[0], sink[1], SK, SV, T, L, bins[l],
                                     np.stack(rk) if rk else np.zeros((0, 128)), np.stack(rv) if rv else np.zeros((0, 128)))
        worst = max(worst, rel_l2(f64(out[l, 0, G:2 * G]), ref))
    assert worst < TOL_ATTN[cfg.torch_dtype], f"shortcut attention rel-L2 {worst:.3e}"
    assert cache.T == T
    gk, gv = cache.export_coeffs(l)
    e_rec = max(rel_l2(c128(gk[0, 1]), SK), rel_l2(c128(gv[0, 1]), SV))
    e_closed = rel_l2(c128(gk[0, 1]), orc.closed_form_shortcut(np.vstack(absorbed), L, bins[l]))
    assert e_rec < TOL_COEF and e_closed < TOL_COEF, f"shortcut coefficients {e_rec:.2e} / {e_closed:.2e}"
    Kt, Vt = cache.reconstruct(l, 0, L)
    e_k = rel_l2(f64(Kt[0, 1]), orc.reconstruct(SK, T, L, bins[l]))
    e_v = rel_l2(f64(Vt[0, 1]), orc.reconstruct(SV, T, L, bins[l]))
    assert max(e_k, e_v) < TOL_REC[cfg.torch_dtype]
    drift = rel_l2(SK, orc.closed_form(np.vstack(absorbed), L, bins[l]))
    print(f"\n[shortcut {dtype} M={L}] coefficients {e_rec:.2e} attention {worst:.2e} reconstruction {max(e_k, e_v):.2e}; "
          f"drift of the shortcut from the exact rule after {steps} appends: {drift:.2e}", flush=True)
    cache.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,n_bins,steps,grid", [(256, 100, 7, (3, 4, 60)), (1000, 77, 3, (0, 7, 143)), (4096, 300, 2, (5, 64, 64)),
                                                 (8192, 600, 9, (8191, 1, 1)), (96, 96, 100, (1, 5, 19))])
def test_reconstruct_on_a_strided_grid(dtype, L, n_bins, steps, grid):
    """iwdft_reconstruct_grid against the oracle's strided reconstruction (slots a0 + j * stride)."""
    cfg = small_cfg(L=L, n_bins=n_bins, group=1, dtype=dtype, steps=steps, n_layers=2, batch=2)
    bins = random_bins(cfg, 73)
    K, V = wl.prefill_tensors(cfg, DEV)
    cache = make_cache(cfg, bins)
    cache.prefill(K, V)
    slices = [(0, 0, 0), (1, 1, 1)]
    ora = SliceOracle(cfg, bins, None, K, V, slices)
    for i in range(steps):
        tk, tv, _ = wl.decode_step(cfg, i, DEV)
        cache.append(tk, tv)
        ora.append(tk, tv)
    a0, stride, n = grid
    worst = 0.0
    for (l, b, h) in slices:
        Kt, Vt = cache.reconstruct(l, a0, n, stride=stride)
        for which, got in ((0, Kt), (1, Vt)):
            ref = orc.reconstruct_grid(ora.S[(l, b, h)][which], ora.T, L, bins[l], a0, stride, n)
            worst = max(worst, rel_l2(f64(got[b, h]), ref))
    assert worst < TOL_REC[cfg.torch_dtype], f"grid reconstruction rel-L2 {worst:.3e}"
    with pytest.raises(B.IwdftError):
        cache.reconstruct(0, a0, n + 1 + (L - 1 - a0 - (n - 1) * stride) // stride, stride=stride)   # one row past M
    with pytest.raises(B.IwdftError):
        B.iwdft_reconstruct_grid(cache.ctx, 0, 0, 0, 1, None, None)
    cache.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,n_bins,steps", [(256, 100, 7), (512, 77, 3), (1024, 300, 1030), (2048, 77, 5), (4096, 1500, 2),
                                            (8192, 600, 9), (16384, 900, 4), (32768, 2100, 3)])
def test_reconstruct_long_ranges_through_ffts(dtype, L, n_bins, steps):
    # long slot ranges take the inverse-FFT kernel (all transform lengths, the decimated form beyond 8192,
    # a non-zero slot shift after appends, wrap-around of the shift); ranges: everything, an offset half,
    # and a short one that stays with the direct contraction -- all against the oracle
    big = L > 8192
    cfg = small_cfg(L=L, dtype=dtype, n_bins=n_bins, steps=steps, group=1, n_layers=1 if big else 2,
                    batch=1 if big else 2)
    bins = random_bins(cfg, 73)
    w = [np.random.default_rng(l).uniform(0.5, 2.0, size=len(b)).astype(np.float32) for l, b in enumerate(bins)]
    K, V = wl.prefill_tensors(cfg, DEV)
    cache = make_cache(cfg, bins, w)
    cache.prefill(K, V)
    ora = SliceOracle(cfg, bins, w, K, V, wl.sample_slices(cfg, 4))
    for i in range(steps):
        tk, tv, _ = wl.decode_step(cfg, i % 32, DEV)
        cache.append(tk, tv)
        ora.append(tk, tv)
    for a0, n in [(0, L), (L // 4 + 3, L // 2), (5, 16)]:
        check_reconstruct(cfg, cache, ora, a0, n, f"rec-fft-{dtype}-L{L} [{a0}, {a0 + n})")
    # and the same numbers as the direct contraction (forced by the flag) to a few ulps of the output
    direct = make_cache(cfg, bins, w, flags=B.IWDFT_FLAG_DIRECT_SYNTHESIS)
    direct.prefill(K, V)
    for i in range(steps):
        tk, tv, _ = wl.decode_step(cfg, i % 32, DEV)
        direct.append(tk, tv)
    Ka, Va = cache.reconstruct(0, 0, L)
    Kb, Vb = direct.reconstruct(0, 0, L)
    assert rel_l2(f64(Ka), f64(Kb)) < TOL_REC[cfg.torch_dtype] and rel_l2(f64(Va), f64(Vb)) < TOL_REC[cfg.torch_dtype]
    cache.close()
    direct.close()


def test_deferred_write_back_many_wraps():
    # more steps than M: the slot shifts of the deferred tokens wrap around inside a batch
    cfg = small_cfg(L=256, n_bins=60, group=2, steps=530, n_layers=1, batch=1, dtype="f32")
    run_stream(cfg, random_bins(cfg, 61), fused=True, write_every=8, tag="defer-wraps")


def test_fused_step_cfg2_windows_full_size():
    cfg = wl.CONFIGS["cfg2w"]
    run_stream(cfg, wl.layer_bins(cfg), steps=3, fused=True, tag="cfg2w-fused")


@pytest.mark.parametrize("prefill,fused,J,steps", [("fft", True, 16, 18), ("fft", True, 8, 10), ("fft", True, 1, 3),
                                                   ("fft", False, 0, 3),
                                                   ("dense", False, 0, 3)])
def test_cfg2_full_size_sampled_slices(prefill, fused, J, steps):
    # ("fft", True, 16) is the launch configuration the benchmark times: FFT prefill, fused decode step,
    # coefficients written back every 16th step (18 steps: one write-back, two tokens left deferred)
    cfg = wl.CONFIGS["cfg2"]
    flags = B.IWDFT_FLAG_FFT_PREFILL if prefill == "fft" else B.IWDFT_FLAG_DENSE_PREFILL
    run_stream(cfg, wl.layer_bins(cfg), flags=flags, steps=steps, fused=fused, write_every=J,
               tag=f"cfg2-{prefill}-fused{int(fused)}-J{J}")


@pytest.mark.parametrize("L,n_bins", [(1, 1), (2, 1), (2, 2), (3, 2), (64, 1), (64, 64)])
def test_degenerate_sizes(L, n_bins):
    # one-token caches, a single kept bin, every bin kept; alternating two-call / fused steps
    cfg = small_cfg(L=L, n_bins=n_bins, group=2, steps=4, n_layers=1, batch=2)
    bins = [np.arange(n_bins, dtype=np.int32)]
    for fused in (False, True):
        run_stream(cfg, bins, rec=(0, L), fused=fused, tag=f"degenerate-L{L}-B{n_bins}-f{int(fused)}")


def test_dc_only_mask_outputs_the_mean_value_row():
    # |B| = {0}: every reconstructed slot is the same vector, so attention returns exactly the
    # reconstructed V row whatever the query: (1/M) * sum of all tokens seen
    cfg = small_cfg(L=1024, n_bins=1, group=2, steps=3, n_layers=1, batch=1, dtype="f32")
    bins = [np.zeros(1, np.int32)]
    K, V = wl.prefill_tensors(cfg, DEV)
    cache = make_cache(cfg, bins)
    cache.prefill(K, V)
    tot = f64(V[0, 0]).sum(axis=1)                    # [kv heads, d]
    for i in range(cfg.steps):
        tk, tv, q = wl.decode_step(cfg, i, DEV)
        out = cache.step(tk, tv, q)
        tot = tot + f64(tv[0, 0])
        ref = np.repeat(tot / cfg.L, cfg.group, axis=0)
        assert rel_l2(f64(out[0, 0]), ref) < 1e-5
    cache.close()


@pytest.mark.parametrize("L,n_bins,group,dtype,S,R", [
    (8192, 4096, 2, "bf16", 0, 0),     # the most bins the register-resident kernels take
    (8192, 4100, 2, "bf16", 0, 0),     # one step beyond: the bin-strided kernels, single transform
    (8192, 8192, 3, "f32", 2, 6),      # every bin kept; a last head pair with one head; windows
    (16384, 5000, 4, "bf16", 0, 0),    # two decimated blocks, running sums kept in the output rows
    (32768, 9000, 2, "f32", 4, 4),     # four blocks, fp32 tokens, windows
    (32768, 16384, 1, "bf16", 0, 0),   # half of all bins (mirror-closed sets collide in every slot), one query head
])
def test_more_than_4096_kept_bins_per_layer(L, n_bins, group, dtype, S, R):
    """Up to 4096 kept bins per layer the FFT kernels hold per-bin values in registers; beyond that the prefill and the
    decode attention walk the bin list in strides of the workgroup (and keep running sums in their output rows), still
    O(M log M).  Every step against the oracle, two calls and fused; the deferred write-back is taken as 1 there."""
    cfg = small_cfg(L=L, n_bins=n_bins, group=group, steps=3, n_layers=1, batch=1, n_kv_heads=2, dtype=dtype,
                    n_sink=S, n_recent=R)
    bins = [np.sort(np.random.default_rng(3).choice(cfg.L, size=n_bins, replace=False)).astype(np.int32)]
    cache = make_cache(cfg, bins, write_every=8)
    assert B.iwdft_prefill_kind(cache.ctx) == "fft" and B.iwdft_attn_kind(cache.ctx) == "fft"
    cache.close()
    run_stream(cfg, bins, rec=(5, 40), tag=f"bins-{L}-{n_bins}")
    run_stream(cfg, bins, rec=(5, 40), fused=True, write_every=8, tag=f"bins-{L}-{n_bins}-fused")
    if n_bins > 4096:   # and against the direct sums of the same library
        K, V = wl.prefill_tensors(cfg, DEV)
        a, d = make_cache(cfg, bins), make_cache(cfg, bins, flags=B.IWDFT_FLAG_DIRECT_SYNTHESIS | B.IWDFT_FLAG_DENSE_PREFILL)
        assert B.iwdft_attn_kind(d.ctx) == "direct" and B.iwdft_prefill_kind(d.ctx) == "dense"
        a.prefill(K, V)
        d.prefill(K, V)
        (ka, va), (kd, vd) = a.export_coeffs(0), d.export_coeffs(0)
        assert rel_l2(c128(ka), c128(kd)) < 2e-5 and rel_l2(c128(va), c128(vd)) < 2e-5
        _, _, q = wl.decode_step(cfg, 0, DEV)
        assert rel_l2(f64(a.attend(q)), f64(d.attend(q))) < (2e-5 if dtype == "f32" else 8e-3)
        a.close()
        d.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,S,R,group,n_bins", [(33, 0, 0, 1, 9), (100, 2, 3, 2, 100), (129, 0, 0, 3, 40), (1000, 10, 50, 4, 250),
                                                (2049, 0, 4, 2, 300), (3000, 0, 0, 8, 1500), (8191, 1, 1, 1, 700)])
def test_any_length_attention_through_chirp_transforms(dtype, L, S, R, group, n_bins):
    """M that is not a power of two (M = context - sink - recent in general): the attention runs O(M log M)
    chirp-z transforms, all four convolution lengths; every step against the oracle (two calls and the fused step,
    which writes back at every step here), and against the direct synthesis of the same library."""
    cfg = small_cfg(L=L, n_bins=n_bins, group=group, dtype=dtype, steps=4, n_layers=2, batch=1, n_sink=S, n_recent=R)
    bins = random_bins(cfg, 83)
    c = make_cache(cfg, bins, write_every=8)
    assert B.iwdft_attn_kind(c.ctx) == "chirp"
    c.close()
    run_stream(cfg, bins, tag=f"chirp-{L}", write_every=8, rec=(0, min(64, L)))
    run_stream(cfg, bins, tag=f"chirp-{L}-fused", fused=True, write_every=8, rec=(0, min(64, L)))
    K, V = wl.prefill_tensors(cfg, DEV)
    a, d = make_cache(cfg, bins), make_cache(cfg, bins, flags=B.IWDFT_FLAG_DIRECT_SYNTHESIS)
    assert B.iwdft_attn_kind(d.ctx) == "direct"
    a.prefill(K, V)
    d.prefill(K, V)
    _, _, q = wl.decode_step(cfg, 0, DEV)
    assert rel_l2(f64(a.attend(q)), f64(d.attend(q))) < (2e-5 if dtype == "f32" else 8e-3)
    a.close()
    d.close()


@pytest.mark.parametrize("L,S,R,group,n_bins,dtype", [
    (16324, 10, 50, 4, 1600, "bf16"),    # 16384 - 60 = 2 * 8162: the paper's windows cut out of a 16K context
    (32708, 10, 50, 2, 3000, "f32"),     # 32768 - 60 = 4 * 8177
    (24570, 0, 0, 3, 5000, "bf16"),      # 3 * 8190, more than 4096 bins, a last head pair with one head
    (8198, 0, 3, 1, 700, "f32"),         # 2 * 4099 (a prime block length), one query head
])
def test_long_contexts_that_are_not_a_power_of_two_through_decimated_chirp_transforms(L, S, R, group, n_bins, dtype):
    """M > 8192 that is not a power of two: Pb = M / Q decimated blocks of Q <= 8192 points, each through the chirp-z
    transforms, softmax online across the blocks.  Every step against the oracle (two calls and fused), and against the
    direct sums of the same library."""
    cfg = small_cfg(L=L, n_bins=n_bins, group=group, dtype=dtype, steps=3, n_layers=1, batch=1, n_sink=S, n_recent=R)
    bins = random_bins(cfg, 29)
    c = make_cache(cfg, bins)
    assert B.iwdft_attn_kind(c.ctx) == "chirp"
    c.close()
    run_stream(cfg, bins, tag=f"chirp-{L}", rec=(0, 64))
    run_stream(cfg, bins, tag=f"chirp-{L}-fused", fused=True, rec=(0, 64))
    K, V = wl.prefill_tensors(cfg, DEV)
    a, d = make_cache(cfg, bins), make_cache(cfg, bins, flags=B.IWDFT_FLAG_DIRECT_SYNTHESIS)
    a.prefill(K, V)
    d.prefill(K, V)
    _, _, q = wl.decode_step(cfg, 0, DEV)
    assert rel_l2(f64(a.attend(q)), f64(d.attend(q))) < (2e-5 if dtype == "f32" else 8e-3)
    a.close()
    d.close()


def test_long_prime_context_takes_the_direct_sums():
    cfg = small_cfg(L=10007, n_bins=300, group=2, dtype="f32", steps=2, n_layers=1, batch=1)
    bins = random_bins(cfg, 5)
    c = make_cache(cfg, bins)
    assert B.iwdft_attn_kind(c.ctx) == "direct"
    c.close()
    run_stream(cfg, bins, tag="direct-10007", rec=(0, 64))


def test_paper_windows_on_a_context_that_is_a_power_of_two_full_size():
    """cfg2's shape with the paper's windows cut out of an 8192-token context (Sec. 5.1: 10 sink + 50 recent tokens,
    M = 8192 - 60 = 8132): the realistic setting, chirp-z attention at full size."""
    cfg = wl.CONFIGS["cfg2x"]
    assert cfg.n_prefill == 8192
    bins = wl.layer_bins(cfg)
    c = make_cache(cfg, bins)
    assert B.iwdft_attn_kind(c.ctx) == "chirp" and B.iwdft_prefill_kind(c.ctx) == "dense"
    c.close()
    run_stream(cfg, bins, steps=3, tag="cfg2w-8132")
    run_stream(cfg, bins, steps=3, fused=True, tag="cfg2w-8132-fused")


@pytest.mark.parametrize("scale", [2.0 ** -6, 2.0 ** 9])
def test_dense_and_fft_prefill_agree_across_the_dense_path_input_range(scale):
    # the dense contraction works on fp16 operand pairs (documented range +-65504, full precision above 2^-14):
    # inside that range a K/V scale of 2^-6 ... 2^9 (values to ~2^-10 and ~2^14 with the 0.1-10 channel scales)
    # leaves both prefills within the coefficient tolerance of the oracle and of each other
    cfg = small_cfg(L=2048, n_bins=500, dtype="bf16", n_layers=1, batch=1, n_kv_heads=2)
    bins = random_bins(cfg, 91)
    K, V = wl.prefill_tensors(cfg, DEV)
    K, V = (K.float() * scale).to(K.dtype), (V.float() * scale).to(V.dtype)
    got = {}
    for name, flag in (("fft", B.IWDFT_FLAG_FFT_PREFILL), ("dense", B.IWDFT_FLAG_DENSE_PREFILL)):
        c = make_cache(cfg, bins, flags=flag)
        c.prefill(K, V)
        got[name] = c.export_coeffs(0)
        ref = orc.prefill(f64(K[0, 0, 1]), bins[0])
        assert rel_l2(c128(got[name][0][0, 1]), ref) < TOL_COEF, name
        c.close()
    assert rel_l2(c128(got["dense"][0]), c128(got["fft"][0])) < 2e-5 and rel_l2(c128(got["dense"][1]), c128(got["fft"][1])) < 2e-5


def test_most_exact_tokens():
    # S + R = 1024 is the most the library takes
    cfg = small_cfg(L=512, n_bins=60, group=2, steps=3, n_layers=1, batch=1, n_sink=500, n_recent=524, dtype="bf16")
    run_stream(cfg, random_bins(cfg, 43), fused=True, tag="max-exact")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("L,S,R,n_bins", [(256, 0, 0, 129), (512, 2, 3, 77), (1024, 0, 0, 300), (2048, 0, 5, 77),
                                          (4096, 0, 0, 1500), (8192, 4, 0, 600), (16384, 0, 0, 900),
                                          (32768, 3, 2, 2100)])
def test_fft_prefill_all_transform_lengths(dtype, L, S, R, n_bins):
    # every transform length of the in-LDS FFT (2^8 .. 2^13) and the decimated form beyond it, ragged
    # scattered bins (both halves of the spectrum, so k and M - k both occur), with and without windows
    big = L > 8192
    cfg = small_cfg(L=L, dtype=dtype, n_bins=n_bins, n_sink=S, n_recent=R, steps=2,
                    n_layers=1 if big else 2, batch=1 if big else 2)
    bins = random_bins(cfg, 37)
    st = run_stream(cfg, bins, flags=B.IWDFT_FLAG_FFT_PREFILL, rec=(3, 50), tag=f"fftpf-{dtype}-L{L}")
    assert st["coef0"] < 2e-5


def test_fft_and_dense_prefill_give_the_same_state():
    cfg = small_cfg(L=4096, dtype="bf16", n_bins=500, n_sink=2, n_recent=3)
    bins = random_bins(cfg, 41)
    K, V = wl.prefill_tensors(cfg, DEV)
    a, b = make_cache(cfg, bins, flags=B.IWDFT_FLAG_FFT_PREFILL), make_cache(cfg, bins, flags=B.IWDFT_FLAG_DENSE_PREFILL)
    assert B.iwdft_prefill_kind(a.ctx) == "fft" and B.iwdft_prefill_kind(b.ctx) == "dense"
    c = make_cache(cfg, bins)                      # no flag: 500 kept bins -> FFT
    d = make_cache(small_cfg(L=4096, n_bins=100), [np.arange(100, dtype=np.int32)] * 2)   # few bins -> dense
    assert B.iwdft_prefill_kind(c.ctx) == "fft" and B.iwdft_prefill_kind(d.ctx) == "dense"
    c.close()
    d.close()
    a.prefill(K, V)
    b.prefill(K, V)
    for l in range(cfg.n_layers):
        (ka, va), (kb, vb) = a.export_coeffs(l), b.export_coeffs(l)
        assert rel_l2(c128(ka), c128(kb)) < 1e-5 and rel_l2(c128(va), c128(vb)) < 1e-5
    a.close()
    b.close()


@pytest.mark.parametrize("L,n_bins", [(1024, 400), (16384, 1100), (32768, 2100), (8192, 5000)])
def test_fft_prefill_of_tensors_that_are_not_16_byte_aligned(L, n_bins):
    """The FFT prefill fetches several channel pairs with one 8- or 16-byte load when K and V allow it; tensors that
    start 8 bytes off take one pair per workgroup instead.  Every pair's transform is the same arithmetic either way:
    the two states agree bit for bit."""
    cfg = small_cfg(L=L, n_bins=n_bins, n_layers=1, batch=1, n_kv_heads=2, dtype="bf16", mask="low")
    bins = wl.layer_bins(cfg)
    K, V = wl.prefill_tensors(cfg, DEV)
    pad = 4                                                    # bf16 elements = 8 bytes
    Ku = torch.empty(K.numel() + pad, dtype=K.dtype, device=DEV)[pad:].view_as(K)
    Vu = torch.empty(V.numel() + pad, dtype=V.dtype, device=DEV)[pad:].view_as(V)
    Ku.copy_(K)
    Vu.copy_(V)
    assert K.data_ptr() % 16 == 0 and Ku.data_ptr() % 16 == 8 and Vu.data_ptr() % 16 == 8
    a = make_cache(cfg, bins, flags=B.IWDFT_FLAG_FFT_PREFILL)
    b = make_cache(cfg, bins, flags=B.IWDFT_FLAG_FFT_PREFILL)
    a.prefill(K, V)
    b.prefill(Ku, Vu)
    (ka, va), (kb, vb) = a.export_coeffs(0), b.export_coeffs(0)
    assert torch.equal(ka, kb) and torch.equal(va, vb)
    a.close()
    b.close()


def test_misaligned_tensors_are_refused_before_any_launch():
    """Token, query, output and prefill tensors are accessed 16 bytes at a time: a tensor that starts elsewhere is an
    IWDFT_ERR_ARG (only the FFT prefill without windows takes K, V aligned to a channel pair, tested above)."""
    def off(t, pad=4):
        u = torch.empty(t.numel() + pad, dtype=t.dtype, device=DEV)[pad:].view_as(t)
        u.copy_(t)
        return u

    for S, R, flags in ((0, 0, B.IWDFT_FLAG_DENSE_PREFILL), (2, 3, B.IWDFT_FLAG_FFT_PREFILL)):
        cfg = small_cfg(L=1024, n_bins=400, n_layers=1, batch=1, n_kv_heads=2, dtype="bf16", n_sink=S, n_recent=R)
        bins = wl.layer_bins(cfg)
        K, V = wl.prefill_tensors(cfg, DEV)
        c = make_cache(cfg, bins, flags=flags)
        for args in ((off(K), V), (K, off(V))):
            with pytest.raises(B.IwdftError) as e:
                c.prefill(*args)
            assert e.value.code == B.IWDFT_ERR_ARG
        c.prefill(K, V)
        tk, tv, q = wl.decode_step(cfg, 0, DEV)
        out = torch.empty_like(q)
        for call in (lambda: c.append(off(tk), tv), lambda: c.append(tk, off(tv)), lambda: c.attend(off(q), out),
                     lambda: c.attend(q, off(out)), lambda: c.step(off(tk), tv, q, out), lambda: c.step(tk, tv, off(q), out),
                     lambda: c.step(tk, tv, q, off(out))):
            with pytest.raises(B.IwdftError) as e:
                call()
            assert e.value.code == B.IWDFT_ERR_ARG
        assert c.T == cfg.L                      # nothing was absorbed by the refused calls
        c.append(tk, tv)
        c.attend(q, out)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out.float()).all())
        c.close()
