"""Full-size parity of the five baseline configurations on sampled slices (the float64 oracle
cannot hold whole 10^2-GB caches): the GPU runs the complete workload shape in the launch
configuration the benchmark times; the oracle follows 8 slices (first, last, seeded picks)."""
import numpy as np
import pytest
import torch

from paper_2507_20030_amd import binding as B
from paper_2507_20030_amd import workload as wl
from test_gpu_parity import (DEV, SliceOracle, check_attn, check_coeffs, check_masks, check_reconstruct,
                             make_cache, run_stream)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("prefill", ["fft", "dense"])
def test_cfg3_batch8_mixed_masks(prefill):
    cfg = wl.CONFIGS["cfg3"]
    bins = wl.layer_bins(cfg)
    assert any(b[-1] >= cfg.n_bins for b in bins) and any(b[-1] == cfg.n_bins - 1 for b in bins)
    flags = B.IWDFT_FLAG_FFT_PREFILL if prefill == "fft" else B.IWDFT_FLAG_DENSE_PREFILL
    run_stream(cfg, bins, flags=flags, steps=3, tag=f"cfg3-{prefill}")


def test_cfg5_wide_outlier_channels():
    cfg = wl.CONFIGS["cfg5"]
    run_stream(cfg, wl.layer_bins(cfg), steps=2, slices=wl.sample_slices(cfg, 6), tag="cfg5")


def test_cfg5_full_length_fused_deferred_write_back():
    """All 128 decode steps of cfg5 in the launch configuration the benchmark times (fused step, coefficients
    written back every 16th step: 8 write-backs), attention checked at every step on 4 slices."""
    cfg = wl.CONFIGS["cfg5"]
    run_stream(cfg, wl.layer_bins(cfg), slices=wl.sample_slices(cfg, 4), fused=True, write_every=16,
               tag="cfg5-fused-J16-full")


def test_cfg3_fused_deferred_write_back():
    """cfg3 in the benchmark's launch configuration: 18 fused steps, one write-back of 16 tokens at M = 32768
    (multi-block transforms with 16 pending tokens), two tokens left deferred for the final flush."""
    cfg = wl.CONFIGS["cfg3"]
    run_stream(cfg, wl.layer_bins(cfg), steps=18, fused=True, write_every=16, tag="cfg3-fused-J16")


def test_cfg2_full_length_fused_deferred_write_back():
    """All 256 decode steps of cfg2 (16 write-backs), attention checked at every step on 2 slices."""
    cfg = wl.CONFIGS["cfg2"]
    run_stream(cfg, wl.layer_bins(cfg), slices=wl.sample_slices(cfg, 2), fused=True, write_every=16,
               tag="cfg2-fused-J16-full")


def _max_rel_l2(a, b):
    if a.is_complex():
        a, b = torch.view_as_real(a), torch.view_as_real(b)
    a, b = a.float(), b.float()
    return float((a - b).norm() / b.norm().clamp_min(1e-30))


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4", "cfg5"])
def test_every_slice_is_tied_to_the_sampled_ones(name):
    """GPU against GPU at full size, over ALL slices (the oracle follows only a sample): (1) the benchmark's
    configuration -- FFT prefill, fused steps, write-back every 16th -- run twice leaves the same bytes in the state
    buffer and returns the same outputs; (2) the two-call path on top of the dense prefill agrees with it to
    rounding on every slice: prefill state, outputs of all 17 steps, final state after the flush."""
    cfg = wl.CONFIGS[name]
    bins = wl.layer_bins(cfg)
    K, V = wl.prefill_tensors(cfg, DEV)
    steps = [wl.decode_step(cfg, i, DEV) for i in range(17)]   # write-back at step 16, one token left deferred

    def run(flags, fused, J):
        c = make_cache(cfg, bins, flags=flags, write_every=J)
        c.prefill(K, V)
        pre = [tuple(t.clone() for t in c.export_coeffs(l)) for l in (0, cfg.n_layers - 1)]
        outs = []
        for tk, tv, q in steps:
            if fused:
                outs.append(c.step(tk, tv, q).clone())
            else:
                c.append(tk, tv)
                outs.append(c.attend(q).clone())
        c.flush()
        torch.cuda.synchronize()
        return c, pre, outs

    a, pre_a, outs_a = run(B.IWDFT_FLAG_FFT_PREFILL, True, 16)
    state_a = a.state.clone()
    a.close()
    del a
    b, pre_b, outs_b = run(B.IWDFT_FLAG_FFT_PREFILL, True, 16)
    assert torch.equal(state_a, b.state), f"{name}: two identical runs left different state bytes"
    assert all(torch.equal(x, y) for x, y in zip(outs_a, outs_b)), f"{name}: two identical runs gave different outputs"
    del state_a, outs_b, pre_b
    c, pre_c, outs_c = run(B.IWDFT_FLAG_DENSE_PREFILL, False, 0)
    worst_pre = max(_max_rel_l2(x, y) for pa, pc in zip(pre_a, pre_c) for x, y in zip(pa, pc))
    assert worst_pre < 2e-5, f"{name}: FFT vs dense prefill coefficients differ by {worst_pre:.2e}"
    worst_out = max(_max_rel_l2(x, y) for x, y in zip(outs_a, outs_c))
    assert worst_out < 1e-2, f"{name}: fused/deferred vs two-call outputs differ by {worst_out:.2e}"
    per_slice = 0.0                               # no single slice may hide behind the norm of the others
    for x, y in zip(outs_a, outs_c):
        d = (x.float() - y.float()).flatten(2).norm(dim=2) / y.float().flatten(2).norm(dim=2).clamp_min(1e-30)
        per_slice = max(per_slice, float(d.max()))
    assert per_slice < 2e-2, f"{name}: worst (layer, sequence) output difference {per_slice:.2e}"
    worst_state = 0.0
    for l in range(cfg.n_layers):
        (kb, vb), (kc, vc) = b.export_coeffs(l), c.export_coeffs(l)
        for x, y in ((kb, kc), (vb, vc)):
            d = (x - y).flatten(2).norm(dim=2) / y.flatten(2).norm(dim=2).clamp_min(1e-30)   # per (sequence, KV head)
            worst_state = max(worst_state, float(d.max()))
    assert worst_state < 2e-5, f"{name}: final coefficients of some slice differ by {worst_state:.2e}"
    print(f"\n[{name} all slices] prefill {worst_pre:.2e} outputs {worst_out:.2e} (worst slice {per_slice:.2e}) "
          f"state {worst_state:.2e}", flush=True)
    b.close()
    c.close()


@pytest.mark.parametrize("fused", [False, True])
def test_cfg4_long_context_drift(fused):
    """1024 streaming appends with decode attention at every step -- as two calls, and as the fused step with the
    coefficients written back every 16th step (the configuration the benchmark times); coefficients are compared
    with the oracle's recursion AND with its from-scratch closed form at steps 1, 16, 256, 1024 (in the deferred
    mode after iwdft_flush: at step 1 the token is still pending)."""
    from oracle import iwdft_oracle as orc
    cfg = wl.CONFIGS["cfg4"]
    bins = wl.layer_bins(cfg)
    slices = wl.sample_slices(cfg, 4)
    K, V = wl.prefill_tensors(cfg, DEV)
    cache = make_cache(cfg, bins, write_every=16 if fused else 0)
    check_masks(cache, bins)
    cache.prefill(K, V)
    ora = SliceOracle(cfg, bins, None, K, V, slices)
    f64 = lambda t: t.detach().cpu().to(torch.float64).numpy()
    hist = {s: [f64(K[s]), []] for s in slices}          # prefill K of each slice + appended rows
    del K, V
    tag = "cfg4-fused-J16" if fused else "cfg4"
    stats = {"coef0": check_coeffs(cache, ora, f"{tag} prefill")}
    out = None
    G = cfg.group
    for i in range(cfg.steps):
        tk, tv, q = wl.decode_step(cfg, i, DEV)
        if fused:
            out = cache.step(tk, tv, q, out)
        else:
            cache.append(tk, tv)
            out = cache.attend(q, out)
        ora.append(tk, tv)
        for s in slices:
            hist[s][1].append(f64(tk[s]))
        step = i + 1
        if step in (1, 16, 256, 1024):
            ref = ora.attend(q)                            # the output this very step returned
            w = max(np.linalg.norm(f64(out[l, b, h * G:(h + 1) * G]) - r) / np.linalg.norm(r) for (l, b, h), r in ref.items())
            assert w < 2e-2, f"{tag} step {step}: attention rel-L2 {w:.3e}"
            stats[f"attn{step}"] = float(w)
            if fused:
                cache.flush()
            stats[f"coef{step}"] = check_coeffs(cache, ora, f"{tag} step {step}")
            worst = 0.0
            SK_layers = {}
            for s in slices:
                l, b, h = s
                if l not in SK_layers:
                    SK_layers[l] = cache.export_coeffs(l)[0]
                xs = np.vstack([hist[s][0], np.stack(hist[s][1])])
                ref = orc.closed_form(xs, cfg.L, bins[l])
                got = SK_layers[l][b, h].cpu().numpy().astype(np.complex128)
                worst = max(worst, float(np.linalg.norm(got - ref) / np.linalg.norm(ref)))
            assert worst < 1e-4, f"{tag} step {step}: drift vs from-scratch recompute {worst:.3e}"
            stats[f"scratch{step}"] = worst
    assert cache.T == cfg.L + cfg.steps
    stats["rec"] = check_reconstruct(cfg, cache, ora, cfg.L - 64, 64, f"{tag} end")
    print(f"\n[{tag}] " + " ".join(f"{k}={v:.2e}" for k, v in stats.items()), flush=True)
    cache.close()


@pytest.mark.parametrize("group,n_bins,shape,dtype,windows", [
    (4, 1100, (16, 8, 8), "bf16", False),   # 4 heads per pass, 3-4 kept bins per thread
    (4, 2100, (16, 8, 8), "bf16", True),    # 4 heads per pass, 5-8 kept bins per thread (256-register transform), windows
    (8, 1100, (8, 8, 8), "bf16", False),    # 8 heads per pass, 3-4 bins per thread
    (8, 2100, (8, 8, 8), "f32", False),     # 8 heads per pass, 5-8 bins per thread, fp32 tokens
    (3, 1100, (5, 2, 103), "bf16", False),  # 1030 slices, 3 query heads: block counts per group that are not multiples
                                            # of 8 (tails of the per-XCD role sequence), a last head pair with one head
])
def test_pipelined_and_serial_phases_agree_bit_for_bit(group, n_bins, shape, dtype, windows):
    """Long contexts with many slices run kernels A and B as a pipeline over groups of slices (the transforms of one
    group share launches with the K stream of the next); IWDFT_FLAG_SERIAL_PHASES runs the three kernels one after
    the other.  Same arithmetic per block, so decode attention, fused read-only steps with pending tokens, the
    write-back step and the final state must agree bit for bit.  One shape per kernel instantiation; the oracle
    parity of the pipelined path is covered by the full-size cfg3 / cfg5 tests above."""
    cfg = wl.Config("pipe", shape[0], shape[1], shape[2], group, 128, 16384, n_bins, 20, dtype, "mixed", seed=11,
                    n_sink=4 if windows else 0, n_recent=12 if windows else 0)
    bins = wl.layer_bins(cfg)
    K, V = wl.prefill_tensors(cfg, DEV)
    steps = [wl.decode_step(cfg, i, DEV) for i in range(18)]

    def run(flags):
        c = make_cache(cfg, bins, flags=flags | B.IWDFT_FLAG_FFT_PREFILL, write_every=16)
        c.prefill(K, V)
        outs = []
        for i, (tk, tv, q) in enumerate(steps):
            if i < 2:                       # the two-call form
                c.append(tk, tv)
                outs.append(c.attend(q).clone())
            else:                           # fused steps: 15 read-only ones with 1..15 pending tokens, one write-back
                outs.append(c.step(tk, tv, q).clone())
        c.flush()
        torch.cuda.synchronize()
        return c, outs

    a, outs_a = run(0)
    b, outs_b = run(B.IWDFT_FLAG_SERIAL_PHASES)
    assert B.iwdft_attn_pipelined(a.ctx) and not B.iwdft_attn_pipelined(b.ctx)
    for i, (x, y) in enumerate(zip(outs_a, outs_b)):
        assert torch.isfinite(x.float()).all(), f"step {i}: non-finite output"
        assert torch.equal(x, y), f"step {i}: pipelined and serial outputs differ (max {float((x.float() - y.float()).abs().max()):.3e})"
    assert torch.equal(a.state, b.state), "final state differs"
    a.close()
    b.close()


def test_cfg3_shape_with_8192_kept_bins_full_size():
    """A quarter of the bins of a 32768-token context (the paper's largest ratio) at cfg3's full shape: bin-strided FFT
    prefill and decode attention, two calls and the fused step, on sampled slices against the oracle."""
    cfg = wl.CONFIGS["cfg3b"]
    bins = wl.layer_bins(cfg)
    c = make_cache(cfg, bins)
    assert B.iwdft_prefill_kind(c.ctx) == "fft" and B.iwdft_attn_kind(c.ctx) == "fft" and not B.iwdft_attn_pipelined(c.ctx)
    c.close()
    run_stream(cfg, bins, steps=2, slices=wl.sample_slices(cfg, 6), tag="cfg3b")
    run_stream(cfg, bins, steps=2, slices=wl.sample_slices(cfg, 4), fused=True, tag="cfg3b-fused")


def test_cfg3_shape_with_the_papers_windows_cut_out_of_the_context_full_size():
    """M = 32768 - 60 = 4 x 8177 at cfg3's full shape: dense prefill, decode attention through four decimated chirp-z
    blocks per pair of query heads, on sampled slices against the oracle."""
    cfg = wl.CONFIGS["cfg3x"]
    assert cfg.n_prefill == 32768
    bins = wl.layer_bins(cfg)
    c = make_cache(cfg, bins)
    assert B.iwdft_prefill_kind(c.ctx) == "dense" and B.iwdft_attn_kind(c.ctx) == "chirp"
    c.close()
    run_stream(cfg, bins, steps=2, slices=wl.sample_slices(cfg, 6), tag="cfg3x")
    run_stream(cfg, bins, steps=2, slices=wl.sample_slices(cfg, 4), fused=True, tag="cfg3x-fused")
