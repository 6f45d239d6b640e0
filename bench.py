#!/usr/bin/env python3
"""Benchmark of the IWDFT hot path on one MI355X.

One *step* is one whole job over the named workload with all inputs already resident in HBM:
    iwdft_prefill(K, V)  ->  decode_steps x iwdft_append_attn(k_i, v_i, q_i)
where iwdft_append_attn is the append followed by the decode attention with the update fused into
the attention kernels and the coefficients written back every --write-every steps (--split runs the
two separate calls instead).  The reconstruction of Eq. reconstruct-idft happens inside the attention
kernels.  The default workload is the largest of the five baseline configurations (cfg5).

Prints ONE JSON line: whole-job appended tokens per second, the roofline of the kernel that takes most
of the job's GPU time (by HIP events between the kernels, on the stream they run on), per-call figures
of this and of the other baseline configurations ("per_config": the two calls the metric names --
iwdft_append tokens/s, compressed_decode_attn us/step -- each as a fraction of the HBM peak, the fused
step, both prefills), and the float64 CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import dataclasses
import gc
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16/bf16 MFMA, published
VALU_F32_PEAK_TFLOPS = 157.3   # fp32 vector, published (256 CUs x 128 lanes x 2 flop x 2.4 GHz)


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


class Sizes:
    """Algorithmic bytes / flops of one launch or call on a configuration."""

    def __init__(self, cfg, bins):
        self.nb_total = sum(len(b) for b in bins) * cfg.batch * cfg.n_kv_heads   # kept bins x slices
        self.coef_bytes = self.nb_total * cfg.head_dim * 8                       # one tensor, complex fp32
        self.append_bytes = 2 * self.coef_bytes * 2                              # K and V, read + write
        self.attn_bytes = 2 * self.coef_bytes                                    # K and V read once
        self.prefill_useful_flop = 2.0 * 2 * self.nb_total * cfg.L * cfg.head_dim * 2   # cos + sin rows, K and V
        self.mfma_split = 2 if cfg.dtype == "bf16" else 3                        # fp16 hi/lo basis (x fp32 input split)
        self.kv_in_bytes = 2 * cfg.n_slices * cfg.L * cfg.head_dim * (2 if cfg.dtype == "bf16" else 4)
        # phase B: one inverse and one forward complex M-point transform per pair of query heads
        pairs = (cfg.group + 1) // 2
        self.fft_flop = 2 * 5.0 * cfg.L * math.log2(cfg.L) * pairs * cfg.n_slices


def gbps(nbytes, ms):
    return nbytes / (ms * 1e-3) / 1e9


def frac(nbytes, ms):
    return gbps(nbytes, ms) / HBM_PEAK_GBS


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3, help="timed whole-job passes")
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="cfg5")
    ap.add_argument("--decode-steps", type=int, default=None, help="override the workload's decode steps")
    ap.add_argument("--split", action="store_true",
                    help="decode with the two separate calls (iwdft_append, compressed_decode_attn) instead of "
                         "the fused iwdft_append_attn")
    ap.add_argument("--write-every", type=int, default=16,
                    help="fused decode step: write the coefficients back every this many steps (1 = every step)")
    ap.add_argument("--group", type=int, default=None,
                    help="query heads per KV head (default: the workload's; 1 = the pure-bandwidth case)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="skip the per-call figures of the other configurations")
    ap.add_argument("--no-calls", action="store_true",
                    help="skip the per-call figures altogether (profiler runs: the timed job only)")
    ap.add_argument("--call-steps", type=int, default=16, help="decode steps per call kind in the per-call figures")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
                 "(every slice is independent, so the path would shard over layers, sequences or KV heads without any exchange)")

    import numpy as np
    import torch
    from paper_2507_20030_amd import binding as B
    from paper_2507_20030_amd import workload as wl

    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        a = torch.ones(1 << 28, dtype=torch.float32, device=dev)  # 1 GiB
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": a.numel() * 4, "copy_calibration_bytes_written": a.numel() * 4}))
        return

    stream = torch.cuda.current_stream()

    # HIP events are created at their first record, which costs far more than a record: all of them
    # are recorded once before they are used for timing.
    def mk(n):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
        for e in evs:
            e.record(stream)
        return evs

    def new_cache(cfg, bins, **kw):
        return B.Cache(cfg.n_layers, cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.torch_dtype,
                       cfg.L, bins, device=dev, n_sink=cfg.n_sink, n_recent=cfg.n_recent, **kw)

    def free(*objs):
        for o in objs:
            if hasattr(o, "close"):
                o.close()
        gc.collect()
        torch.cuda.empty_cache()

    traffic_all = {}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath) and os.path.getsize(tpath) > 0:
        traffic_all = json.load(open(tpath))

    # ------------------------------------------------------------------ per-call figures of one configuration
    def measure_calls(cfg, bins, K, V, pool, n, want_j16):
        """HIP-event timings of the calls the metric names, outside any timed job: both prefills, n x
        (iwdft_append, compressed_decode_attn) with the library's phase marks, n fused steps with write_every = 1,
        and (want_j16) 2 x 16 fused steps with write_every = 16."""
        sz = Sizes(cfg, bins)
        out = torch.empty_like(pool[0][2])
        res = {"n_slices": cfg.n_slices, "kept_bins": cfg.n_bins, "M": cfg.L, "group": cfg.group,
               "coefficient_GB_per_tensor": sz.coef_bytes / 1e9}
        c1 = new_cache(cfg, bins)
        res["attn_kind"] = B.iwdft_attn_kind(c1.ctx)
        res["attn_pipelined"] = B.iwdft_attn_pipelined(c1.ctx)   # phases A and B share launches: phase_A_ms = A + B
        pe = mk(2)
        c1.prefill(K, V, stream)
        pe[0].record(stream)
        c1.prefill(K, V, stream)
        pe[1].record(stream)
        torch.cuda.synchronize()
        pre_ms = pe[0].elapsed_time(pe[1])
        pre_kind = B.iwdft_prefill_kind(c1.ctx)
        res["iwdft_prefill"] = {"kind": pre_kind, "ms": pre_ms,
                                "algorithmic_GB": (sz.kv_in_bytes + 2 * sz.coef_bytes) / 1e9,
                                "frac_hbm_peak": frac(sz.kv_in_bytes + 2 * sz.coef_bytes, pre_ms),
                                "dense_equivalent_TFLOPps": sz.prefill_useful_flop / (pre_ms * 1e-3) / 1e12}
        # the two calls of the metric
        for i in range(2):
            tk, tv, q = pool[i % len(pool)]
            c1.append(tk, tv, stream)
            c1.attend(q, out, 0.0, stream)
        sp = [mk(3) for _ in range(n)]
        B.iwdft_phase_timing(c1.ctx, True)
        for i in range(n):
            tk, tv, q = pool[i % len(pool)]
            sp[i][0].record(stream)
            c1.append(tk, tv, stream)
            sp[i][1].record(stream)
            c1.attend(q, out, 0.0, stream)
            sp[i][2].record(stream)
        torch.cuda.synchronize()
        ph, calls = B.iwdft_phase_times(c1.ctx)
        B.iwdft_phase_timing(c1.ctx, False)
        ph = [m / max(calls, 1) for m in ph]
        app = np.array([e[0].elapsed_time(e[1]) for e in sp])
        att = np.array([e[1].elapsed_time(e[2]) for e in sp])
        res["iwdft_append"] = {"avg_ms": float(app.mean()), "min_ms": float(app.min()),
                               "tokens_per_s": cfg.batch / (float(app.mean()) * 1e-3),
                               "algorithmic_GB": sz.append_bytes / 1e9, "frac_hbm_peak": frac(sz.append_bytes, float(app.mean()))}
        res["compressed_decode_attn"] = {"avg_us": 1e3 * float(att.mean()), "min_us": 1e3 * float(att.min()),
                                         "algorithmic_GB": sz.attn_bytes / 1e9,
                                         "frac_hbm_peak": frac(sz.attn_bytes, float(att.mean())),
                                         "phase_A_ms": ph[0], "phase_B_ms": ph[1], "phase_C_ms": ph[2],
                                         "phase_A_frac_hbm_peak": frac(sz.coef_bytes, ph[0]),
                                         "phase_C_frac_hbm_peak": frac(sz.coef_bytes, ph[2]),
                                         "phase_B_fp32_TFLOPps": sz.fft_flop / (ph[1] * 1e-3) / 1e12 if ph[1] > 0 else None}
        if res["attn_pipelined"]:
            res["compressed_decode_attn"]["phase_A_frac_hbm_peak"] = None    # phase "A" holds A + B here
            # the same call with the three kernels one after the other (IWDFT_FLAG_SERIAL_PHASES)
            free(c1)
            c1 = new_cache(cfg, bins, flags=B.IWDFT_FLAG_SERIAL_PHASES)
            c1.prefill(K, V, stream)
            c1.attend(pool[0][2], out, 0.0, stream)
            se = mk(2)
            B.iwdft_phase_timing(c1.ctx, True)
            se[0].record(stream)
            for i in range(n):
                c1.attend(pool[i % len(pool)][2], out, 0.0, stream)
            se[1].record(stream)
            torch.cuda.synchronize()
            ph, calls = B.iwdft_phase_times(c1.ctx)
            B.iwdft_phase_timing(c1.ctx, False)
            ph = [m / max(calls, 1) for m in ph]
            res["compressed_decode_attn_serial_phases"] = {
                "avg_us": 1e3 * se[0].elapsed_time(se[1]) / n, "frac_hbm_peak": frac(sz.attn_bytes, se[0].elapsed_time(se[1]) / n),
                "phase_A_ms": ph[0], "phase_B_ms": ph[1], "phase_C_ms": ph[2],
                "phase_A_frac_hbm_peak": frac(sz.coef_bytes, ph[0]), "phase_C_frac_hbm_peak": frac(sz.coef_bytes, ph[2]),
                "phase_B_fp32_TFLOPps": sz.fft_flop / (ph[1] * 1e-3) / 1e12 if ph[1] > 0 else None}
        # fused step, coefficients written back at every step
        for i in range(2):
            c1.step(*pool[i % len(pool)], out, 0.0, stream)
        fe = [mk(2) for _ in range(n)]
        B.iwdft_phase_timing(c1.ctx, True)
        for i in range(n):
            fe[i][0].record(stream)
            c1.step(*pool[i % len(pool)], out, 0.0, stream)
            fe[i][1].record(stream)
        torch.cuda.synchronize()
        ph, calls = B.iwdft_phase_times(c1.ctx)
        B.iwdft_phase_timing(c1.ctx, False)
        ph = [m / max(calls, 1) for m in ph]
        f1 = np.array([e[0].elapsed_time(e[1]) for e in fe])
        res["iwdft_append_attn_write_every_1"] = {
            "avg_ms": float(f1.mean()), "min_ms": float(f1.min()), "algorithmic_GB": sz.append_bytes / 1e9,
            "frac_hbm_peak": frac(sz.append_bytes, float(f1.mean())),
            "phase_A_ms": ph[0], "phase_B_ms": ph[1], "phase_C_ms": ph[2],
            "phase_A_frac_hbm_peak": frac(2 * sz.coef_bytes, ph[0]), "phase_C_frac_hbm_peak": frac(2 * sz.coef_bytes, ph[2])}
        # materialising reconstruction of one layer
        Kt = torch.empty((cfg.batch, cfg.n_kv_heads, cfg.L, cfg.head_dim), dtype=cfg.torch_dtype, device=dev)
        Vt = torch.empty_like(Kt)
        re = mk(2)
        B.iwdft_reconstruct(c1.ctx, 0, 0, cfg.L, Kt, Vt, stream)
        re[0].record(stream)
        B.iwdft_reconstruct(c1.ctx, 0, 0, cfg.L, Kt, Vt, stream)
        re[1].record(stream)
        torch.cuda.synchronize()
        res["iwdft_reconstruct_one_layer_ms"] = re[0].elapsed_time(re[1])
        del Kt, Vt
        free(c1)
        # the dense (matrix-core) prefill on its own, whatever the library picks for the job
        if pre_kind == "dense":
            dense_ms = pre_ms
        else:
            dc = new_cache(cfg, bins, flags=B.IWDFT_FLAG_DENSE_PREFILL)
            dc.prefill(K, V, stream)
            de = mk(2)
            de[0].record(stream)
            dc.prefill(K, V, stream)
            de[1].record(stream)
            torch.cuda.synchronize()
            dense_ms = de[0].elapsed_time(de[1])
            free(dc)
        ex = sz.mfma_split * sz.prefill_useful_flop / (dense_ms * 1e-3) / 1e12
        res["iwdft_prefill_dense"] = {"ms": dense_ms, "useful_TFLOP": sz.prefill_useful_flop / 1e12,
                                      "useful_TFLOPps": sz.prefill_useful_flop / (dense_ms * 1e-3) / 1e12,
                                      "executed_TFLOPps": ex, "frac_mfma_f16_peak": ex / MFMA_F16_PEAK_TFLOPS,
                                      "useful_frac_mfma_f16_peak": ex / sz.mfma_split / MFMA_F16_PEAK_TFLOPS}
        if want_j16:
            cj = new_cache(cfg, bins, write_every=16)
            cj.prefill(K, V, stream)
            for i in range(16):
                cj.step(*pool[i % len(pool)], out, 0.0, stream)
            je = [mk(2) for _ in range(32)]
            for i in range(32):
                if i % 16 == 3:
                    B.iwdft_phase_timing(cj.ctx, True)
                je[i][0].record(stream)
                cj.step(*pool[i % len(pool)], out, 0.0, stream)
                je[i][1].record(stream)
                if i % 16 == 6:
                    B.iwdft_phase_timing(cj.ctx, False)
            torch.cuda.synchronize()
            ph, calls = B.iwdft_phase_times(cj.ctx)
            ph = [m / max(calls, 1) for m in ph]
            ms = np.array([e[0].elapsed_time(e[1]) for e in je])
            ro = np.array([ms[i] for i in range(32) if i % 16 != 15 and not 3 <= i % 16 <= 6])
            wb = np.array([ms[i] for i in range(32) if i % 16 == 15])
            avg = (float(ro.mean()) * 15 + float(wb.mean())) / 16
            avg_bytes = sz.attn_bytes + (sz.append_bytes - sz.attn_bytes) / 16
            res["iwdft_append_attn_write_every_16"] = {
                "avg_ms": avg, "read_only_step_ms": float(ro.mean()), "write_back_step_ms": float(wb.mean()),
                "algorithmic_GB_per_step": avg_bytes / 1e9, "frac_hbm_peak": frac(avg_bytes, avg),
                "tokens_per_s": cfg.batch / (avg * 1e-3),
                "phase_A_ms": ph[0], "phase_B_ms": ph[1], "phase_C_ms": ph[2],
                "phase_A_frac_hbm_peak": frac(sz.coef_bytes, ph[0]), "phase_C_frac_hbm_peak": frac(sz.coef_bytes, ph[2])}
            free(cj)
        return res

    # ------------------------------------------------------------------------------------- the timed job
    cfg = wl.CONFIGS[args.config]
    if args.group is not None:
        cfg = dataclasses.replace(cfg, group=args.group)
    dsteps = cfg.steps if args.decode_steps is None else args.decode_steps
    bins = wl.layer_bins(cfg)
    sz = Sizes(cfg, bins)
    log(f"{cfg.name}: generating inputs")
    K, V = wl.prefill_tensors(cfg, dev)
    fused = not args.split
    J = max(1, args.write_every) if fused else 1
    cache = new_cache(cfg, bins, write_every=J)
    n_pool = min(dsteps, 32)  # decode inputs are cycled from a resident pool
    pool = [wl.decode_step(cfg, i, dev) for i in range(n_pool)]
    out = torch.empty_like(pool[0][2])

    def decode(c, i, marks=None, split=False):
        tk, tv, q = pool[i % n_pool]
        if marks is not None:
            marks[0].record(stream)
        if split:
            c.append(tk, tv, stream)
            if marks is not None:
                marks[1].record(stream)
            c.attend(q, out, 0.0, stream)
        else:
            c.step(tk, tv, q, out, 0.0, stream)
        if marks is not None:
            marks[2].record(stream)

    # Event records between the kernels cost a few us each, so only a sample of the decode steps of
    # the timed region carries them.  In every group of 8 steps: steps 4 and 7 have events around the
    # call(s) (with write_every = 8 or 16 the write-back steps are among them); in the FIRST timed job
    # steps 2 and 5 of every group also carry the library's phase marks around its three kernels, which is
    # how the dominant kernel of the job is found (write_every > 1: these are read-only steps; the phases of
    # the rarer write-back steps are timed on the same context right after the timed region).
    sampled = lambda i: i % 8 in (4, 7) or dsteps < 8
    ev = [{i: mk(3) for i in range(dsteps) if sampled(i)} for _ in range(args.steps)]
    pre = [mk(2) for _ in range(args.steps)]
    writes_back = lambda i: (i + 1) % J == 0    # decode step i of a job (pending count restarts at the prefill)
    marked = lambda i: (i % 8 in (2, 5) or dsteps < 8) and (J == 1 or not writes_back(i))

    def run_job(s, marks):
        if s is not None:
            pre[s][0].record(stream)
        cache.prefill(K, V, stream)
        if s is not None:
            pre[s][1].record(stream)
        for i in range(dsteps):
            m = marks and marked(i)
            if m:
                B.iwdft_phase_timing(cache.ctx, True)
            decode(cache, i, ev[s].get(i) if s is not None else None, split=not fused)
            if m:
                B.iwdft_phase_timing(cache.ctx, False)

    log(f"{cfg.name}: {args.warmup} warm-up + {args.steps} timed jobs of prefill + {dsteps} decode steps")
    run_job(None, True)                 # untimed: creates the library's marks
    B.iwdft_phase_times(cache.ctx)
    for _ in range(max(args.warmup - 1, 0)):
        run_job(None, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        run_job(s, s == 0)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ph_ro, n_ro = B.iwdft_phase_times(cache.ctx)     # kernels A, B, C of the marked steps of the first timed job
    ph_ro = [m / max(n_ro, 1) for m in ph_ro]
    pre_kind = B.iwdft_prefill_kind(cache.ctx)
    attn_kind = B.iwdft_attn_kind(cache.ctx)
    pipelined = B.iwdft_attn_pipelined(cache.ctx)    # read-only steps: kernels A and B share launches (phase 0 = A + B)
    pre_ms = np.array([p[0].elapsed_time(p[1]) for p in pre])
    call_ms = lambda rows, pick, a=0, b=2: np.array([e[a].elapsed_time(e[b]) for row in rows
                                                    for i, e in row.items() if pick(i)] or [float("nan")])
    if fused:
        plain_ms = call_ms(ev, lambda i: not writes_back(i))   # steps that only read the coefficients
        wb_ms = call_ms(ev, writes_back)                       # steps that write them back
    else:
        app_ms, att_ms = call_ms(ev, lambda i: True, 0, 1), call_ms(ev, lambda i: True, 1, 2)

    # Phases of the write-back steps (write_every > 1), on the same context right after the timed region.
    ph_wb = ph_ro
    if fused and J > 1:
        cache.prefill(K, V, stream)
        for _ in range(3):
            for i in range(J):
                if i == J - 1:
                    B.iwdft_phase_timing(cache.ctx, True)
                decode(cache, i)
                if i == J - 1:
                    B.iwdft_phase_timing(cache.ctx, False)
        torch.cuda.synchronize()
        ph_wb, n_wb = B.iwdft_phase_times(cache.ctx)
        ph_wb = [m / max(n_wb, 1) for m in ph_wb]
    free(cache)
    del cache

    tokens = args.steps * dsteps * cfg.batch
    pre_avg = float(pre_ms.mean())
    job_ms = 1e3 * elapsed / args.steps

    # GPU time of one job by kernel: prefill + (read-only steps x phases) + (write-back steps x phases)
    if fused:
        n_wb_steps = sum(1 for i in range(dsteps) if writes_back(i)) if J > 1 else dsteps
        n_ro_steps = dsteps - n_wb_steps
        share = {
            "prefill": pre_avg,
            "A_read_only": n_ro_steps * ph_ro[0], "B_read_only": n_ro_steps * ph_ro[1], "C_read_only": n_ro_steps * ph_ro[2],
            "A_write_back": n_wb_steps * ph_wb[0], "B_write_back": n_wb_steps * ph_wb[1], "C_write_back": n_wb_steps * ph_wb[2],
        }
        if J == 1:
            for k_ in ("A_read_only", "B_read_only", "C_read_only"):
                share[k_] = 0.0
        b_ms = (share["B_read_only"] + share["B_write_back"]) / dsteps
        name_a = ("attn_ab_kernel (phases A + B pipelined over groups of slices, read-only steps)" if pipelined and J > 1
                  else "attn_qc_kernel<plain> (phase A, read-only steps)")
        share_kernel = {name_a: share["A_read_only"],
                        "attn_out_kernel<plain> (phase C, read-only steps)": share["C_read_only"],
                        "attn_fft_kernel (phase B, every step)": share["B_read_only"] + share["B_write_back"],
                        "attn_qc_kernel<update> (phase A, write-back steps)": share["A_write_back"],
                        "attn_out_kernel<update> (phase C, write-back steps)": share["C_write_back"],
                        "prefill": pre_avg}
    else:
        share_kernel = {"append_kernel (iwdft_append)": float(app_ms.mean()) * dsteps,
                        "attn_qc_kernel<plain> (phase A)": ph_ro[0] * dsteps,
                        "attn_fft_kernel (phase B)": ph_ro[1] * dsteps,
                        "attn_out_kernel<plain> (phase C)": ph_ro[2] * dsteps, "prefill": pre_avg}
        b_ms = ph_ro[1]
    dom = max(share_kernel, key=share_kernel.get)
    tkey = None
    if dom.startswith("attn_fft_kernel"):
        # bound by vector-ALU issue and LDS, not by HBM: textbook flops of its transforms against the fp32 vector peak
        roofline = {"kernel": dom, "bound": "alu", "achieved": sz.fft_flop / (b_ms * 1e-3) / 1e12,
                    "peak": VALU_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": sz.fft_flop / (b_ms * 1e-3) / 1e12 / VALU_F32_PEAK_TFLOPS,
                    "algorithmic": "2 x 5 M log2 M flops (one inverse + one forward M-point complex transform) per "
                                   "pair of query heads and slice; HBM traffic of this kernel is negligible"}
        tkey = f"attn_fft_{cfg.name}"
    else:
        if dom.startswith("append_kernel"):
            rb, rms, tkey = sz.append_bytes, float(app_ms.mean()), f"append_{cfg.name}"
        elif dom.startswith("prefill"):
            rb, rms, tkey = sz.kv_in_bytes + 2 * sz.coef_bytes, pre_avg, f"prefill_{pre_kind}_{cfg.name}"
        elif "phase A, write-back" in dom:
            rb, rms, tkey = 2 * sz.coef_bytes, ph_wb[0], f"step_qc_{cfg.name}"
        elif "phase C, write-back" in dom:
            rb, rms, tkey = 2 * sz.coef_bytes, ph_wb[2], f"step_out_{cfg.name}"
        elif dom.startswith("attn_ab_kernel"):
            rb, rms, tkey = sz.coef_bytes, ph_ro[0], f"attn_ab_{cfg.name}"
        elif "phase A" in dom:
            rb, rms, tkey = sz.coef_bytes, ph_ro[0], f"attn_qc_{cfg.name}"
        else:
            rb, rms, tkey = sz.coef_bytes, ph_ro[2], f"attn_out_{cfg.name}"
        roofline = {"kernel": dom, "bound": "hbm", "achieved": gbps(rb, rms), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": frac(rb, rms), "algorithmic_GB": rb / 1e9}
        if dom.startswith("attn_ab_kernel"):
            # these launches stream the K coefficients once (the algorithmic bytes) AND run every transform of the step
            roofline["also_runs_fp32_TFLOPps"] = sz.fft_flop / (rms * 1e-3) / 1e12
            roofline["note"] = ("one pass over the K coefficients plus all transforms of the step (vector ALU); the "
                                "three kernels one after the other: see per_config ... compressed_decode_attn_serial_phases")
    roofline["traffic"] = traffic_all.get(tkey)     # GB per launch from rocprofv3 counters, null if not profiled
    if roofline["traffic"] is None:
        roofline["traffic_note"] = f"no counter run recorded for {tkey}"
    roofline["job_gpu_time_by_kernel_ms"] = share_kernel

    if not fused:
        step_def = "prefill + decode_steps x (iwdft_append, compressed_decode_attn)"
    elif J == 1:
        step_def = "prefill + decode_steps x iwdft_append_attn (append fused into the decode attention)"
    else:
        step_def = (f"prefill + decode_steps x iwdft_append_attn (append fused into the decode attention, "
                    f"coefficients written back every {J} steps)")
    result = {
        "metric": "IWDFT tokens appended/sec + compressed decode-attn us/step (frac of HBM peak)",
        "value": tokens / elapsed,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": job_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{cfg.name}: {cfg.n_layers} layers x batch {cfg.batch} x {cfg.n_kv_heads} KV heads x "
                        f"head_dim {cfg.head_dim}, {cfg.dtype} K/V, fp32 complex coefficients, prefill {cfg.L} tokens, "
                        f"{cfg.n_bins} kept bins/layer ({cfg.mask}), {dsteps} x (append + decode attention), "
                        f"{cfg.group} query heads per KV head",
            "storage_dtype": cfg.dtype,
            "decode_steps": dsteps,
            "write_every": J,
            "step_definition": step_def,
            "prefill_kind": pre_kind,
            "attn_kind": attn_kind,
            "attn_pipelined": pipelined,
        },
        "job": {"prefill_ms": pre_avg},
        "roofline": roofline,
    }
    if fused:
        avg_step = (float(plain_ms.mean()) * (J - 1) + float(wb_ms.mean())) / J if J > 1 else float(wb_ms.mean())
        avg_bytes = sz.attn_bytes + (sz.append_bytes - sz.attn_bytes) / J      # reads every step, writes every J-th
        result["job"].update({
            "decode_step_avg_ms": avg_step, "algorithmic_GB_per_step": avg_bytes / 1e9,
            "decode_step_frac_hbm_peak": frac(avg_bytes, avg_step),
            "read_only_step_ms": float(plain_ms.mean()) if J > 1 else None, "write_back_step_ms": float(wb_ms.mean()),
            "read_only_phases_ms": ph_ro, "write_back_phases_ms": ph_wb,
            "read_only_phase_A_frac_hbm_peak": frac(sz.coef_bytes * (1 if J > 1 else 2), ph_ro[0]),
            "read_only_phase_C_frac_hbm_peak": frac(sz.coef_bytes * (1 if J > 1 else 2), ph_ro[2]),
        })
        result["decode_step_us"] = 1e3 * avg_step
    else:
        result["job"].update({"iwdft_append_ms": float(app_ms.mean()), "compressed_decode_attn_ms": float(att_ms.mean()),
                              "phases_ms": ph_ro})
        result["decode_step_us"] = 1e3 * float(app_ms.mean() + att_ms.mean())

    per_config = {}
    if not args.no_calls:
        log(f"{cfg.name}: per-call figures")
        per_config[cfg.name] = measure_calls(cfg, bins, K, V, pool, args.call_steps, want_j16=False)
        me = per_config[cfg.name]
        result["append_tokens_per_s"] = me["iwdft_append"]["tokens_per_s"]
        result["append_frac_hbm_peak"] = me["iwdft_append"]["frac_hbm_peak"]
        result["decode_attn_us_per_step"] = me["compressed_decode_attn"]["avg_us"]
        result["decode_attn_frac_hbm_peak"] = me["compressed_decode_attn"]["frac_hbm_peak"]

    if not args.no_cpu_baseline:
        log(f"{cfg.name}: CPU oracle baseline")
        result["cpu_baseline"] = cpu_baseline(cfg, bins, K, V, pool, np, torch)
    del K, V, pool, out
    free()

    if not (args.no_per_config or args.no_calls):
        for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5"):
            if name == cfg.name:
                continue
            c = wl.CONFIGS[name]
            log(f"{name}: per-call figures")
            b = wl.layer_bins(c)
            Kc, Vc = wl.prefill_tensors(c, dev)
            pc = [wl.decode_step(c, i, dev) for i in range(min(c.steps, 16))]
            per_config[name] = measure_calls(c, b, Kc, Vc, pc, args.call_steps, want_j16=True)
            del Kc, Vc, pc
            free()
    if per_config:
        result["per_config"] = {k_: per_config[k_] for k_ in sorted(per_config)}
    print(json.dumps(result), flush=True)


def cpu_baseline(cfg, bins, K, V, pool, np, torch):
    """The float64 oracle, as it stands, on a bounded sample: a few slices, a few decode steps,
    scaled to the whole workload (slices are independent).  Single thread."""
    from oracle import iwdft_oracle as orc
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)
    except Exception:  # pragma: no cover
        limiter = None
    from paper_2507_20030_amd import workload as wl
    slices = wl.sample_slices(cfg, 24)
    steps = min(8, len(pool))
    f64 = lambda t: t.detach().cpu().to(torch.float64).numpy()
    host = [(f64(K[l, b, h]), f64(V[l, b, h])) for (l, b, h) in slices]
    host_steps = [[(f64(tk[l, b, h]), f64(tv[l, b, h]), f64(q[l, b, h * cfg.group:(h + 1) * cfg.group]))
                   for (tk, tv, q) in pool[:steps]] for (l, b, h) in slices]
    t_pre = t_app = t_att = 0.0
    for (l, b, h), (k0, v0), hs in zip(slices, host, host_steps):
        t = time.perf_counter()
        SK, SV, T = orc.prefill(k0, bins[l]), orc.prefill(v0, bins[l]), cfg.L
        t_pre += time.perf_counter() - t
        for (tk, tv, q) in hs:
            t = time.perf_counter()
            SK, SV = orc.append(SK, tk, T, bins[l], cfg.L), orc.append(SV, tv, T, bins[l], cfg.L)
            T += 1
            t_app += time.perf_counter() - t
            t = time.perf_counter()
            orc.decode_attention(q, SK, SV, T, cfg.L, bins[l])
            t_att += time.perf_counter() - t
    if limiter is not None:
        limiter.restore_original_limits()
    n = len(slices)
    scale = cfg.n_slices / n
    pre_s = t_pre * scale
    step_s = (t_app + t_att) / steps * scale
    dsteps = cfg.steps
    job_s = pre_s + dsteps * step_s
    return {
        "value": dsteps * cfg.batch / job_s,
        "unit": "tokens/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"{n} of {cfg.n_slices} slices, prefill + {steps} decode steps each, numpy float64 single thread "
                  f"({t_pre + t_app + t_att:.1f} s of CPU work), scaled by n_slices/{n} and to {dsteps} decode steps",
        "prefill_s_scaled": pre_s,
        "append_s_per_step_scaled": t_app / steps * scale,
        "attn_s_per_step_scaled": t_att / steps * scale,
        "host_cores_available": len(os.sched_getaffinity(0)),
        # slices are independent, so the oracle would scale over the host cores at best linearly
        "value_all_cores_estimate": dsteps * cfg.batch / job_s * len(os.sched_getaffinity(0)),
    }


if __name__ == "__main__":
    main()
