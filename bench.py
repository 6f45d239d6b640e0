#!/usr/bin/env python3
"""Benchmark of the IWDFT hot path on one MI355X.

One *step* is one whole job over the named workload with all inputs already resident in HBM:
    iwdft_prefill(K, V)  ->  decode_steps x iwdft_append_attn(k_i, v_i, q_i)
where iwdft_append_attn is the append followed by the decode attention with the update fused into
the attention kernels and the coefficients written back every --write-every steps (--split runs the
two separate calls instead).  The reconstruction of
Eq. reconstruct-idft happens inside the attention kernels; the materialising iwdft_reconstruct call
is timed separately and reported under "kernels", and so are the two separate calls of the metric
(append tokens/s, decode attention us/step).

Prints ONE JSON line: whole-job appended tokens per second, the per-call and per-kernel timings
measured with HIP events inside the timed region, the roofline of the dominant kernel and the
float64 CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3, help="timed whole-job passes")
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--decode-steps", type=int, default=None, help="override the workload's decode steps")
    ap.add_argument("--split", action="store_true",
                    help="decode with the two separate calls (iwdft_append, compressed_decode_attn) instead of "
                         "the fused iwdft_append_attn")
    ap.add_argument("--write-every", type=int, default=16,
                    help="fused decode step: write the coefficients back every this many steps (1 = every step)")
    ap.add_argument("--group", type=int, default=None,
                    help="query heads per KV head (default: the workload's; 1 = the pure-bandwidth case)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
                 "(every slice is independent; see DESIGN.md for how the path would shard)")

    import numpy as np
    import torch
    from paper_2507_20030_amd import binding as B
    from paper_2507_20030_amd import workload as wl

    if args.copy_calibration:
        a = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")  # 1 GiB
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": a.numel() * 4, "copy_calibration_bytes_written": a.numel() * 4}))
        return

    cfg = wl.CONFIGS[args.config]
    if args.group is not None:
        import dataclasses
        cfg = dataclasses.replace(cfg, group=args.group)
    dsteps = cfg.steps if args.decode_steps is None else args.decode_steps
    dev = "cuda:0"
    torch.cuda.set_device(0)
    bins = wl.layer_bins(cfg)
    K, V = wl.prefill_tensors(cfg, dev)
    fused = not args.split
    J = max(1, args.write_every) if fused else 1

    def new_cache(**kw):
        return B.Cache(cfg.n_layers, cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.torch_dtype,
                       cfg.L, bins, device=dev, **kw)
    cache = new_cache(write_every=J)
    n_pool = min(dsteps, 32)  # decode inputs are cycled from a resident pool
    pool = [wl.decode_step(cfg, i, dev) for i in range(n_pool)]
    out = torch.empty_like(pool[0][2])
    stream = torch.cuda.current_stream()

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
    # the timed region carries them.  In every group of 8 steps: step 2 has the library's phase marks
    # around its three attention kernels, steps 4 and 7 have events around the call(s); with write_every =
    # 8 or 16 the steps that write the coefficients back are among the latter.
    # HIP events are created at their first record, which costs far more than a record: all of them
    # are recorded once before the timed region.
    def mk(n):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
        for e in evs:
            e.record(stream)
        return evs
    sampled = lambda i: i % 8 in (4, 7) or dsteps < 8
    ev = [{i: mk(3) for i in range(dsteps) if sampled(i)} for _ in range(args.steps)]
    pre = [mk(2) for _ in range(args.steps)]
    marked = lambda i: i % 8 == 2 or dsteps < 8
    writes_back = lambda i: (i + 1) % J == 0    # decode step i of a job (pending count restarts at the prefill)

    def run_job(s):
        if s is not None:
            pre[s][0].record(stream)
        cache.prefill(K, V, stream)
        if s is not None:
            pre[s][1].record(stream)
        for i in range(dsteps):
            if marked(i):
                B.iwdft_phase_timing(cache.ctx, True)
            decode(cache, i, ev[s].get(i) if s is not None else None, split=not fused)
            if marked(i):
                B.iwdft_phase_timing(cache.ctx, False)

    for _ in range(args.steps):                 # untimed: creates the library's marks
        run_job(None)
    B.iwdft_phase_times(cache.ctx)
    for _ in range(args.warmup):
        run_job(None)
    B.iwdft_phase_times(cache.ctx)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        run_job(s)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    phase_ms, phase_calls = B.iwdft_phase_times(cache.ctx)
    phase_avg = [m / max(phase_calls, 1) for m in phase_ms]  # kernels A, B, C of the marked steps
    pre_kind = B.iwdft_prefill_kind(cache.ctx)

    pre_ms = np.array([p[0].elapsed_time(p[1]) for p in pre])
    call_ms = lambda rows, pick, a=0, b=2: np.array([e[a].elapsed_time(e[b]) for row in rows
                                                    for i, e in row.items() if pick(i)] or [float("nan")])
    if fused:
        plain_ms = call_ms(ev, lambda i: not writes_back(i))   # steps that only read the coefficients
        wb_ms = call_ms(ev, writes_back)                       # steps that write them back
    else:
        app_ms, att_ms = call_ms(ev, lambda i: True, 0, 1), call_ms(ev, lambda i: True, 1, 2)
    cache.close()
    del cache

    # After the timed region, on a second context that writes back at every step: the fused step with
    # write_every = 1 (phase marks on every step), and the two separate calls the metric names.
    c1 = new_cache()
    c1.prefill(K, V, stream)
    n_extra = min(dsteps, 64)
    if fused:
        for i in range(4):
            decode(c1, i)
        B.iwdft_phase_timing(c1.ctx, True)
        e1 = [mk(3) for _ in range(n_extra)]
        for i in range(n_extra):
            decode(c1, i, e1[i])
        torch.cuda.synchronize()
        f1_phase, f1_calls = B.iwdft_phase_times(c1.ctx)
        B.iwdft_phase_timing(c1.ctx, False)
        f1_ms = np.array([e[0].elapsed_time(e[2]) for e in e1])
        f1_phase = [m / max(f1_calls, 1) for m in f1_phase]
        sp = [mk(3) for _ in range(n_extra)]
        for i in range(n_extra):
            decode(c1, i, sp[i], split=True)
        torch.cuda.synchronize()
        app_ms = np.array([e[0].elapsed_time(e[1]) for e in sp])
        att_ms = np.array([e[1].elapsed_time(e[2]) for e in sp])

    # materialising reconstruction of one layer, timed on its own (not part of the job)
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    Kt = torch.empty((cfg.batch, cfg.n_kv_heads, cfg.L, cfg.head_dim), dtype=cfg.torch_dtype, device=dev)
    Vt = torch.empty_like(Kt)
    B.iwdft_reconstruct(c1.ctx, 0, 0, cfg.L, Kt, Vt, stream)
    r0.record(stream)
    B.iwdft_reconstruct(c1.ctx, 0, 0, cfg.L, Kt, Vt, stream)
    r1.record(stream)
    torch.cuda.synchronize()
    rec_ms = r0.elapsed_time(r1)
    c1.close()
    del c1, Kt, Vt

    # the dense (matrix-core) prefill on its own, whatever the job used
    if pre_kind == "dense":
        dense_ms = float(pre_ms.mean())
    else:
        dcache = new_cache(flags=B.IWDFT_FLAG_DENSE_PREFILL)
        dcache.prefill(K, V, stream)
        de = mk(2 * 3)
        for i in range(3):
            de[2 * i].record(stream)
            dcache.prefill(K, V, stream)
            de[2 * i + 1].record(stream)
        torch.cuda.synchronize()
        dense_ms = float(np.mean([de[2 * i].elapsed_time(de[2 * i + 1]) for i in range(3)]))
        dcache.close()
        del dcache

    # what the matrix cores sustain on the dense prefill's instruction with nothing else running (zero and
    # random operands: the part is power-limited, and the second figure is the ceiling real data can approach)
    probe = torch.empty(1 << 18, dtype=torch.float32, device=dev)
    mfma_sustained = {}
    for label, rnd in (("zero_operands", False), ("random_operands", True)):
        B.iwdft_mfma_probe(probe, 200, rnd, stream)
        pe = mk(2)
        pe[0].record(stream)
        flops = B.iwdft_mfma_probe(probe, 2000, rnd, stream)
        pe[1].record(stream)
        torch.cuda.synchronize()
        mfma_sustained[label + "_TFLOPps"] = flops / (pe[0].elapsed_time(pe[1]) * 1e-3) / 1e12
    del probe

    nb_total = sum(len(b) for b in bins) * cfg.batch * cfg.n_kv_heads      # kept bins x slices
    coef_bytes = nb_total * cfg.head_dim * 8                               # one tensor, complex fp32
    append_bytes = 2 * coef_bytes * 2                                      # K and V, read + write
    attn_bytes = 2 * coef_bytes                                            # K and V read once
    prefill_useful_flop = 2.0 * 2 * nb_total * cfg.L * cfg.head_dim * 2     # cos+sin rows, K and V
    mfma_split = 2 if cfg.dtype == "bf16" else 3                           # fp16 hi/lo basis (x fp32 input split)
    kv_in_bytes = 2 * cfg.n_slices * cfg.L * cfg.head_dim * (2 if cfg.dtype == "bf16" else 4)
    app_avg, att_avg, pre_avg = float(app_ms.mean()), float(att_ms.mean()), float(pre_ms.mean())
    tokens = args.steps * dsteps * cfg.batch
    gbps = lambda nbytes, ms: nbytes / (ms * 1e-3) / 1e9
    frac = lambda nbytes, ms: gbps(nbytes, ms) / HBM_PEAK_GBS

    traffic_all = {}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        traffic_all = json.load(open(tpath))

    # Dominant kernel of the timed job, from the library's phase marks.
    if not fused:
        roof_kernel, roof_bytes, roof_ms = "append_kernel (iwdft_append)", append_bytes, app_avg
        traffic = traffic_all.get(f"append_{cfg.name}")
    elif J == 1:    # every step writes back; phase A is a read-modify-write of every K coefficient
        roof_kernel = "attn_qc_kernel<update> (iwdft_append_attn, phase A: K update + scores)"
        roof_bytes, roof_ms = 2 * coef_bytes, phase_avg[0]
        traffic = traffic_all.get(f"step_qc_{cfg.name}")
    elif phase_avg[2] >= phase_avg[0]:   # J - 1 of J steps only read: phase C streams every V coefficient once
        roof_kernel = "attn_out_kernel<plain> (iwdft_append_attn, phase C: output from the V coefficients)"
        roof_bytes, roof_ms = coef_bytes, phase_avg[2]
        traffic = traffic_all.get(f"attn_out_{cfg.name}")
    else:
        roof_kernel = "attn_qc_kernel<plain> (iwdft_append_attn, phase A: scores from the K coefficients)"
        roof_bytes, roof_ms = coef_bytes, phase_avg[0]
        traffic = traffic_all.get(f"attn_qc_{cfg.name}")

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
        "ms_per_step": 1e3 * elapsed / args.steps,
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
            "decode_steps": dsteps,
            "write_every": J,
            "step_definition": step_def,
        },
        "decode_attn_us_per_step": 1e3 * att_avg,
        "append_tokens_per_s": cfg.batch / (app_avg * 1e-3),
        "kernels": {
            "iwdft_append": {"avg_ms": app_avg, "median_ms": float(np.median(app_ms)), "min_ms": float(app_ms.min()),
                             "algorithmic_GB": append_bytes / 1e9,
                             "GBps": gbps(append_bytes, app_avg), "frac_hbm_peak": frac(append_bytes, app_avg)},
            "compressed_decode_attn": {"avg_ms": att_avg, "median_ms": float(np.median(att_ms)),
                                       "min_ms": float(att_ms.min()),
                                       "algorithmic_GB": attn_bytes / 1e9,
                                       "GBps": gbps(attn_bytes, att_avg), "frac_hbm_peak": frac(attn_bytes, att_avg)},
            "iwdft_prefill": {"kind": pre_kind, "avg_ms": pre_avg,
                              "algorithmic_GB": (kv_in_bytes + 2 * coef_bytes) / 1e9,
                              "GBps": gbps(kv_in_bytes + 2 * coef_bytes, pre_avg),
                              "dense_equivalent_TFLOPps": prefill_useful_flop / (pre_avg * 1e-3) / 1e12,
                              "fft_TFLOP": 5.0 * cfg.L * math.log2(cfg.L) * cfg.n_slices * cfg.head_dim / 1e12},
            "iwdft_prefill_dense": {"avg_ms": dense_ms, "useful_TFLOP": prefill_useful_flop / 1e12,
                                    "useful_TFLOPps": prefill_useful_flop / (dense_ms * 1e-3) / 1e12,
                                    "executed_TFLOPps": mfma_split * prefill_useful_flop / (dense_ms * 1e-3) / 1e12,
                                    "frac_mfma_f16_peak": mfma_split * prefill_useful_flop / (dense_ms * 1e-3) / 1e12
                                                          / MFMA_F16_PEAK_TFLOPS,
                                    "mfma_probe": mfma_sustained},
            "iwdft_reconstruct_one_layer": {"ms": rec_ms},
        },
        "roofline": {
            "kernel": roof_kernel,
            "bound": "hbm",
            "achieved": gbps(roof_bytes, roof_ms),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": frac(roof_bytes, roof_ms),
            "traffic": traffic,
        },
    }
    k = result["kernels"]
    if fused:
        after = "separate context after the timed region"
        k["iwdft_append"]["measured"] = k["compressed_decode_attn"]["measured"] = after
        # write_every = 1: every coefficient read once and written once per step = the bytes of one append
        k["iwdft_append_attn_write_every_1"] = {
            "measured": after if J > 1 else "timed region", "avg_ms": float(f1_ms.mean()), "min_ms": float(f1_ms.min()),
            "algorithmic_GB": append_bytes / 1e9, "frac_hbm_peak": frac(append_bytes, float(f1_ms.mean())),
            "phase_A_K_update_scores_ms": f1_phase[0], "phase_B_softmax_transforms_ms": f1_phase[1],
            "phase_C_V_update_output_ms": f1_phase[2],
            "phase_A_frac_hbm_peak": frac(2 * coef_bytes, f1_phase[0]),
            "phase_C_frac_hbm_peak": frac(2 * coef_bytes, f1_phase[2]),
        }
        avg_step = (float(plain_ms.mean()) * (J - 1) + float(wb_ms.mean())) / J if J > 1 else float(wb_ms.mean())
        avg_bytes = attn_bytes + (append_bytes - attn_bytes) / J      # reads every step, writes every J-th
        k["iwdft_append_attn"] = {
            "write_every": J, "avg_ms": avg_step, "algorithmic_GB_per_step": avg_bytes / 1e9,
            "frac_hbm_peak": frac(avg_bytes, avg_step),
            "read_only_step_ms": float(plain_ms.mean()) if J > 1 else None,
            "write_back_step_ms": float(wb_ms.mean()),
            "marked_steps": "read-only" if J > 1 else "write-back",
            "phase_A_ms": phase_avg[0], "phase_B_ms": phase_avg[1], "phase_C_ms": phase_avg[2],
            "phase_A_frac_hbm_peak": frac(coef_bytes * (1 if J > 1 else 2), phase_avg[0]),
            "phase_C_frac_hbm_peak": frac(coef_bytes * (1 if J > 1 else 2), phase_avg[2]),
        }
        result["decode_step_us"] = 1e3 * avg_step
    else:
        k["compressed_decode_attn"].update(
            {"phase_A_ms": phase_avg[0], "phase_B_ms": phase_avg[1], "phase_C_ms": phase_avg[2]})
        result["decode_step_us"] = 1e3 * (app_avg + att_avg)

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, bins, K, V, pool, np, torch)
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
    slices = wl.sample_slices(cfg, 32)
    steps = min(12, len(pool))
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
        "sample": f"{n} of {cfg.n_slices} slices, prefill + {steps} decode steps each, numpy float64 single thread, "
                  f"scaled by n_slices/{n} and to {dsteps} decode steps",
        "prefill_s_scaled": pre_s,
        "append_s_per_step_scaled": t_app / steps * scale,
        "attn_s_per_step_scaled": t_att / steps * scale,
        "host_cores_available": len(os.sched_getaffinity(0)),
        # slices are independent, so the oracle would scale over the host cores at best linearly
        "value_all_cores_estimate": dsteps * cfg.batch / job_s * len(os.sched_getaffinity(0)),
    }


if __name__ == "__main__":
    main()
