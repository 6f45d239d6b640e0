#!/usr/bin/env python3
"""Benchmark of the IWDFT hot path on one MI355X.

One *step* is one whole job over the named workload with all inputs already resident in HBM:
    iwdft_prefill(K, V)  ->  decode_steps x ( iwdft_append(k_i, v_i) ; compressed_decode_attn(q_i) )
(the reconstruction of Eq. reconstruct-idft happens inside the attention kernels; the materialising
iwdft_reconstruct call is timed separately and reported under "kernels").

Prints ONE JSON line: whole-job appended tokens per second, the per-call timings measured with
HIP events inside the timed region, the roofline of the dominant kernel (the streaming update)
and the float64 CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
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
    dsteps = cfg.steps if args.decode_steps is None else args.decode_steps
    dev = "cuda:0"
    torch.cuda.set_device(0)
    bins = wl.layer_bins(cfg)
    K, V = wl.prefill_tensors(cfg, dev)
    cache = B.Cache(cfg.n_layers, cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.torch_dtype,
                    cfg.L, bins, device=dev)
    n_pool = min(dsteps, 32)  # decode inputs are cycled from a resident pool
    pool = [wl.decode_step(cfg, i, dev) for i in range(n_pool)]
    out = torch.empty_like(pool[0][2])
    stream = torch.cuda.current_stream()

    def job(events=None):
        cache.prefill(K, V, stream)
        for i in range(dsteps):
            tk, tv, q = pool[i % n_pool]
            if events is not None:
                e = events[i]
                e[0].record(stream)
                cache.append(tk, tv, stream)
                e[1].record(stream)
                cache.attend(q, out, 0.0, stream)
                e[2].record(stream)
            else:
                cache.append(tk, tv, stream)
                cache.attend(q, out, 0.0, stream)

    for _ in range(args.warmup):
        job()
    torch.cuda.synchronize()

    ev = [[[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(dsteps)]
          for _ in range(args.steps)]
    pre = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        pre[s][0].record(stream)
        cache.prefill(K, V, stream)
        pre[s][1].record(stream)
        for i in range(dsteps):
            tk, tv, q = pool[i % n_pool]
            e = ev[s][i]
            e[0].record(stream)
            cache.append(tk, tv, stream)
            e[1].record(stream)
            cache.attend(q, out, 0.0, stream)
            e[2].record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    app_ms = np.array([[e[0].elapsed_time(e[1]) for e in row] for row in ev])
    att_ms = np.array([[e[1].elapsed_time(e[2]) for e in row] for row in ev])
    pre_ms = np.array([p[0].elapsed_time(p[1]) for p in pre])

    # materialising reconstruction of one layer, timed on its own (not part of the job)
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    Kt = torch.empty((cfg.batch, cfg.n_kv_heads, cfg.L, cfg.head_dim), dtype=cfg.torch_dtype, device=dev)
    Vt = torch.empty_like(Kt)
    B.iwdft_reconstruct(cache.ctx, 0, 0, cfg.L, Kt, Vt, stream)
    r0.record(stream)
    B.iwdft_reconstruct(cache.ctx, 0, 0, cfg.L, Kt, Vt, stream)
    r1.record(stream)
    torch.cuda.synchronize()
    rec_ms = r0.elapsed_time(r1)

    nb_total = sum(len(b) for b in bins) * cfg.batch * cfg.n_kv_heads      # kept bins x slices
    coef_bytes = nb_total * cfg.head_dim * 8                               # one tensor, complex fp32
    append_bytes = 2 * coef_bytes * 2                                      # K and V, read + write
    attn_bytes = 2 * coef_bytes                                            # K and V read once
    prefill_useful_flop = 2.0 * 2 * nb_total * cfg.L * cfg.head_dim * 2     # cos+sin rows, K and V
    app_avg, att_avg, pre_avg = float(app_ms.mean()), float(att_ms.mean()), float(pre_ms.mean())
    tokens = args.steps * dsteps * cfg.batch

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(f"append_{cfg.name}")

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
            "step_definition": "prefill + decode_steps x (append, decode attention)",
        },
        "decode_attn_us_per_step": 1e3 * att_avg,
        "append_tokens_per_s": cfg.batch / (app_avg * 1e-3),
        "kernels": {
            "iwdft_append": {"avg_ms": app_avg, "min_ms": float(app_ms.min()), "algorithmic_GB": append_bytes / 1e9,
                             "GBps": append_bytes / (app_avg * 1e-3) / 1e9,
                             "frac_hbm_peak": append_bytes / (app_avg * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "compressed_decode_attn": {"avg_ms": att_avg, "min_ms": float(att_ms.min()),
                                       "algorithmic_GB": attn_bytes / 1e9,
                                       "GBps": attn_bytes / (att_avg * 1e-3) / 1e9,
                                       "frac_hbm_peak": attn_bytes / (att_avg * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "iwdft_prefill": {"avg_ms": pre_avg, "useful_TFLOP": prefill_useful_flop / 1e12,
                              "useful_TFLOPps": prefill_useful_flop / (pre_avg * 1e-3) / 1e12},
            "iwdft_reconstruct_one_layer": {"ms": rec_ms},
        },
        "roofline": {
            "kernel": "append_kernel (iwdft_append)",
            "bound": "hbm",
            "achieved": append_bytes / (app_avg * 1e-3) / 1e9,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": append_bytes / (app_avg * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "traffic": traffic,
        },
    }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, bins, K, V, pool, np, torch)
    cache.close()
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
    slices = wl.sample_slices(cfg, 4)
    steps = min(4, len(pool))
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
    }


if __name__ == "__main__":
    main()
