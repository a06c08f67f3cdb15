#!/usr/bin/env python3
"""Benchmark of the tiered decode-attention hot path on one MI355X.

One "step" is one pass of the whole path over a batch of synthetic input: for every layer, append the new
token's K/V rows and run tiered attention with score accumulation; every Delta steps, classify and migrate
(T1 offload + prefetch on the side streams).  Inputs are resident in HBM before the timed region starts.
Prints one JSON line (metric: KV GB/s of the whole job, with the HBM-roofline figure of the attention kernel,
the T1 prefetch overhead against the all-in-HBM twin, and the CPU oracle timed on a bounded sample).
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E bandwidth
# HBM bytes per launch of the attention kernel from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE), each
# scaled by the same counter's reading for the library's plain row-copy kernel of known size (the context preload:
# 134 217 728 bytes read and written per launch; FETCH_SIZE reads 1 per 2031 bytes, WRITE_SIZE 1 per KiB).
# See profiles/attn_tiered_14b_hbm_traffic.txt.
MEASURED_TRAFFIC = {"14b": {"fetch_bytes": 122_190_000, "write_bytes": 5_800_000}}
LINK_PEAK_GBPS = 64.0       # PCIe Gen5 x16, one direction


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def call_bytes(cfg, n_full, n_t2, out_es=4):
    """Algorithmic bytes of one layer call: every live row once (K and V), q and out, score read-modify-write.
    n_full, n_t2 are position counts summed over the batch."""
    es = 4 if cfg.kv_dtype == "f32" else 2
    D, Hkv, Hq, B = cfg.head_dim, cfg.n_kv_heads, cfg.n_q_heads, cfg.batch
    t2_row = (D + 4) if cfg.t2_format == "int8_row" else (D // 2 + (D // 32) * 2)
    kv = Hkv * (n_full * 2 * D * es + n_t2 * 2 * t2_row)
    return kv + B * Hq * D * (es + out_es) + (n_full + n_t2) * 4 * 2


BOUNCE_MIB = 0   # --bounce-mib: size of each bounce ring of the T1 transport (0: the library's default)
SCORER = "attention"   # --scorer


def run_job(cfg, policy, mode, steps, warmup, profile_steps, label, rule=0):
    import torch
    import paper_2605_09490_amd as tkv
    from tkv_synth import Workload

    wl = Workload(cfg, device="cuda")
    sizes = {"bounce_bytes": BOUNCE_MIB << 20, "scorer": SCORER}
    if mode == "stream":
        # the two frames are sized for T1's share of the final length plus 30 % (a migrate takes the slots of the rows
        # that enter T1 before it releases those of the rows that leave); the HBM pool still takes the whole context,
        # which is appended before the first tiering
        n_end = cfg.context + cfg.decode_steps
        sizes["staging_rows"] = min(cfg.max_tokens, int(1.3 * policy[1] * n_end) // 1_000_000 + 64)
    gpu = tkv.TieredKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.max_tokens,
                       kv_dtype=cfg.kv_dtype, t2_format=cfg.t2_format, n_prompt=cfg.n_prompt, k_sink=cfg.k_sink,
                       k_window=cfg.k_window, prefetch_mode=mode, **sizes)
    for l in range(cfg.n_layers):
        k, v = wl.context_kv(l)
        gpu.append(l, k, v)
    del k, v
    total = warmup + steps + profile_steps
    k_all, v_all, q_all = wl.decode_inputs(0, total)
    out_all = torch.empty((cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
    # one attention pass so the first ranking is not all ties, then the initial tiering + cold fill
    gpu.decode_step(k_all[0], v_all[0], q_all[0], out_all)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    gpu.classify(policy, count_rule=rule)
    gpu.migrate()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gpu.wait_prefetch()
    t2 = time.perf_counter()
    st0 = gpu.get_stats()
    res = {"label": label, "first_migrate_ms": (t1 - t0) * 1e3, "cold_fill_ms": (t2 - t0) * 1e3,
           "cold_fill_bytes": st0["h2d_bytes"]}
    delta = cfg.reclassify_every

    def loop(first, n, count_bytes):
        nbytes = 0
        for s in range(first, first + n):
            if count_bytes:
                tc = gpu_counts[0]
                nbytes += cfg.n_layers * call_bytes(cfg, tc[0] + tc[1] + cfg.batch, tc[2])
                tc[0] += cfg.batch
            gpu.decode_step(k_all[s], v_all[s], q_all[s], out_all)
            if (s + 1) % delta == 0:
                gpu.classify(policy, count_rule=rule)
                gpu.migrate()
                if count_bytes:
                    gpu_counts[0] = list(gpu.get_stats()["tier_count"])
        return nbytes

    gpu_counts = [None]
    loop(1, warmup - 1, False)
    torch.cuda.synchronize()
    gpu.wait_prefetch()
    gpu_counts[0] = list(gpu.get_stats()["tier_count"])
    st1 = gpu.get_stats()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    nbytes = loop(warmup, steps, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gpu.wait_prefetch()
    st2 = gpu.get_stats()
    res.update({"wall_s": t1 - t0, "bytes": nbytes, "ms_per_step": (t1 - t0) * 1e3 / steps,
                "tier_count": st2["tier_count"], "events": st2["n_migrate"] - st1["n_migrate"],
                "h2d_bytes": st2["h2d_bytes"] - st1["h2d_bytes"], "h2d_ms": st2["h2d_ms"] - st1["h2d_ms"],
                "d2h_bytes": st2["d2h_bytes"] - st1["d2h_bytes"], "d2h_ms": st2["d2h_ms"] - st1["d2h_ms"],
                "classify_ms": st2["classify_ms"] - st1["classify_ms"], "migrate_ms": st2["migrate_ms"] - st1["migrate_ms"],
                "attend_waits": st2["attend_waits"] - st1["attend_waits"],
                "lazy_old_reads": st2["lazy_old_reads"] - st1["lazy_old_reads"]})
    if profile_steps:
        gpu.set_profile(True)
        b0 = loop(warmup + steps, profile_steps, True)
        torch.cuda.synchronize()
        st3 = gpu.get_stats()
        gpu.set_profile(False)
        launches = st3["attn_kernel_launches"] - st2["attn_kernel_launches"]
        kms = st3["attn_kernel_ms"] - st2["attn_kernel_ms"]
        res.update({"kernel_launches": launches, "kernel_avg_us": kms * 1e3 / max(launches, 1),
                    "kernel_bytes_per_launch": b0 / max(launches, 1)})
        import numpy as np
        n = gpu.layer_length(0)
        sc = np.sort(gpu.get_scores()[:, :n].astype(np.float64), axis=1)[:, ::-1]
        res["top20_share"] = float((sc[:, : n // 5].sum(1) / sc.sum(1)).mean())
        res["bottom50_share"] = float((sc[:, n // 2:].sum(1) / sc.sum(1)).mean())
        # Eq. 1 at full size: every attention call adds one unit of probability per query head, so with the scale
        # 1/(L*Hq) each sequence's scores (evicted positions keep theirs) sum to the number of decode steps so far
        steps_done = 1 + (warmup - 1) + steps + profile_steps
        if SCORER == "attention":
            res["score_mass_rel_err"] = float(np.abs(sc.sum(1) / steps_done - 1.0).max())
    res["device_bytes"] = st2["device_bytes"]
    res["pinned_bytes"] = st2["pinned_bytes"]
    res["gpu"] = gpu
    res["wl"] = wl
    return res


def cpu_baseline(cfg, res, budget_s=20.0):
    """The CPU oracle as it stands, timed on a bounded sample of the same workload: the first two layers, all
    sequences, the GPU run's final tier assignment, a few attention-and-score calls."""
    import numpy as np
    import torch
    from oracle import tkv_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    gpu, wl = res["gpu"], res["wl"]
    layers = [0, 1][: cfg.n_layers]
    n = gpu.layer_length(0)
    tiers = gpu.get_tiers()[:, :n]
    orc = O.OracleCache(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, n,
                        kv_dtype=cfg.kv_dtype, t2_format=cfg.t2_format, k_sink=cfg.k_sink, k_window=cfg.k_window,
                        layers=layers)
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    # rows as the GPU holds them are not needed for timing: same shapes and distributions, drawn again
    for l in layers:
        k, v = wl.context_kv(l)
        pad = n - k.shape[1]
        kk, vv = f64(k), f64(v)
        if pad > 0:
            kk = np.concatenate([kk, kk[:, :pad]], axis=1)
            vv = np.concatenate([vv, vv[:, :pad]], axis=1)
        orc.append(l, kk, vv)
    orc.tier[:, :n] = tiers            # placement only; T2 rows keep full-precision values for the timing run
    q = f64(wl.step_q(0, 0))
    n_full = int(((tiers == 0) | (tiers == 1)).sum())
    n_t2 = int((tiers == 2).sum())
    per_call = call_bytes(cfg, n_full, n_t2)
    calls, t0 = 0, time.perf_counter()
    while True:
        for l in layers:
            orc.attend_and_score(l, q)
            calls += 1
        if time.perf_counter() - t0 > budget_s or calls >= 64:
            break
    dt = time.perf_counter() - t0
    return {"value": per_call * calls / dt / 1e9, "unit": "GB/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{calls} attend_and_score calls on layers {layers} of the {cfg.name} workload "
                      f"(batch {cfg.batch}, {n} tokens, final GPU tier assignment), {dt:.1f} s, numpy fp64",
            "s_per_layer_call": dt / calls, "s_per_step_extrapolated": dt / calls * cfg.n_layers}


def link_probe():
    import torch
    n = 256 << 20
    d = torch.empty(n, dtype=torch.uint8, device="cuda")
    d2 = torch.empty_like(d)
    h = torch.empty(n, dtype=torch.uint8, pin_memory=True)
    out = {}
    for name, fn in (("d2d_copy", lambda: d2.copy_(d)), ("h2d_pinned", lambda: d.copy_(h, non_blocking=True)),
                     ("d2h_pinned", lambda: h.copy_(d, non_blocking=True))):
        fn(); torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(4):
            fn()
        torch.cuda.synchronize()
        gb = 4 * n / (time.perf_counter() - t0) / 1e9
        out[name + "_GBps"] = round(gb * (2 if name == "d2d_copy" else 1), 1)   # d2d: read + write
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="14b")
    ap.add_argument("--mode", default="lazy", choices=["lazy", "wait", "stream"],
                    help="T1 transport: lazy / wait keep all of T1 staged in HBM (differential prefetch); stream keeps two "
                         "layer-sized frames and moves T1 over the link at every step")
    ap.add_argument("--profile-steps", type=int, default=-1,
                    help="extra decode steps, after the timed ones, in which every attention launch is timed by HIP events "
                         "(default: one re-tiering period, so the window holds the same mix of steps right after an event "
                         "and steady ones as the timed region)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-twin", action="store_true")
    ap.add_argument("--kv-dtype", default="", choices=["", "bf16", "f16", "f32"], help="K, V and query type (default: the workload's own)")
    ap.add_argument("--delta", type=int, default=0, help="re-tier every DELTA steps (default: the workload's own)")
    ap.add_argument("--k-window", type=int, default=-1, help="protected recent window (default: the workload's own)")
    ap.add_argument("--bounce-mib", type=int, default=0, help="size of each T1 bounce ring in MiB (default: the library's own)")
    ap.add_argument("--scorer", default="attention", choices=["attention", "vatp"],
                    help="cumulative attention (Eq. 1, the paper's method) or the value-aware variant of its scoring ablation")
    ap.add_argument("--count-rule", default="total", choices=["total", "alg1"],
                    help="band sizes as fixed fractions of all candidates, or Algorithm 1's floors (evicts again at every event)")
    args = ap.parse_args()
    global BOUNCE_MIB, SCORER
    BOUNCE_MIB = args.bounce_mib
    SCORER = args.scorer
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no sharding, no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from tkv_synth import CONFIGS
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    probe = link_probe()     # before the caches exist: the largest workload leaves little pinned memory to spare
    base = CONFIGS[args.workload]
    warmup = max(args.warmup, 1)
    if args.profile_steps < 0:
        args.profile_steps = args.delta or base.reclassify_every
    cfg = dataclasses.replace(base, decode_steps=warmup + args.steps + args.profile_steps,
                              reclassify_every=args.delta or base.reclassify_every,
                              kv_dtype=args.kv_dtype or base.kv_dtype,
                              k_window=base.k_window if args.k_window < 0 else args.k_window)
    rule = 1 if args.count_rule == "alg1" else 0
    pol = cfg.policy_ppm
    twin_pol = (pol[0] + pol[1], 0, pol[2], pol[3])
    log(f"[bench] workload {cfg.name}: L={cfg.n_layers} B={cfg.batch} Hq/Hkv={cfg.n_q_heads}/{cfg.n_kv_heads} D={cfg.head_dim} "
        f"{cfg.kv_dtype} ctx={cfg.context} policy={pol} t2={cfg.t2_format} mode={args.mode}")
    other_mode = "wait" if args.mode == "lazy" else "lazy"
    stream = args.mode == "stream"
    # Job order: the all-HBM twin (same tier counts, T1 share kept in T0) and the other prefetch mode run first, then
    # the job `value` is taken from, then all three once more.  The overhead is a difference of two wall times and the
    # clock of a GPU that has just left idle drifts, so kinds are compared on the faster of their two runs; `value`
    # itself is always the one designated run (the first of the measured mode).
    kinds = [args.mode] if args.no_twin else (["twin", args.mode] if stream else
                                              ["twin", other_mode, args.mode, "twin", other_mode, args.mode])
    runs = {k: [] for k in kinds}
    runs_all_in = {k: [] for k in kinds}     # timed loop + the initial tiering with its cold fill
    main_res, cpu = None, None
    mem = {}
    for kind in kinds:
        is_main = kind == args.mode and main_res is None
        r = run_job(cfg, twin_pol if kind == "twin" else pol, ("lazy" if stream else args.mode) if kind == "twin" else kind,
                    args.steps, warmup, args.profile_steps if is_main else 0, kind, rule)
        runs[kind].append(r["wall_s"])
        runs_all_in[kind].append(r["wall_s"] + r["cold_fill_ms"] * 1e-3)
        log(f"[bench] {kind}: {r['ms_per_step']:.3f} ms/step" + (f", cold fill {r['cold_fill_ms']:.1f} ms" if is_main else ""))
        mem[kind] = r.pop("device_bytes")
        if is_main:
            main_res = r
            if not args.no_cpu:
                cpu = cpu_baseline(cfg, main_res)
                log(f"[bench] oracle: {cpu['s_per_layer_call']*1e3:.1f} ms per layer call on {cpu['cores']} threads")
        r.pop("gpu").close(); r.pop("wl")
    extra = {}
    if not args.no_twin:
        best = {k: min(v) for k, v in runs.items()}
        best_all = {k: min(v) for k, v in runs_all_in.items()}
        extra = {
            "prefetch_overhead_all_in_pct": round(100.0 * (best_all[args.mode] - best_all["twin"]) / best_all["twin"], 2),
            "prefetch_overhead_pct": round(100.0 * (best[args.mode] - best["twin"]) / best["twin"], 2),
            **({} if stream else {f"prefetch_overhead_pct_{other_mode}": round(100.0 * (best[other_mode] - best["twin"]) / best["twin"], 2)}),
            "ms_per_step_runs": {k: [round(w * 1e3 / args.steps, 4) for w in v] for k, v in runs.items()},
        }
    value = main_res["bytes"] / main_res["wall_s"] / 1e9
    kernel_GBps = main_res["kernel_bytes_per_launch"] / (main_res["kernel_avg_us"] * 1e-6) / 1e9 if main_res.get("kernel_avg_us") else None
    h2d_GBps = main_res["h2d_bytes"] / (main_res["h2d_ms"] * 1e-3) / 1e9 if main_res["h2d_ms"] > 0 else None
    d2h_GBps = main_res["d2h_bytes"] / (main_res["d2h_ms"] * 1e-3) / 1e9 if main_res["d2h_ms"] > 0 else None
    line = {
        "metric": "tiered decode-attn KV GB/s & % of HBM peak; T1 prefetch overhead % of step",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": warmup,
        "ms_per_step": round(main_res["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.kv_dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}-shaped: {cfg.n_layers} layers, {cfg.n_q_heads}/{cfg.n_kv_heads} heads, d {cfg.head_dim}, "
                               f"{cfg.kv_dtype} KV, batch {cfg.batch}, {cfg.context}-token context, tiers ppm {list(pol)}, "
                               f"T2 {cfg.t2_format}, re-tier every {cfg.reclassify_every} steps, prefetch {args.mode}"
                               + (f", k_window {cfg.k_window}" if args.k_window >= 0 else "")
                               + (", Algorithm-1 count rule" if rule else "")
                               + (", value-aware scorer" if SCORER != "attention" else "")},
        "hbm_peak_frac": round(value / HBM_PEAK_GBPS, 4),
        "decode_steps_per_s": round(1e3 / main_res["ms_per_step"], 1),
        "roofline": {"bound": "hbm", "achieved": round(kernel_GBps, 1) if kernel_GBps else None, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(kernel_GBps / HBM_PEAK_GBPS, 4) if kernel_GBps else None,
                     "traffic": (sum(MEASURED_TRAFFIC[cfg.name].values()) if cfg.name in MEASURED_TRAFFIC else None),
                     "kernel": "k_attn_tiered", "avg_us": round(main_res.get("kernel_avg_us", 0), 2),
                     "algorithmic_bytes_per_launch": int(main_res.get("kernel_bytes_per_launch", 0)),
                     "launches_timed": main_res.get("kernel_launches")},
        "cpu_baseline": cpu,
        "t1": {"events_in_timed_region": main_res["events"], "h2d_bytes": main_res["h2d_bytes"], "d2h_bytes": main_res["d2h_bytes"],
               "h2d_GBps": round(h2d_GBps, 1) if h2d_GBps else None, "d2h_GBps": round(d2h_GBps, 1) if d2h_GBps else None,
               "h2d_link_frac": round(h2d_GBps / LINK_PEAK_GBPS, 3) if h2d_GBps else None,
               "cold_fill_ms": round(main_res["cold_fill_ms"], 1), "cold_fill_bytes": main_res["cold_fill_bytes"],
               "classify_ms_per_event": round(main_res["classify_ms"] / max(main_res["events"], 1), 3),
               "migrate_ms_per_event": round(main_res["migrate_ms"] / max(main_res["events"], 1), 3),
               "attend_waits": main_res["attend_waits"], "lazy_old_reads": main_res["lazy_old_reads"],
               "device_bytes": mem.get(args.mode), "device_bytes_all_in_hbm_twin": mem.get("twin"),
               "pinned_bytes": main_res["pinned_bytes"], **extra},
        "tier_count": main_res["tier_count"],
        "score_top20_share": round(main_res.get("top20_share", 0), 3), "score_bottom50_share": round(main_res.get("bottom50_share", 0), 3),
        "score_mass_rel_err": main_res.get("score_mass_rel_err"),
        "probe": probe, "host_cores": os.cpu_count(),
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
