"""GPU parity at the benchmark's shapes: the per-layer launch configuration depends on (batch, heads, head_dim,
context, tier mix), not on the layer count, so these cases keep the full per-layer shape of the benchmark configurations and
cut the number of layers (and, for the production-batch config, the number of sequences) to what the CPU oracle
finishes in seconds.  Every output element and every score is compared, not a sample."""
import dataclasses

import numpy as np
import pytest
import torch

from tkv_synth import CONFIGS, small_config

pytestmark = pytest.mark.gpu


def _run_shape(cfg, mode, steps_before=1, steps_after=2):
    from gpu_common import Pair, assert_out_close, assert_scores_close, to_f64
    print(f"[case] {cfg.name}-shaped L={cfg.n_layers} B={cfg.batch} Hq={cfg.n_q_heads} Hkv={cfg.n_kv_heads} D={cfg.head_dim} "
          f"ctx={cfg.context} t2={cfg.t2_format} mode={mode}", flush=True)
    p = Pair(cfg, prefetch_mode=mode)
    L = cfg.n_layers
    k_all, v_all, q_all = p.wl.decode_inputs(0, steps_before + steps_after)
    calls, worst = 0, 0.0

    def step(s):
        nonlocal calls, worst
        out = p.gpu.decode_step(k_all[s], v_all[s], q_all[s])
        for l in range(L):
            p.orc.append(l, to_f64(k_all[s, l]), to_f64(v_all[s, l]))
            ref = p.orc.attend_and_score(l, to_f64(q_all[s, l]))
            worst = max(worst, assert_out_close(to_f64(out[l]), ref, cfg.kv_dtype, f"step {s} layer {l}"))
            calls += 1

    for s in range(steps_before):
        step(s)
    n = p.gpu.layer_length(0)
    p.gpu.classify(cfg.policy_ppm)
    plan = p.gpu.get_pending_tiers()[:, :n]
    want = p.orc.classify(cfg.policy_ppm, score_f32=p.gpu.get_scores())[:, :n]
    assert np.array_equal(plan, want)
    p.gpu.migrate()
    p.orc.migrate()
    for s in range(steps_before, steps_before + steps_after):
        step(s)
    ss = 1.0 / (cfg.n_layers * cfg.n_q_heads)
    n = p.gpu.layer_length(0)
    assert_scores_close(p.gpu.get_scores(), p.orc.score, n, calls * cfg.n_q_heads * ss)
    st = p.gpu.get_stats()
    print(f"[case] worst output error {worst:.2e} of the head max-norm; tiers {st['tier_count']}", flush=True)
    assert st["tier_count"][1] > 0 and st["tier_count"][2] > 0
    p.close()


def test_14b_shape():
    _run_shape(dataclasses.replace(CONFIGS["14b"], n_layers=2, decode_steps=3), "lazy")


def test_7b_shape():
    _run_shape(dataclasses.replace(CONFIGS["7b"], n_layers=2, decode_steps=3), "wait")


def test_32b_shape():
    _run_shape(dataclasses.replace(CONFIGS["32b"], n_layers=1, decode_steps=3), "lazy")


def test_prod_shape_all_64_sequences_one_workgroup_per_pair():
    """The production-batch launch as the bench runs it: 64 sequences x 4 kv heads = 256 pairs, so every pair gets ONE
    workgroup (S = 1) whose eight waves share all F tiles and all int4 Q tiles of a 16384-token list.  The GPU runs
    the whole batch; four of its sequences (first, last, two in between) are checked against an oracle that holds
    just those four (sequences are independent): outputs, scores after a forced four-tier plan, and a chunk of three
    query tokens through the matrix-core launch at the same shape."""
    import paper_2605_09490_amd as tkv
    from gpu_common import assert_out_close, assert_scores_close, to_f64
    from oracle import tkv_oracle as O
    from tkv_synth import Workload
    cfg = dataclasses.replace(CONFIGS["prod"], n_layers=1, decode_steps=5)
    pick = [0, 21, 42, 63]
    print(f"[case] prod-shaped, all {cfg.batch} sequences, ctx={cfg.context}, checking sequences {pick}", flush=True)
    wl = Workload(cfg, device="cuda")
    gpu = tkv.TieredKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.max_tokens,
                       kv_dtype=cfg.kv_dtype, t2_format=cfg.t2_format, k_sink=cfg.k_sink, k_window=cfg.k_window,
                       prefetch_mode="lazy")
    orc = O.OracleCache(cfg.n_layers, len(pick), cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.max_tokens,
                        kv_dtype=cfg.kv_dtype, t2_format=cfg.t2_format, k_sink=cfg.k_sink, k_window=cfg.k_window)
    k, v = wl.context_kv(0)
    gpu.append(0, k, v)
    orc.append(0, to_f64(k[pick]), to_f64(v[pick]))
    del k, v
    n = cfg.context
    rng = np.random.default_rng(3)
    tiers = rng.choice(4, size=(cfg.batch, n), p=(0.4, 0.37, 0.2, 0.03)).astype(np.uint8)
    tiers[:, :4] = 0
    tiers[:, n - 128:] = 0
    gpu.set_tiers(tiers); gpu.migrate()
    orc.set_tiers(tiers[pick]); orc.migrate()
    calls = 0
    for step in range(2):
        ks, vs = wl.step_kv(step, 0)
        q = wl.step_q(step, 0)
        gpu.append(0, ks, vs)
        orc.append(0, to_f64(ks[pick]), to_f64(vs[pick]))
        out = gpu.attend_and_score(0, q)
        ref = orc.attend_and_score(0, to_f64(q[pick]))
        assert_out_close(to_f64(out[pick]), ref, cfg.kv_dtype, f"step {step}")
        calls += 1
    T = 3
    ks, vs = zip(*[wl.step_kv(2 + j, 0) for j in range(T)])
    kc, vc = torch.cat(ks, dim=1), torch.cat(vs, dim=1)
    gpu.append(0, kc, vc)
    orc.append(0, to_f64(kc[pick]), to_f64(vc[pick]))
    q = torch.stack([wl.step_q(2 + j, 0) for j in range(T)], dim=1).contiguous()
    out = gpu.attend_and_score_chunk(0, q)
    ref = orc.attend_and_score_chunk(0, to_f64(q[pick]))
    for j in range(T):
        assert_out_close(to_f64(out[pick, j]), ref[:, j], cfg.kv_dtype, f"chunk query {j}")
    calls += T
    nn = gpu.layer_length(0)
    ss = 1.0 / (cfg.n_layers * cfg.n_q_heads)
    assert_scores_close(gpu.get_scores()[pick], orc.score, nn, calls * cfg.n_q_heads * ss)
    gpu.close()


def test_prod_shape_subset_of_sequences():
    # 16384-token context, int4-g32 T2; 4 of the 64 sequences (sequences are independent units of work)
    _run_shape(dataclasses.replace(CONFIGS["prod"], n_layers=1, batch=4, decode_steps=2), "lazy", steps_after=1)


def test_decode_step_equals_per_layer_calls():
    """tkv_decode_step is tkv_append + tkv_attend_and_score per layer: same bits."""
    from gpu_common import Pair
    cfg = small_config(n_layers=3, batch=2, n_q_heads=10, n_kv_heads=2, head_dim=128, kv_dtype="bf16", context=500,
                       decode_steps=4)
    a, b = Pair(cfg), Pair(cfg)
    k_all, v_all, q_all = a.wl.decode_inputs(0, 4)
    for s in range(4):
        oa = a.gpu.decode_step(k_all[s], v_all[s], q_all[s])
        for l in range(cfg.n_layers):
            b.gpu.append(l, k_all[s, l], v_all[s, l])
            ob = b.gpu.attend_and_score(l, q_all[s, l])
            assert torch.equal(oa[l], ob)
        if s == 1:
            for p in (a, b):
                p.gpu.classify(cfg.policy_ppm)
                p.gpu.migrate()
    assert np.array_equal(a.gpu.get_scores().view(np.uint32), b.gpu.get_scores().view(np.uint32))
    assert np.array_equal(a.gpu.get_tiers(), b.gpu.get_tiers())
    a.close(); b.close()


def test_many_tiles_per_wave():
    """256 (sequence, kv head) pairs leave two workgroups per pair: every wave walks 8+ tiles of list F and the Q waves
    several of list Q, so the steady-state part of the fetch pipeline (not only its first and last tile) is compared
    element by element."""
    cfg = small_config(name="deep", n_layers=1, batch=32, n_q_heads=8, n_kv_heads=8, head_dim=64, kv_dtype="bf16",
                       context=4200, decode_steps=3, policy_ppm=(300_000, 400_000, 270_000, 30_000), k_window=64)
    _run_shape(cfg, "lazy", steps_before=1, steps_after=1)


def test_batch_above_the_kernel_argument_limit():
    """More than 64 sequences: list lengths and the wave split are read from device counters instead of kernel
    arguments."""
    cfg = small_config(name="wide", n_layers=1, batch=70, n_q_heads=4, n_kv_heads=2, head_dim=64, kv_dtype="f32",
                       context=200, decode_steps=3, policy_ppm=(400_000, 300_000, 250_000, 50_000), k_window=16)
    _run_shape(cfg, "wait", steps_before=1, steps_after=1)


def test_one_sequence_many_splits():
    """A single long sequence with 8 kv heads of 8 query heads each is split 32 ways per kv head: the per-split softmax
    statistics (8 x 32 x 2 x 8 floats) exceed the finishing kernel's LDS copy and are read from memory instead."""
    cfg = small_config(name="solo", n_layers=1, batch=1, n_q_heads=64, n_kv_heads=8, head_dim=64, kv_dtype="bf16",
                       context=9000, decode_steps=3, policy_ppm=(300_000, 400_000, 270_000, 30_000), k_window=64)
    _run_shape(cfg, "wait", steps_before=1, steps_after=1)


def test_14b_full_depth_score_mass():
    """The benchmark's own configuration at full depth (48 layers, batch 8, 4096-token context, lazy prefetch): after
    s decode steps with one re-tiering in between, every sequence's cumulative scores sum to s (Eq. 1 with the scale
    1/(L*Hq): each call adds one unit of probability per query head; evicted positions keep what they had), and an
    evicted position's score does not change any more."""
    import paper_2605_09490_amd as tkv
    from tkv_synth import Workload
    cfg = dataclasses.replace(CONFIGS["14b"], decode_steps=4)
    print(f"[case] 14b full depth L={cfg.n_layers} B={cfg.batch} ctx={cfg.context}", flush=True)
    wl = Workload(cfg, device="cuda")
    gpu = tkv.TieredKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.max_tokens,
                       kv_dtype=cfg.kv_dtype, t2_format=cfg.t2_format, k_sink=cfg.k_sink, k_window=cfg.k_window,
                       prefetch_mode="lazy")
    for l in range(cfg.n_layers):
        k, v = wl.context_kv(l)
        gpu.append(l, k, v)
    del k, v
    k_all, v_all, q_all = wl.decode_inputs(0, 4)
    gpu.decode_step(k_all[0], v_all[0], q_all[0])
    gpu.classify(cfg.policy_ppm)
    gpu.migrate()
    n = gpu.layer_length(0)
    tiers = gpu.get_tiers()[:, :n]
    frozen = gpu.get_scores()[:, :n][tiers == 3].copy()
    assert frozen.size > 0
    for s in range(1, 4):
        gpu.decode_step(k_all[s], v_all[s], q_all[s])
    sc = gpu.get_scores().astype(np.float64)
    n2 = gpu.layer_length(0)
    assert np.abs(sc[:, :n2].sum(1) / 4.0 - 1.0).max() < 1e-4
    assert np.array_equal(gpu.get_scores()[:, :n][tiers == 3], frozen)
    st = gpu.get_stats()
    assert st["tier_count"][1] > 0 and st["tier_count"][2] > 0 and st["tier_count"][3] > 0
    gpu.close()


def test_14b_shape_chunk_of_four_query_tokens():
    """Four query tokens per sequence at the 14B per-layer shape (two layers), after one decode step and a
    re-tiering: every query's output and the scores against the oracle; prints the time of the chunk call."""
    from gpu_common import Pair, assert_out_close, assert_scores_close, to_f64
    cfg = dataclasses.replace(CONFIGS["14b"], n_layers=2, decode_steps=5)
    print(f"[case] 14b-shaped chunk L={cfg.n_layers} B={cfg.batch} ctx={cfg.context}", flush=True)
    p = Pair(cfg, prefetch_mode="lazy")
    L, T = cfg.n_layers, 4
    k_all, v_all, q_all = p.wl.decode_inputs(0, 1 + T)
    p.gpu.decode_step(k_all[0], v_all[0], q_all[0])
    for l in range(L):
        p.orc.append(l, to_f64(k_all[0, l]), to_f64(v_all[0, l]))
        p.orc.attend_and_score(l, to_f64(q_all[0, l]))
    n = p.gpu.layer_length(0)
    p.gpu.classify(cfg.policy_ppm)
    plan = p.gpu.get_pending_tiers()[:, :n]
    p.gpu.migrate()
    p.orc.set_tiers(plan); p.orc.migrate()
    p.gpu.wait_prefetch()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for l in range(L):
        k = torch.cat([k_all[1 + j, l] for j in range(T)], dim=1)          # [B, T, Hkv, D]
        v = torch.cat([v_all[1 + j, l] for j in range(T)], dim=1)
        p.append(l, k, v)
    for l in range(L):
        q = torch.stack([q_all[1 + j, l] for j in range(T)], dim=1).contiguous()
        ev0.record()
        out = p.gpu.attend_and_score_chunk(l, q)
        ev1.record()
        ref = p.orc.attend_and_score_chunk(l, to_f64(q))
        torch.cuda.synchronize()
        print(f"[case] layer {l}: chunk of {T} took {ev0.elapsed_time(ev1) * 1e3:.1f} us", flush=True)
        for j in range(T):
            assert_out_close(to_f64(out[:, j]), ref[:, j], cfg.kv_dtype, f"layer {l} query {j}")
    ss = 1.0 / (cfg.n_layers * cfg.n_q_heads)
    assert_scores_close(p.gpu.get_scores(), p.orc.score, n + T, (1 + T) * L * cfg.n_q_heads * ss)
    p.close()


def test_14b_shape_streamed_t1():
    """The 14B per-layer shape with streamed T1 (three layers, so a frame is refilled while the other is read): all
    outputs and scores against the oracle."""
    _run_shape(dataclasses.replace(CONFIGS["14b"], n_layers=3, decode_steps=3), "stream")


def test_batch_above_the_kernel_argument_limit_streamed_t1():
    """More than 64 sequences with streamed T1: the second attention launch and the finishing kernel take the T1
    list's length and its first logits tile from device counters."""
    cfg = small_config(name="wide", n_layers=2, batch=70, n_q_heads=4, n_kv_heads=2, head_dim=64, kv_dtype="bf16",
                       context=200, decode_steps=3, policy_ppm=(400_000, 300_000, 250_000, 50_000), k_window=16)
    _run_shape(cfg, "stream", steps_before=1, steps_after=2)


def test_host_code_under_sanitizers():
    """A randomised sequence of plans, decode steps, store rewrites and inspections in all three prefetch modes, run by a
    build of the host code with AddressSanitizer and UndefinedBehaviorSanitizer (host side only; the kernels are the
    ordinary ones): any host-memory error or undefined arithmetic in the bookkeeping aborts it."""
    import os
    import subprocess
    from paper_2605_09490_amd import build
    assert os.path.exists(build.HOST_CHECK), "build the sanitized host check first: python paper_2605_09490_amd/build.py"
    print(f"[case] {build.HOST_CHECK}", flush=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:protect_shadow_gap=0", UBSAN_OPTIONS="halt_on_error=1")
    r = subprocess.run([build.HOST_CHECK], capture_output=True, text=True, timeout=200, env=env)
    print(r.stdout[-600:], flush=True)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert "host sanitizer check passed" in r.stdout
