"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle on the same seeded inputs.
Tolerances: attention output 2e-3 (bf16 KV) / 1e-5 (fp32 KV) of each head vector's max-norm; cumulative scores
1e-4 relative; tier assignment, compaction, T2 codes and moved row bits exact."""
import numpy as np
import pytest
import torch

from oracle import tkv_oracle as O
from tkv_synth import CONFIGS, small_config

pytestmark = pytest.mark.gpu


def _pair(cfg, **kw):
    from gpu_common import Pair
    print(f"[case] {cfg.name} L={cfg.n_layers} B={cfg.batch} Hq={cfg.n_q_heads} Hkv={cfg.n_kv_heads} D={cfg.head_dim} "
          f"{cfg.kv_dtype} ctx={cfg.context} {kw}", flush=True)
    return Pair(cfg, **kw)


def _mass(cfg, calls):
    ss = cfg.score_scale if cfg.score_scale is not None else 1.0 / (cfg.n_layers * cfg.n_q_heads)
    return calls * cfg.n_q_heads * ss


def _total(p, cfg, calls, n, scorer):
    """What the underflow floor of the score tolerance is a fraction of: the total a sequence's scores have received.
    Attention scorer: the closed form (one unit per query head and call).  Value-aware scorer: every unit is weighted by
    a value-row norm, so the total is the reference's own sum over the sequence (the largest over the batch)."""
    if scorer != "attention":
        return float(p.orc.score_mag[:, :n].sum(axis=1).max())
    return _mass(cfg, calls)


@pytest.mark.parametrize("kv_dtype,D,Hq,Hkv,ctx", [
    ("f32", 64, 8, 2, 512),      # group 4, the tiny config's shape
    ("f32", 128, 4, 4, 130),     # group 1, ragged
    ("bf16", 128, 10, 2, 700),   # group 5 (14B/32B shape), several splits + tail
    ("f16", 128, 10, 2, 700),    # binary16 rows and queries (the paper's own KV type)
    ("f16", 64, 8, 2, 333),
    ("bf16", 128, 14, 2, 257),   # group 7 (7B shape), one entry past a split boundary
    ("bf16", 64, 16, 2, 256),    # group 8, exactly one split
    ("bf16", 128, 6, 2, 1),      # single token
    ("bf16", 64, 6, 3, 255),     # group 2
    ("bf16", 128, 4, 4, 300),    # group 1 on bf16 rows: dot-instruction results feed the hand-written DPP steps directly
    ("bf16", 64, 3, 3, 65),      # group 1, head_dim 64
])
def test_all_t0_attention_and_scores(kv_dtype, D, Hq, Hkv, ctx):
    from gpu_common import assert_out_close, assert_scores_close
    cfg = small_config(n_layers=2, batch=3, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, kv_dtype=kv_dtype,
                       context=ctx, decode_steps=3, sigma=1.0)
    p = _pair(cfg)
    calls = 0
    for step in range(cfg.decode_steps):
        for l in range(cfg.n_layers):
            k, v = p.wl.step_kv(step, l)
            p.append(l, k, v)
            got, ref = p.attend(l, p.wl.step_q(step, l))
            calls += 1
            assert_out_close(got, ref, kv_dtype, f"step {step} layer {l}")
    n = ctx + cfg.decode_steps
    assert_scores_close(p.gpu.get_scores(), p.orc.score, n, _mass(cfg, calls))
    # closed form: every layer call adds Hq * score_scale to each sequence's total
    assert np.allclose(p.gpu.get_scores()[:, :n].astype(np.float64).sum(1), _mass(cfg, calls), rtol=1e-4)
    p.close()


def test_bf16_output_rounding():
    """out_dtype = bf16 adds exactly one round-to-nearest-even of the binary32 result."""
    from gpu_common import Pair, to_f64
    cfg = small_config(n_layers=1, batch=2, n_q_heads=10, n_kv_heads=2, head_dim=128, kv_dtype="bf16", context=333,
                       decode_steps=0)
    a, b = Pair(cfg), Pair(cfg, out_dtype="bf16")
    q = a.wl.step_q(0, 0)
    o32 = a.gpu.attend_and_score(0, q)
    o16 = b.gpu.attend_and_score(0, q)
    assert o16.dtype == torch.bfloat16
    assert torch.equal(o32.to(torch.bfloat16), o16)
    a.close(); b.close()
    # the same for binary16 rows with a binary16 output
    cfg = small_config(n_layers=1, batch=2, n_q_heads=10, n_kv_heads=2, head_dim=128, kv_dtype="f16", context=333,
                       decode_steps=0)
    a, b = Pair(cfg), Pair(cfg, out_dtype="f16")
    q = a.wl.step_q(0, 0)
    o32 = a.gpu.attend_and_score(0, q)
    o16 = b.gpu.attend_and_score(0, q)
    assert o16.dtype == torch.float16
    assert torch.equal(o32.to(torch.float16), o16)
    a.close(); b.close()


def _random_tiers(rng, B, n, frac=(0.4, 0.3, 0.2, 0.1), protect=(4, 16)):
    t = rng.choice(4, size=(B, n), p=frac).astype(np.uint8)
    t[:, :protect[0]] = 0
    t[:, n - protect[1]:] = 0
    return t


@pytest.mark.parametrize("kv_dtype,D,Hq,Hkv,t2", [
    ("f32", 64, 8, 2, "int8_row"),
    ("bf16", 128, 10, 2, "int8_row"),
    ("f16", 128, 10, 2, "int8_row"),
    ("f16", 64, 6, 2, "int4_g32"),
    ("bf16", 128, 14, 2, "int4_g32"),
    ("bf16", 64, 8, 2, "int4_g32"),
    ("f32", 128, 8, 2, "int4_g32"),
])
@pytest.mark.parametrize("mode", ["wait", "lazy"])
def test_forced_tiers_attention_codes_and_lists(kv_dtype, D, Hq, Hkv, t2, mode):
    from gpu_common import assert_out_close, assert_scores_close
    cfg = small_config(n_layers=2, batch=2, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, kv_dtype=kv_dtype,
                       context=600, decode_steps=4, t2_format=t2, sigma=1.0)
    p = _pair(cfg, prefetch_mode=mode)
    rng = np.random.default_rng(5)
    n = cfg.context
    tiers = _random_tiers(rng, cfg.batch, n)
    p.force_tiers(tiers)
    assert np.array_equal(p.gpu.get_tiers()[:, :n], tiers)
    # compaction: per tier the ascending positions
    for b in range(cfg.batch):
        for t in range(4):
            assert np.array_equal(p.gpu.get_index_list(t, b), np.nonzero(tiers[b] == t)[0])
    # T2 codes and scales of EVERY compressed row (all layers, sequences, kv heads, K and V): bit-exact against the
    # binary32 definition
    from gpu_common import assert_t2_rows_exact
    assert assert_t2_rows_exact(p, tiers, what="first plan") > 0
    # a T1 row reads back from the pinned host store with the bits it was appended with
    b, pos = 0, int(np.nonzero(tiers[0] == 1)[0][3])
    k_ctx, v_ctx = p.wl.context_kv(1)
    row = p.gpu.get_row(1, b, 1, pos, 0)
    want = k_ctx[b, pos, 1].cpu()
    want = want.numpy() if kv_dtype == "f32" else want.view(torch.uint16).numpy()
    assert np.array_equal(row, want)
    calls = 0
    for step in range(cfg.decode_steps):
        for l in range(cfg.n_layers):
            k, v = p.wl.step_kv(step, l)
            p.append(l, k, v)
            got, ref = p.attend(l, p.wl.step_q(step, l))
            calls += 1
            assert_out_close(got, ref, kv_dtype, f"step {step} layer {l}")
    nn = n + cfg.decode_steps
    assert_scores_close(p.gpu.get_scores(), p.orc.score, nn, _mass(cfg, calls))
    s = p.gpu.get_scores()
    assert np.all(s[:, :n][tiers == 3] == 0.0)
    # second plan: promotions out of T2 (lossy value kept), T1 -> T0, T1 -> T2, more evictions
    tiers2 = np.zeros((cfg.batch, nn), np.uint8)
    tiers2[:, :n] = tiers
    move = rng.random((cfg.batch, n)) < 0.5
    newt = _random_tiers(rng, cfg.batch, n, frac=(0.35, 0.35, 0.2, 0.1))
    tiers2[:, :n] = np.where((tiers != 3) & move, newt, tiers)
    p.force_tiers(tiers2)
    assert np.array_equal(p.gpu.get_tiers()[:, :nn], tiers2)
    for b in range(cfg.batch):
        for t in range(4):
            assert np.array_equal(p.gpu.get_index_list(t, b), np.nonzero(tiers2[b] == t)[0])
    # rows encoded from a staged T1 copy, rows that kept their codes (T2 -> T2), rows re-encoded from a promoted value
    assert assert_t2_rows_exact(p, tiers2[:, :n], what="second plan") > 0
    for step in range(cfg.decode_steps, cfg.decode_steps + 2):
        for l in range(cfg.n_layers):
            got, ref = p.attend(l, p.wl.step_q(step, l))
            calls += 1
            assert_out_close(got, ref, kv_dtype, f"after 2nd plan, step {step} layer {l}")
    assert_scores_close(p.gpu.get_scores(), p.orc.score, nn, _mass(cfg, calls))
    st = p.gpu.get_stats()
    assert st["d2h_bytes"] == st["h2d_bytes"] > 0
    p.close()


@pytest.mark.parametrize("mode", ["wait", "lazy"])
@pytest.mark.parametrize("kv_dtype,D,Hq,Hkv", [("bf16", 128, 10, 2), ("f32", 64, 8, 2), ("f16", 128, 10, 2)])
def test_prop1_t1_placement_is_bit_invisible(mode, kv_dtype, D, Hq, Hkv):
    """Zero-error offloading: the run with rows in T1 (round trip through pinned host memory and the
    staging buffer) gives the same bits as the run with those rows left in T0 -- outputs and scores."""
    from gpu_common import Pair
    cfg = small_config(n_layers=3, batch=2, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, kv_dtype=kv_dtype,
                       context=900, decode_steps=6, sigma=1.2)
    rng = np.random.default_rng(9)
    n = cfg.context
    tiers = _random_tiers(rng, cfg.batch, n, frac=(0.3, 0.5, 0.15, 0.05))
    twin = np.where(tiers == 1, 0, tiers).astype(np.uint8)
    outs = []
    for tt in (tiers, twin):
        print(f"[case] prop1 {mode} {kv_dtype} t1_rows={(tt == 1).sum()}", flush=True)
        p = Pair(cfg, prefetch_mode=mode)
        p.gpu.set_tiers(tt)
        p.gpu.migrate()
        res = []
        for step in range(cfg.decode_steps):
            for l in range(cfg.n_layers):
                k, v = p.wl.step_kv(step, l)
                p.gpu.append(l, k, v)
                res.append(p.gpu.attend_and_score(l, p.wl.step_q(step, l)).cpu())
        outs.append((torch.stack(res), p.gpu.get_scores().copy()))
        p.close()
    assert torch.equal(outs[0][0].view(torch.uint8), outs[1][0].view(torch.uint8))
    assert np.array_equal(outs[0][1].view(np.uint32), outs[1][1].view(np.uint32))


@pytest.mark.parametrize("kv_dtype,D,Hq,Hkv,t2", [("bf16", 128, 10, 2, "int8_row"), ("f16", 64, 8, 2, "int4_g32")])
def test_prop1_holds_for_chunks_of_query_tokens(kv_dtype, D, Hq, Hkv, t2):
    """Zero-error offloading on the chunk path (several query tokens as columns of one launch): with rows in T1 the
    outputs of every query token and the scores have the same bits as with those rows left in T0."""
    from gpu_common import Pair
    cfg = small_config(n_layers=2, batch=2, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, kv_dtype=kv_dtype,
                       context=700, decode_steps=8, sigma=1.2, t2_format=t2)
    rng = np.random.default_rng(13)
    tiers = _random_tiers(rng, cfg.batch, cfg.context, frac=(0.3, 0.45, 0.2, 0.05))
    twin = np.where(tiers == 1, 0, tiers).astype(np.uint8)
    outs = []
    for tt in (tiers, twin):
        print(f"[case] prop1 chunk {kv_dtype} t1_rows={(tt == 1).sum()}", flush=True)
        p = Pair(cfg, prefetch_mode="lazy")
        p.gpu.set_tiers(tt)
        p.gpu.migrate()
        res, step = [], 0
        for T in (5, 3):
            for l in range(cfg.n_layers):
                ks, vs = zip(*[p.wl.step_kv(step + j, l) for j in range(T)])
                p.gpu.append(l, torch.cat(ks, dim=1), torch.cat(vs, dim=1))
            for l in range(cfg.n_layers):
                q = torch.stack([p.wl.step_q(step + j, l) for j in range(T)], dim=1).contiguous()
                res.append(p.gpu.attend_and_score_chunk(l, q).cpu().reshape(-1))
            step += T
        outs.append((torch.cat(res), p.gpu.get_scores().copy()))
        p.close()
    assert torch.equal(outs[0][0].view(torch.uint8), outs[1][0].view(torch.uint8))
    assert np.array_equal(outs[0][1].view(np.uint32), outs[1][1].view(np.uint32))


@pytest.mark.parametrize("mode", ["wait", "lazy"])
def test_rows_returning_to_t1_reuse_their_host_copy(mode):
    """A row that goes T1 -> T0 -> T1 is not transferred a second time (its bits in the pinned store are still
    current): no bytes move, the row is copied inside HBM into a staging slot, and attention stays bit-identical to
    the all-T0 twin; rows that pass through T2 on the way lose the host copy and are transferred again."""
    from gpu_common import Pair
    cfg = small_config(n_layers=2, batch=2, n_q_heads=10, n_kv_heads=2, head_dim=128, kv_dtype="bf16", context=700,
                       decode_steps=6, sigma=1.0)
    rng = np.random.default_rng(21)
    n = cfg.context
    t_a = _random_tiers(rng, cfg.batch, n, frac=(0.4, 0.6, 0.0, 0.0))
    cand = t_a == 1
    flip = cand & (rng.random(t_a.shape) < 0.5)
    t_b = np.where(flip, 0, t_a).astype(np.uint8)                 # half of the T1 rows come up to T0
    via_t2 = flip & (rng.random(t_a.shape) < 0.3)
    t_c = np.where(via_t2, 2, t_b).astype(np.uint8)               # some of those go on to T2 ...
    t_d = t_a.copy()                                              # ... and everything returns to where it started
    twin_seq = [np.where(t == 1, 0, t).astype(np.uint8) for t in (t_a, t_b, t_c, t_d)]
    outs = []
    for seq_t in ((t_a, t_b, t_c, t_d), twin_seq):
        p = Pair(cfg, prefetch_mode=mode)
        res, moved = [], []
        step = 0
        for tt in seq_t:
            p.gpu.set_tiers(tt)
            before = p.gpu.get_stats()["h2d_bytes"]
            p.gpu.migrate()
            for l in range(cfg.n_layers):
                k, v = p.wl.step_kv(step, l)
                p.gpu.append(l, k, v)
                res.append(p.gpu.attend_and_score(l, p.wl.step_q(step, l)).cpu())
            step += 1
            p.gpu.wait_prefetch()
            moved.append(p.gpu.get_stats()["h2d_bytes"] - before)
        outs.append((torch.stack(res), p.gpu.get_scores().copy(), moved))
        p.close()
    row_bytes = cfg.n_kv_heads * 2 * cfg.head_dim * 2 * cfg.n_layers
    moved = outs[0][2]
    print(f"[case] reuse {mode}: bytes per migrate {moved}", flush=True)
    assert moved[0] == int(cand.sum()) * row_bytes
    assert moved[1] == 0 and moved[2] == 0
    assert moved[3] == int(via_t2.sum()) * row_bytes              # only the rows whose values changed in T2
    assert outs[1][2] == [0, 0, 0, 0]
    assert torch.equal(outs[0][0].view(torch.uint8), outs[1][0].view(torch.uint8))
    assert np.array_equal(outs[0][1].view(np.uint32), outs[1][1].view(np.uint32))


@pytest.mark.parametrize("mode,kv_dtype,D,Hq,Hkv,t2", [
    ("lazy", "bf16", 128, 10, 2, "int8_row"),
    ("lazy", "f16", 128, 10, 2, "int4_g32"),
    ("wait", "bf16", 128, 10, 2, "int4_g32"),
    ("lazy", "f32", 64, 8, 2, "int8_row"),
])
def test_random_walk_of_plans(mode, kv_dtype, D, Hq, Hkv, t2):
    """Eight forced plans in a row, each moving a random 40 % of the surviving positions to a random tier (every
    transition, rows that return to T1 with or without a detour through T2, slots freed and taken again), with
    tokens appended in between; after every plan the tier array, the four index lists, one attention call per layer
    and the stored bits of a few T0 / T1 rows are compared with the oracle, and the scores at the end."""
    st = _plan_walk(mode, kv_dtype, D, Hq, Hkv, t2)
    assert st["n_rehome"] == 0


@pytest.mark.parametrize("mode", ["wait", "lazy", "stream"])
@pytest.mark.parametrize("piece_rows", [100, 600])
def test_walk_with_small_bounce_rings(mode, piece_rows):
    """The same walk over 5 layers with bounce rings whose pieces hold 100 or 600 positions of one layer, against the
    ~200-350 positions that enter T1 at a plan: with 100 every layer's rows take several copies, with 600 the rows
    of two layers share a piece and one strided copy (a last group of one layer, and a first plan whose rows fill a
    piece alone).  Every T1 row of the last layer is read back from the pinned store after every plan."""
    tok_bytes = 2 * 2 * 64 * 2
    st = _plan_walk(mode, "bf16", 64, 8, 2, "int8_row", all_t1_rows=True, rounds=5, layers=5,
                    bounce_bytes=4 * piece_rows * tok_bytes)
    assert st["n_rehome"] == 0
    copies_one_per_layer = 5 * 5
    if piece_rows == 100:
        assert st["d2h_copies"] > copies_one_per_layer
    else:
        assert 0 < st["d2h_copies"] < copies_one_per_layer


@pytest.mark.parametrize("mode,layers", [("wait", 2), ("lazy", 2), ("stream", 2), ("stream", 5)])
def test_pinned_store_is_rewritten_when_it_runs_out(mode, layers):
    """A longer walk of the same kind with a pinned store of 520 rows: T1 holds ~300 rows and ~100 enter at every plan, so the store
    (rows are handed out in order) runs out every second or third plan and is rewritten from the staged copies; after every
    plan EVERY T1 row of one (layer, kv head) is read back from the pinned store and compared bit by bit.  (Streamed
    T1 has no staged copies: there the rows pass through the frames on their way to their new place, and the store
    is also rewritten, beside the frame pass of a plan, as soon as its stale rows would cost more link time than
    that.)"""
    st = _plan_walk(mode, "bf16", 128, 10, 2, "int8_row", host_rows=520, all_t1_rows=True, rounds=16, layers=layers)
    print(f"[case] store rewritten {st['n_rehome']} + {st['n_repack']} times, {st['host_rows_used']} rows in use", flush=True)
    assert st["n_rehome"] + st["n_repack"] >= 2 and st["host_rows_used"] <= 520
    assert (st["n_repack"] > 0) == (mode == "stream")


@pytest.mark.parametrize("kv_dtype,D,Hq,Hkv,t2,layers", [
    ("bf16", 128, 10, 2, "int8_row", 5),
    ("f16", 128, 10, 2, "int8_row", 3),
    ("f32", 64, 8, 2, "int4_g32", 2),
    ("bf16", 64, 3, 3, "int8_row", 1),
])
def test_streamed_t1_walk(kv_dtype, D, Hq, Hkv, t2, layers):
    """Streamed T1: no per-layer staging buffer; every attention call reads its layer's T1 rows from one of two
    frames refilled from the pinned store.  The same random walk of plans (rows leaving T1 for T0 and T2 are read back
    through the frames, rows returning to T1 with a valid host copy move nothing), every T1 row's bits in the pinned
    store, outputs and scores against the oracle; with 5, 2 and 1 layers (frames recycled, one layer per frame, one
    frame)."""
    st = _plan_walk("stream", kv_dtype, D, Hq, Hkv, t2, all_t1_rows=True, layers=layers)
    assert st["h2d_bytes"] > st["d2h_bytes"] > 0        # T1 crosses the link again at every step


def _plan_walk(mode, kv_dtype, D, Hq, Hkv, t2, host_rows=None, all_t1_rows=False, rounds=8, layers=2, **create_kw):
    from gpu_common import assert_out_close, assert_scores_close, assert_t2_rows_exact
    cfg = small_config(n_layers=layers, batch=2, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, kv_dtype=kv_dtype,
                       context=500, decode_steps=rounds, t2_format=t2, sigma=1.0)
    p = _pair(cfg, prefetch_mode=mode, **({"host_rows": host_rows} if host_rows else {}), **create_kw)
    rng = np.random.default_rng(77)
    n = cfg.context
    tiers = np.zeros((cfg.batch, n), np.uint8)
    calls = 0
    for rnd in range(rounds):
        move = (rng.random((cfg.batch, n)) < 0.4) & (tiers != 3)
        prop = _random_tiers(rng, cfg.batch, n, frac=(0.3, 0.35, 0.25, 0.1), protect=(4, 8))
        tiers = np.where(move, prop, tiers).astype(np.uint8)
        tiers[:, :4] = 0
        tiers[:, n - 8:] = 0
        print(f"[case] walk {mode} {kv_dtype} round {rnd} n={n} counts={np.bincount(tiers.ravel(), minlength=4)}", flush=True)
        p.force_tiers(tiers)
        assert np.array_equal(p.gpu.get_tiers()[:, :n], tiers)
        for b in range(cfg.batch):
            for t in range(4):
                assert np.array_equal(p.gpu.get_index_list(t, b), np.nonzero(tiers[b] == t)[0])
        # stored bits of a few full-precision rows (T0 in HBM, T1 in the pinned store)
        for t in (0, 1):
            pos_t = np.nonzero(tiers[1] == t)[0]
            for pos in (pos_t if (t == 1 and all_t1_rows) else rng.choice(pos_t, size=min(3, len(pos_t)), replace=False)):
                for which, store in ((0, p.orc.K), (1, p.orc.V)):
                    row = p.gpu.get_row(cfg.n_layers - 1, 1, 1, int(pos), which)
                    if kv_dtype == "bf16":
                        row = (row.astype(np.uint32) << 16).view(np.float32)
                    elif kv_dtype == "f16":
                        row = row.view(np.float16)
                    assert np.array_equal(row.astype(np.float64), store[cfg.n_layers - 1][1, 1, int(pos)]), (rnd, t, pos, which)
        # codes and scales of every T2 row of one (layer, sequence, kv head): rows encoded from HBM, from a staged or
        # streamed T1 copy, re-encoded after a promotion, or kept as they were
        assert_t2_rows_exact(p, tiers, layers=[cfg.n_layers - 1], seqs=[1], kv_heads=[cfg.n_kv_heads - 1], what=f"round {rnd}")
        for l in range(cfg.n_layers):
            k, v = p.wl.step_kv(rnd, l)
            p.append(l, k, v)
            got, ref = p.attend(l, p.wl.step_q(rnd, l))
            calls += 1
            assert_out_close(got, ref, kv_dtype, f"round {rnd} layer {l}")
        n += 1
        tiers = np.concatenate([tiers, np.zeros((cfg.batch, 1), np.uint8)], axis=1)
    assert_scores_close(p.gpu.get_scores(), p.orc.score, n, _mass(cfg, calls), mag64=p.orc.score_mag)
    p.gpu.wait_prefetch()
    st = p.gpu.get_stats()
    assert st["tier_count"] == [int(c) for c in np.bincount(tiers[:, :n - 1].ravel(), minlength=4) + np.array([cfg.batch, 0, 0, 0])]
    p.close()
    return st


@pytest.mark.parametrize("rule", [0, 1])
@pytest.mark.parametrize("seed", range(4))
def test_classify_bit_exact_given_scores(seed, rule):
    """Tier assignment is an integer function of the binary32 score array: the GPU's radix select must
    reproduce the oracle's explicit sort, ties and already-evicted positions included; with both count rules (fixed
    fractions of all candidates, and Algorithm 1's floors that evict again at every event)."""
    from gpu_common import Pair
    rng = np.random.default_rng(seed)
    ctx = int(rng.integers(300, 2500))
    cfg = small_config(n_layers=1, batch=4, n_q_heads=4, n_kv_heads=2, head_dim=64, kv_dtype="bf16", context=ctx,
                       decode_steps=0, k_sink=int(rng.integers(0, 6)), k_window=int(rng.integers(0, 200)),
                       n_prompt=int(rng.integers(0, 50)))
    p = _pair(cfg)
    n = ctx
    s = (rng.random((cfg.batch, cfg.max_tokens)) ** 6).astype(np.float32)
    s[1] = rng.choice(np.array([0, 1e-3, 0.5, 0.5000001, 2.0], np.float32), size=cfg.max_tokens)   # heavy ties
    s[2, : n // 2] = 0.0
    p.gpu.set_scores(s)
    pols = [(300000, 520000, 150000, 30000), (500000, 300000, 150000, 50000), (100000, 100000, 100000, 700000),
            (0, 0, 0, 1000000)]
    tier_prev = np.zeros((cfg.batch, n), np.uint8)
    if rule == 1:
        pols = [pols[0], pols[0], pols[1], pols[0], pols[2]] + ([pols[3]] if seed % 2 == 0 else [])   # repeated events compound
    for pol in pols[: 3 if (seed % 2 and rule == 0) else len(pols)]:
        p.gpu.classify(pol, count_rule=rule)
        got = p.gpu.get_pending_tiers()[:, :n]
        for b in range(cfg.batch):
            want = O.classify_sequence(s[b], tier_prev[b], n, cfg.n_prompt, cfg.k_sink, cfg.k_window, pol, rule)
            assert np.array_equal(got[b], want), f"seq {b} policy {pol}: {(got[b] != want).sum()} positions differ"
        p.gpu.migrate()
        tier_prev = p.gpu.get_tiers()[:, :n].copy()
        assert np.array_equal(tier_prev, got)
        for b in range(cfg.batch):
            lists = O.compact_lists(tier_prev[b], n)
            for t in range(4):
                assert np.array_equal(p.gpu.get_index_list(t, b), lists[t])
    p.close()


def test_tiny_config_teacher_forced():
    """The tiny benchmark configuration: 1 layer, 8/2 heads, d 64, fp32, 512-token context, 32 steps, re-tiering every 8 steps
    (plus once before the first step).  At each event the oracle's ranking of the GPU's score array must equal
    the GPU's plan bit for bit; the oracle then adopts that plan (teacher forcing)."""
    from gpu_common import assert_out_close, assert_scores_close
    cfg = CONFIGS["tiny"]
    p = _pair(cfg)
    calls = 0

    def retier():
        n = p.gpu.layer_length(0)
        p.gpu.classify(cfg.policy_ppm)
        plan = p.gpu.get_pending_tiers()[:, :n]
        s_gpu = p.gpu.get_scores()
        want = p.orc.classify(cfg.policy_ppm, score_f32=s_gpu)[:, :n]
        assert np.array_equal(plan, want)
        free = p.orc.classify(cfg.policy_ppm)[:, :n]
        print(f"[tiny] n={n} free-running oracle differs from the GPU plan at {(free != plan).sum()} positions", flush=True)
        p.gpu.migrate()
        p.orc.set_tiers(plan)
        p.orc.migrate()

    retier()   # all scores are zero: ties broken by position
    for step in range(cfg.decode_steps):
        k, v = p.wl.step_kv(step, 0)
        p.append(0, k, v)
        got, ref = p.attend(0, p.wl.step_q(step, 0))
        calls += 1
        assert_out_close(got, ref, "f32", f"step {step}")
        if (step + 1) % cfg.reclassify_every == 0:
            assert_scores_close(p.gpu.get_scores(), p.orc.score, p.gpu.layer_length(0), _mass(cfg, calls), f"step {step}")
            retier()
    st = p.gpu.get_stats()
    assert sum(st["tier_count"]) == cfg.context + cfg.decode_steps
    p.close()


def test_error_paths_leave_the_gpu_alone():
    import paper_2605_09490_amd as tkv
    from gpu_common import Pair
    cfg = small_config(n_layers=2, batch=1, context=40, decode_steps=2)
    p = Pair(cfg)
    q = p.wl.step_q(0, 0)
    with pytest.raises(tkv.TkvError) as e:
        p.gpu.migrate()
    assert e.value.status == tkv.TKV_ESTATE
    with pytest.raises(tkv.TkvError) as e:
        p.gpu.classify((1, 2, 3, 4))
    assert e.value.status == tkv.TKV_EINVAL
    with pytest.raises(tkv.TkvError) as e:      # unknown count rule
        p.gpu.classify(cfg.policy_ppm, count_rule=2)
    assert e.value.status == tkv.TKV_EINVAL
    k, v = p.wl.step_kv(0, 0)
    p.gpu.append(0, k, v)
    with pytest.raises(tkv.TkvError) as e:      # layer 1 is one token short
        p.gpu.classify(cfg.policy_ppm)
    assert e.value.status == tkv.TKV_ESTATE
    with pytest.raises(tkv.TkvError) as e:
        p.gpu.attend_and_score(1, q)
    assert e.value.status == tkv.TKV_ESTATE
    p.gpu.append(1, *p.wl.step_kv(0, 1))
    p.gpu.append(0, *p.wl.step_kv(1, 0))
    p.gpu.append(1, *p.wl.step_kv(1, 1))
    with pytest.raises(tkv.TkvError) as e:
        p.gpu.append(0, k, v)
    assert e.value.status == tkv.TKV_ECAPACITY
    t = np.zeros((1, 42), np.uint8)
    t[0, 10] = 3
    p.gpu.set_tiers(t); p.gpu.migrate()
    t[0, 10] = 0
    p.gpu.set_tiers(t)
    with pytest.raises(tkv.TkvError) as e:      # an evicted position cannot come back
        p.gpu.migrate()
    assert e.value.status == tkv.TKV_ESTATE
    p.close()


def test_allocator_failure_gives_enomem():
    """An allocator callback that returns NULL part-way through tkv_create: TKV_ENOMEM, everything handed out so far
    is given back, no handle."""
    import ctypes as C
    import paper_2605_09490_amd as tkv
    from paper_2605_09490_amd import binding
    lib = tkv.load_library()
    held, calls = {}, {"n": 0, "freed": 0}

    def dev_alloc(nbytes, _ctx):
        calls["n"] += 1
        if calls["n"] > 5:
            return None
        t = torch.empty(int(nbytes), dtype=torch.uint8, device="cuda")
        held[t.data_ptr()] = t
        return t.data_ptr()

    def dev_free(ptr, _ctx):
        calls["freed"] += 1
        held.pop(ptr, None)

    def pin_alloc(nbytes, _ctx):
        t = torch.empty(int(nbytes), dtype=torch.uint8, pin_memory=True)
        held[t.data_ptr()] = t
        return t.data_ptr()

    cbs = (binding.ALLOC_FN(dev_alloc), binding.FREE_FN(dev_free), binding.ALLOC_FN(pin_alloc), binding.FREE_FN(dev_free))
    cfg = binding.tkv_config()
    cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.max_tokens = 1, 1, 4, 2, 64, 128
    cfg.kv_dtype, cfg.out_dtype, cfg.t2_format = binding.TKV_BF16, binding.TKV_F32, binding.TKV_T2_INT8_ROW
    cfg.dev_alloc, cfg.dev_free, cfg.pin_alloc, cfg.pin_free = cbs
    h = C.c_void_p()
    assert lib.tkv_create(C.byref(cfg), C.byref(h)) == tkv.TKV_ENOMEM
    assert not h.value and calls["freed"] == 5 and not held


def test_pool_capacities_are_checked_before_anything_moves():
    import paper_2605_09490_amd as tkv
    from gpu_common import Pair, assert_out_close
    cfg = small_config(n_layers=2, batch=2, n_q_heads=8, n_kv_heads=2, head_dim=64, kv_dtype="bf16", context=200,
                       decode_steps=4)
    # staging buffer too small for the plan: ECAPACITY, the plan stays pending, tiers unchanged, attention still right
    p = Pair(cfg, staging_rows=10, t2_rows=50)
    t = np.zeros((cfg.batch, 200), np.uint8)
    t[:, 50:90] = 1
    p.gpu.set_tiers(t)
    with pytest.raises(tkv.TkvError) as e:
        p.gpu.migrate()
    assert e.value.status == tkv.TKV_ECAPACITY
    assert np.all(p.gpu.get_tiers() == 0)
    t[:, 60:90] = 2                                   # 10 rows to T1, 30 to T2: fits
    p.gpu.set_tiers(t); p.gpu.migrate()
    p.orc.set_tiers(t); p.orc.migrate()
    k, v = p.wl.step_kv(0, 0)
    for l in range(2):
        p.append(l, *p.wl.step_kv(0, l))
        got, ref = p.attend(l, p.wl.step_q(0, l))
        assert_out_close(got, ref, "bf16")
    t2 = np.zeros((cfg.batch, 201), np.uint8)
    t2[:, :201] = np.pad(t, ((0, 0), (0, 1)))
    t2[:, 100:160] = 2                                # 90 rows in T2 > 50 slots
    p.gpu.set_tiers(t2)
    with pytest.raises(tkv.TkvError) as e:
        p.gpu.migrate()
    assert e.value.status == tkv.TKV_ECAPACITY
    p.close()
    # streamed T1: the frames are too small for the plan; afterwards a plan that fits works
    p = Pair(cfg, staging_rows=10, prefetch_mode="stream")
    t = np.zeros((cfg.batch, 200), np.uint8)
    t[:, 50:90] = 1
    p.gpu.set_tiers(t)
    with pytest.raises(tkv.TkvError) as e:
        p.gpu.migrate()
    assert e.value.status == tkv.TKV_ECAPACITY
    assert np.all(p.gpu.get_tiers() == 0)
    t[:, 58:90] = 0                                   # 8 rows to T1
    p.gpu.set_tiers(t); p.gpu.migrate()
    p.orc.set_tiers(t); p.orc.migrate()
    for l in range(2):
        p.append(l, *p.wl.step_kv(0, l))
        got, ref = p.attend(l, p.wl.step_q(0, l))
        assert_out_close(got, ref, "bf16")
    p.close()
    # pinned host store too small
    p = Pair(cfg, host_rows=16)
    t = np.zeros((cfg.batch, 200), np.uint8)
    t[:, 50:70] = 1                                   # 2 x 20 rows > 16
    p.gpu.set_tiers(t)
    with pytest.raises(tkv.TkvError) as e:
        p.gpu.migrate()
    assert e.value.status == tkv.TKV_ECAPACITY
    p.close()
    # HBM pool too small for the appended tokens
    p = Pair(cfg, t0_rows=201, preload=True)
    p.gpu.append(0, *p.wl.step_kv(0, 0))
    with pytest.raises(tkv.TkvError) as e:
        p.gpu.append(0, *p.wl.step_kv(1, 0))
    assert e.value.status == tkv.TKV_ECAPACITY
    p.close()


@pytest.mark.parametrize("mode,kv_dtype,D,Hq,Hkv,t2", [
    ("lazy", "bf16", 128, 10, 2, "int8_row"),
    ("stream", "f16", 128, 8, 2, "int4_g32"),
    ("wait", "f32", 64, 6, 2, "int8_row"),
])
def test_value_aware_scorer_walk(mode, kv_dtype, D, Hq, Hkv, t2):
    """The plan walk with the value-aware scorer of the scoring ablation: every head's weight times the Euclidean norm
    of the value row it reads (taken when the row is appended, whatever tier the row is in later); scores against
    the oracle's at the end, outputs as always."""
    _plan_walk(mode, kv_dtype, D, Hq, Hkv, t2, layers=3, scorer="vatp")


@pytest.mark.parametrize("mode,kv_dtype,D,Hq,Hkv,t2,scorer,weight", [
    ("lazy", "bf16", 128, 10, 2, "int8_row", "redundancy", 1.0),
    ("wait", "f16", 64, 8, 2, "int4_g32", "combined", 2.5),
    ("stream", "bf16", 128, 14, 2, "int8_row", "redundancy", 0.4),
    ("lazy", "f32", 64, 6, 2, "int8_row", "combined", 1.0),
])
def test_redundancy_scorers_walk(mode, kv_dtype, D, Hq, Hkv, t2, scorer, weight):
    """The plan walk with the redundancy-penalised scorers of the scoring ablation ("attn - redundancy", "attn x val -
    redundancy"): the penalty is the clamped cosine of a key row with the row appended before it (taken at append,
    whatever happens to either row later), spread over the positions a query attends to.  The walk's appended rows
    are random, so half of the cosines are clamped to zero and the rest are small: scores against the oracle's."""
    _plan_walk(mode, kv_dtype, D, Hq, Hkv, t2, layers=3, scorer=scorer, redundancy_weight=weight)


def test_redundancy_of_crafted_key_rows():
    """Key rows whose neighbours are copies, scaled copies, opposed, orthogonal or zero: after one attention call per
    layer the scores are the oracle's (cosines 1, 1, 0 (clamped), 0, 0), also across an append boundary where the
    neighbour is the row kept from the previous append, and after that neighbour has been evicted."""
    from gpu_common import Pair, assert_scores_close, to_f64
    cfg = small_config(n_layers=2, batch=2, n_q_heads=4, n_kv_heads=2, head_dim=64, kv_dtype="bf16", context=40,
                       decode_steps=4, sigma=1.0, k_window=4, k_sink=2)
    p = Pair(cfg, prefetch_mode="lazy", preload=False, scorer="redundancy", redundancy_weight=3.0)
    g = torch.Generator(device="cpu").manual_seed(5)
    base = torch.randn((cfg.batch, 1, cfg.n_kv_heads, cfg.head_dim), generator=g)
    other = torch.randn((cfg.batch, 1, cfg.n_kv_heads, cfg.head_dim), generator=g)
    orth = other - (other * base).sum(-1, keepdim=True) / (base * base).sum(-1, keepdim=True) * base
    rows = [base, base, 2.0 * base, -base, orth, torch.zeros_like(base), base, 0.5 * base]
    k = torch.cat(rows + [torch.randn((cfg.batch, 32, cfg.n_kv_heads, cfg.head_dim), generator=g)], dim=1).to(torch.bfloat16).cuda()
    v = torch.randn(k.shape, generator=g).to(torch.bfloat16).cuda()
    for l in range(cfg.n_layers):
        p.append(l, k[:, :5].contiguous(), v[:, :5].contiguous())      # the boundary falls between "-base" and "orth" ...
    tiers = np.zeros((cfg.batch, 5), np.uint8); tiers[:, 4] = 3      # ... and "orth"'s own row is evicted afterwards
    tiers[:, 3] = 3                                                   # as is the neighbour the next append compares with
    p.force_tiers(tiers)
    for l in range(cfg.n_layers):
        p.append(l, k[:, 5:].contiguous(), v[:, 5:].contiguous())
    n = k.shape[1]
    calls = 0
    for l in range(cfg.n_layers):
        q = torch.randn((cfg.batch, cfg.n_q_heads, cfg.head_dim), generator=g).to(torch.bfloat16).cuda()
        p.attend(l, q); calls += 1
    rho = p.orc.rho[0][:, :, :8]
    want = np.array([0, 1, 1, 0, 0, 0, 0, 1], np.float64)
    assert np.allclose(rho, want[None, None, :], atol=2e-2)          # bf16 rounding of the crafted rows
    assert_scores_close(p.gpu.get_scores(), p.orc.score, n, float(p.orc.score_mag[:, :n].sum(axis=1).max()),
                        "crafted neighbours", mag64=p.orc.score_mag)
    assert (p.orc.score[:, :n] < 0).any()                             # the penalty really takes scores below zero
    p.close()


@pytest.mark.parametrize("mode,scorer", [("lazy", "vatp"), ("stream", "vatp"), ("stream", "attention"),
                                         ("lazy", "redundancy"), ("wait", "combined")])
def test_whole_steps_and_classify(mode, scorer):
    """Whole decode steps (one append launch for all layers, so the norms of the new rows of every layer come from one
    launch) with re-tiering by the value-aware scores: the plan is the oracle's for the GPU's score array, bit for bit,
    and the scores agree with the oracle's to the usual tolerance."""
    _whole_steps(mode, scorer)


@pytest.mark.parametrize("mode,scorer", [("lazy", "attention"), ("wait", "redundancy")])
def test_whole_steps_and_classify_with_a_log_normal_attention_profile(mode, scorer):
    """The same with inputs whose attention is spread log-normally over the positions (the profile the method is
    described on) instead of collapsing onto a few: every candidate carries a distinct, non-negligible score, so the
    band boundaries are decided among close values rather than among ties at zero."""
    _whole_steps(mode, scorer, recipe="bias")


def _whole_steps(mode, scorer, **cfg_kw):
    from gpu_common import assert_scores_close
    cfg = small_config(n_layers=3, batch=2, n_q_heads=10, n_kv_heads=2, head_dim=128, kv_dtype="bf16", context=700,
                       decode_steps=12, sigma=1.0, k_window=16, **cfg_kw)
    p = _pair(cfg, prefetch_mode=mode, scorer=scorer)
    pol = (300000, 400000, 200000, 100000)
    calls = 0
    for step in range(cfg.decode_steps):
        ks, vs, qs = zip(*[(*p.wl.step_kv(step, l), p.wl.step_q(step, l)) for l in range(cfg.n_layers)])
        k_all, v_all, q_all = torch.stack(ks), torch.stack(vs), torch.stack(qs)
        p.gpu.decode_step(k_all, v_all, q_all)
        for l in range(cfg.n_layers):
            from gpu_common import to_f64
            p.orc.append(l, to_f64(ks[l]), to_f64(vs[l]))
            p.orc.attend_and_score(l, to_f64(qs[l]))
            calls += 1
        if step % 4 == 3:
            n = p.gpu.layer_length(0)
            s_gpu = p.gpu.get_scores()
            assert_scores_close(s_gpu, p.orc.score, n, _total(p, cfg, calls, n, scorer), f"step {step}", mag64=p.orc.score_mag)
            p.gpu.classify(pol)
            plan = p.gpu.get_pending_tiers()[:, :n]
            assert np.array_equal(plan, p.orc.classify(pol, score_f32=s_gpu)[:, :n])
            p.gpu.migrate()
            p.orc.set_tiers(plan); p.orc.migrate()
    # the scores really are not the attention-only ones
    if scorer == "vatp":
        assert p.orc.score.sum() > 2.0 * cfg.batch * _mass(cfg, calls)
    st = p.gpu.get_stats()
    print(f"[case] {mode} {scorer}: store rewritten beside a plan {st['n_repack']} times", flush=True)
    if mode == "stream":
        # every T1 row of one (layer, sequence, kv head) in the pinned store, bit for bit
        n = p.gpu.layer_length(0)
        tiers = p.gpu.get_tiers()[:, :n]
        for pos in np.nonzero(tiers[1] == 1)[0]:
            row = p.gpu.get_row(cfg.n_layers - 1, 1, 1, int(pos), 1)
            row = (row.astype(np.uint32) << 16).view(np.float32)
            assert np.array_equal(row.astype(np.float64), p.orc.V[cfg.n_layers - 1][1, 1, int(pos)]), pos
        assert st["n_repack"] >= 1
    p.close()


@pytest.mark.parametrize("mode,kv_dtype,D,Hq,Hkv,t2,scorer,batch", [
    ("lazy", "bf16", 128, 10, 2, "int8_row", "attention", 2),
    ("stream", "bf16", 128, 10, 2, "int4_g32", "attention", 2),
    ("wait", "f32", 64, 8, 2, "int8_row", "vatp", 2),
    ("lazy", "f16", 128, 7, 1, "int8_row", "attention", 3),
    ("lazy", "bf16", 64, 2, 1, "int8_row", "attention", 66),      # list lengths from the device counters
    # the chunk launch on the matrix cores: int4 codes, both element types, groups of 1 .. 8 heads
    ("lazy", "bf16", 128, 8, 1, "int4_g32", "attention", 2),      # G = 8: 4 tokens per launch
    ("lazy", "f16", 64, 4, 1, "int4_g32", "vatp", 2),             # G = 4, 64-byte code rows: 8 tokens per launch
    ("wait", "bf16", 64, 3, 3, "int8_row", "attention", 2),       # G = 1: the 9-token chunk in one launch
    ("lazy", "bf16", 128, 12, 2, "int4_g32", "attention", 2),     # G = 6: 5 tokens per launch, 30 columns
    ("lazy", "f16", 128, 10, 2, "int8_row", "attention", 2),      # G = 5, binary16
    ("lazy", "bf16", 64, 6, 2, "int4_g32", "attention", 3),       # G = 3, 32-byte code rows
    ("lazy", "bf16", 128, 10, 2, "int8_row", "redundancy", 2),    # the penalty per query token: its own count of positions
    ("wait", "f32", 64, 8, 2, "int8_row", "combined", 2),
])
def test_chunks_of_query_tokens(mode, kv_dtype, D, Hq, Hkv, t2, scorer, batch):
    """Several query tokens per sequence at once: chunks of 6, 1 and 9 tokens appended to every layer and attended
    causally (query j sees the positions up to its own), over a cache with all four tiers; every query's output and
    the scores at the end against the oracle.  With 9 tokens the chunk crosses a 64-entry tile boundary of list F
    for at least one query.  A chunk that reaches behind the last migrate is refused."""
    import paper_2605_09490_amd as tkv
    from gpu_common import assert_out_close, assert_scores_close
    cfg = small_config(n_layers=2, batch=batch, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, kv_dtype=kv_dtype,
                       context=200 if batch > 8 else 450, decode_steps=16, t2_format=t2, sigma=1.0)
    p = _pair(cfg, prefetch_mode=mode, scorer=scorer)
    rng = np.random.default_rng(31)
    n = cfg.context
    tiers = _random_tiers(rng, cfg.batch, n, frac=(0.35, 0.3, 0.25, 0.1), protect=(4, 8))
    p.force_tiers(tiers)
    calls, step = 0, 0
    for T in (6, 1, 9):
        for l in range(cfg.n_layers):
            ks, vs = zip(*[p.wl.step_kv(step + j, l) for j in range(T)])
            p.append(l, torch.cat(ks, dim=1), torch.cat(vs, dim=1))
        for l in range(cfg.n_layers):
            q = torch.stack([p.wl.step_q(step + j, l) for j in range(T)], dim=1).contiguous()
            print(f"[case] chunk T={T} layer {l} n={n + T}", flush=True)
            got, ref = p.attend_chunk(l, q)
            calls += T
            for j in range(T):
                assert_out_close(got[:, j], ref[:, j], kv_dtype, f"chunk {T} layer {l} query {j}")
        step += T
        n += T
    assert_scores_close(p.gpu.get_scores(), p.orc.score, n, _total(p, cfg, calls, n, scorer), mag64=p.orc.score_mag)
    # 16 positions were appended since the plan: a chunk of 17 would reach into re-tiered positions
    q17 = torch.zeros((cfg.batch, 17, Hq, D), dtype=q.dtype, device=q.device)
    with pytest.raises(tkv.TkvError) as e:
        p.gpu.attend_and_score_chunk(0, q17)
    assert e.value.status == tkv.TKV_ESTATE
    p.close()


@pytest.mark.parametrize("mix,mode", [("all_t2", "lazy"), ("all_t3", "wait"), ("all_t1", "wait"), ("all_t1", "stream"),
                                      ("all_t3", "stream"), ("mixed_per_sequence", "lazy")])
def test_degenerate_tier_mixes(mix, mode):
    """Plans at the edges: every unprotected position compressed, evicted or offloaded (list F, or list Q, then holds
    next to nothing: some workgroups have no tile at all), and a batch whose sequences each sit at a different edge.
    Outputs and scores against the oracle over three decode steps, then everything that can return goes back to T0."""
    from gpu_common import assert_out_close, assert_scores_close
    cfg = small_config(n_layers=2, batch=3, n_q_heads=10, n_kv_heads=2, head_dim=128, kv_dtype="bf16", context=390,
                       decode_steps=3, sigma=1.0)
    p = _pair(cfg, prefetch_mode=mode)
    n = cfg.context
    tiers = np.zeros((cfg.batch, n), np.uint8)
    inner = slice(2, n - 3)
    if mix == "mixed_per_sequence":
        tiers[0, inner], tiers[1, inner], tiers[2, inner] = 2, 3, 1
    else:
        tiers[:, inner] = {"all_t2": 2, "all_t3": 3, "all_t1": 1}[mix]
    p.force_tiers(tiers)
    calls = 0
    for step in range(cfg.decode_steps):
        for l in range(cfg.n_layers):
            p.append(l, *p.wl.step_kv(step, l))
            got, ref = p.attend(l, p.wl.step_q(step, l))
            calls += 1
            assert_out_close(got, ref, "bf16", f"{mix} step {step} layer {l}")
    n += cfg.decode_steps
    assert_scores_close(p.gpu.get_scores(), p.orc.score, n, _mass(cfg, calls))
    back = np.zeros((cfg.batch, n), np.uint8)
    back[:, :cfg.context] = np.where(tiers == 3, 3, 0)
    p.force_tiers(back)
    for l in range(cfg.n_layers):
        got, ref = p.attend(l, p.wl.step_q(0, l))
        assert_out_close(got, ref, "bf16", f"{mix} back in T0, layer {l}")
    st = p.gpu.get_stats()
    assert st["tier_count"][1] == 0 and st["tier_count"][2] == 0
    p.close()


def test_streamed_t1_store_rewritten_when_t1_rows_are_only_evicted():
    """Streamed T1, a plan whose only change is that two thirds of T1 are evicted: no row has to be read back through
    the frames for a mover, but the store is still rewritten packed (its stale rows would outweigh what is left);
    then a plan that empties T1 altogether.  Outputs, scores and every remaining T1 row's bits in the pinned store."""
    from gpu_common import assert_out_close, assert_scores_close
    cfg = small_config(n_layers=3, batch=2, n_q_heads=10, n_kv_heads=2, head_dim=128, kv_dtype="bf16", context=420,
                       decode_steps=4, sigma=1.0)
    p = _pair(cfg, prefetch_mode="stream")
    rng = np.random.default_rng(41)
    n = cfg.context
    tiers = _random_tiers(rng, cfg.batch, n, frac=(0.3, 0.5, 0.2, 0.0))
    p.force_tiers(tiers)
    calls = 0

    def step_all(step):
        nonlocal calls
        for l in range(cfg.n_layers):
            p.append(l, *p.wl.step_kv(step, l))
            got, ref = p.attend(l, p.wl.step_q(step, l))
            calls += 1
            assert_out_close(got, ref, "bf16", f"step {step} layer {l}")

    step_all(0)
    t1 = np.argwhere(tiers == 1)
    drop = t1[rng.random(len(t1)) < 0.67]
    tiers2 = np.zeros((cfg.batch, n + 1), np.uint8); tiers2[:, :n] = tiers
    tiers2[drop[:, 0], drop[:, 1]] = 3
    p.force_tiers(tiers2)
    st = p.gpu.get_stats()
    assert st["n_repack"] == 1 and st["host_rows_used"] == st["tier_count"][1] == int((tiers2 == 1).sum())
    for pos in np.nonzero(tiers2[1] == 1)[0]:
        row = (p.gpu.get_row(2, 1, 0, int(pos), 0).astype(np.uint32) << 16).view(np.float32)
        assert np.array_equal(row.astype(np.float64), p.orc.K[2][1, 0, int(pos)]), pos
    step_all(1)
    tiers3 = np.zeros((cfg.batch, n + 2), np.uint8); tiers3[:, :n + 1] = np.where(tiers2 == 1, 3, tiers2)
    p.force_tiers(tiers3)
    st = p.gpu.get_stats()
    assert st["n_repack"] == 2 and st["host_rows_used"] == 0 and st["tier_count"][1] == 0
    step_all(2)
    assert_scores_close(p.gpu.get_scores(), p.orc.score, n + 3, _mass(cfg, calls))
    p.close()


def test_streamed_t1_with_a_sequence_that_has_no_t1_rows():
    """Streamed T1 where one sequence keeps nothing in T1 (its share of the second attention launch has no tiles and
    must contribute neutral partials) and the other keeps nothing in T2."""
    from gpu_common import assert_out_close, assert_scores_close
    cfg = small_config(n_layers=3, batch=2, n_q_heads=10, n_kv_heads=2, head_dim=128, kv_dtype="bf16", context=400,
                       decode_steps=3, sigma=1.0)
    p = _pair(cfg, prefetch_mode="stream")
    rng = np.random.default_rng(11)
    n = cfg.context
    tiers = np.zeros((cfg.batch, n), np.uint8)
    tiers[0] = _random_tiers(rng, 1, n, frac=(0.3, 0.7, 0.0, 0.0))[0]
    tiers[1] = _random_tiers(rng, 1, n, frac=(0.4, 0.0, 0.5, 0.1))[0]
    p.force_tiers(tiers)
    calls = 0
    for step in range(cfg.decode_steps):
        for l in range(cfg.n_layers):
            p.append(l, *p.wl.step_kv(step, l))
            got, ref = p.attend(l, p.wl.step_q(step, l))
            calls += 1
            assert_out_close(got, ref, "bf16", f"step {step} layer {l}")
    assert_scores_close(p.gpu.get_scores(), p.orc.score, n + cfg.decode_steps, _mass(cfg, calls))
    # now the first sequence gives up all of T1 as well: the second launch disappears
    t2 = np.zeros((cfg.batch, n + cfg.decode_steps), np.uint8)
    t2[:, :n] = np.where(tiers == 1, 0, tiers)
    p.force_tiers(t2)
    for l in range(cfg.n_layers):
        got, ref = p.attend(l, p.wl.step_q(0, l))
        calls += 1
        assert_out_close(got, ref, "bf16", f"no T1 left, layer {l}")
    assert_scores_close(p.gpu.get_scores(), p.orc.score, n + cfg.decode_steps, _mass(cfg, calls))
    p.close()


def _crafted_rows(D, t2, kv_dtype):
    """Rows [n, D] (binary32 values, all exactly representable in bf16 and, except where noted, binary16) that sit on the
    encoder's edges: exact halves after the division (round-to-nearest-even decides the code), an all-zero row, a zero
    group, an absmax whose binary16 scale underflows to zero or to a subnormal, an absmax that makes the binary32 scale
    subnormal, and a row whose largest element is negative."""
    rows = []
    half = np.array([0.5, 1.5, 2.5, 3.5, 4.5, 5.5, 6.5, -0.5, -1.5, -2.5, -3.5, -4.5, -5.5, -6.5], np.float32)
    if t2 == "int8_row":
        r = np.zeros(D, np.float32); r[0] = 127.0                      # scale exactly 1: x / scale = x
        r[1:15] = half; r[15:19] = [126.5, 125.5, -126.5, -125.5]; r[19] = -127.0
        rows.append(r)
        r = np.zeros(D, np.float32); r[5] = -254.0                     # largest element negative, scale exactly 2
        r[6:20] = 2.0 * half; r[20:24] = [1.0, 3.0, -1.0, -3.0]        # quotients 0.5, 1.5, -0.5, -1.5
        rows.append(r)
        r = np.zeros(D, np.float32); r[D - 1] = 2.0 ** -14             # small scale 2^-14 / 127; quotients 63.5, -63.5, 0.99
        r[0:4] = [2.0 ** -15, -(2.0 ** -15), 2.0 ** -21, 0.0]
        rows.append(r)
        if kv_dtype != "f16":                                          # below binary16's range
            r = np.zeros(D, np.float32); r[3] = 2.0 ** -125            # scale = 2^-125 / 127 is a binary32 subnormal
            r[4:8] = [2.0 ** -126, -(2.0 ** -127), 2.0 ** -130, 2.0 ** -133]
            rows.append(r)
    else:
        r = np.zeros(D, np.float32)
        for g in range(D // 32):
            r[32 * g] = 7.0 if g % 2 == 0 else -7.0                    # scale exactly 1 in every group
            r[32 * g + 1: 32 * g + 15] = half if g % 2 == 0 else -half
        rows.append(r)
        r = np.zeros(D, np.float32)
        r[0:32] = np.arange(-16, 16, dtype=np.float32) * np.float32(0.1875)   # absmax 3: the scale 3/7 is not exact in binary16
        r[32:64] = 0.0                                                 # a zero group beside live ones
        if D > 64:
            r[64] = 2.0 ** -24; r[65] = -(2.0 ** -24); r[66] = 2.0 ** -24   # a/7 < 2^-25: the binary16 scale is zero, codes zero
            r[96] = 2.0 ** -22; r[97] = 2.0 ** -23; r[98] = -(2.0 ** -24); r[99] = 3 * 2.0 ** -24   # scale = 2^-24 (subnormal): codes 4, 2, -1, 3
        else:
            r[32] = 2.0 ** -22; r[33] = 2.0 ** -23; r[34] = -(2.0 ** -24); r[35] = 3 * 2.0 ** -24
        rows.append(r)
        r = np.zeros(D, np.float32); r[::32] = 2.0 ** -24                  # every group underflows: all codes and scales zero
        rows.append(r)
        r = np.zeros(D, np.float32); r[0] = 14.0; r[1:15] = 2.0 * half     # scale exactly 2: quotients on halves again
        r[40] = -3.5; r[41] = 1.75; r[42] = -0.25                          # scale 0.5 exactly: 3.5/7
        rows.append(r)
    rows.append(np.zeros(D, np.float32))                                   # absmax 0
    return np.stack(rows)


@pytest.mark.parametrize("mode", ["wait", "stream"])
@pytest.mark.parametrize("t2", ["int8_row", "int4_g32"])
@pytest.mark.parametrize("kv_dtype,D", [("bf16", 128), ("f16", 128), ("f32", 64)])
def test_t2_codec_on_crafted_rows(kv_dtype, D, t2, mode):
    """The encoder's edge cases, bit for bit against the oracle's binary32 definition: crafted rows (see _crafted_rows)
    planted as the K and the V rows of chosen positions, compressed from HBM and (second plan) from a T1 copy, read
    back code by code and scale by scale; then attention through them, and their promoted values after T2 -> T0."""
    from gpu_common import assert_out_close, assert_scores_close, assert_t2_rows_exact, to_f64
    cfg = small_config(n_layers=2, batch=2, n_q_heads=4, n_kv_heads=2, head_dim=D, kv_dtype=kv_dtype, context=96,
                       decode_steps=3, t2_format=t2, sigma=1.0, k_sink=0, k_window=0)
    p = _pair(cfg, prefetch_mode=mode, preload=False)
    crafted = _crafted_rows(D, t2, kv_dtype)
    nc = len(crafted)
    pos_a = [3 + 2 * i for i in range(nc)]            # compressed by the first plan, straight from HBM
    pos_b = [40 + 3 * i for i in range(nc)]           # first to T1, compressed from there by the second plan
    for l in range(cfg.n_layers):
        k, v = p.wl.context_kv(l)
        for i in range(nc):
            row = torch.from_numpy(crafted[i]).to(k.dtype).to(k.device)
            assert torch.equal(row.float().cpu(), torch.from_numpy(crafted[i])), "crafted values must be exact in storage"
            for pos in (pos_a[i], pos_b[i]):
                k[:, pos, l % 2] = row            # K row of one kv head (the other keeps its random row)
                v[:, pos, 1 - l % 2] = row.flip(0) if t2 == "int8_row" else row
        p.append(l, k.contiguous(), v.contiguous())
    n = cfg.context
    rng = np.random.default_rng(3)
    tiers = _random_tiers(rng, cfg.batch, n, frac=(0.4, 0.3, 0.3, 0.0), protect=(1, 1))
    tiers[:, pos_a] = 2
    tiers[:, pos_b] = 1
    p.force_tiers(tiers)
    assert assert_t2_rows_exact(p, tiers, what="crafted, from HBM") > 0
    calls = 0
    qs = 2.0 ** -5      # the crafted key rows reach 254: small queries keep the logits (and their binary32 rounding) ordinary
    for step in range(2):
        for l in range(cfg.n_layers):
            p.append(l, *p.wl.step_kv(step, l))
            got, ref = p.attend(l, p.wl.step_q(step, l) * qs)
            calls += 1
            assert_out_close(got, ref, kv_dtype, f"crafted step {step} layer {l}")
    n += 2
    tiers2 = np.zeros((cfg.batch, n), np.uint8); tiers2[:, :n - 2] = tiers
    tiers2[:, pos_b] = 2                              # encoded from the staged / streamed T1 copy
    tiers2[:, pos_a] = 0                              # promoted: binary32(code * scale) rounded to the KV dtype
    p.force_tiers(tiers2)
    assert assert_t2_rows_exact(p, tiers2, what="crafted, from T1") > 0
    for pos in pos_a:
        for l in range(cfg.n_layers):
            for kvh in range(cfg.n_kv_heads):
                for which, store in ((0, p.orc.K), (1, p.orc.V)):
                    row = p.gpu.get_row(l, 1, kvh, pos, which)
                    if kv_dtype == "bf16":
                        row = (row.astype(np.uint32) << 16).view(np.float32)
                    elif kv_dtype == "f16":
                        row = row.view(np.float16)
                    assert np.array_equal(row.astype(np.float64), store[l][1, kvh, pos]), (pos, l, kvh, which)
    for l in range(cfg.n_layers):
        p.append(l, *p.wl.step_kv(2, l))
        got, ref = p.attend(l, p.wl.step_q(2, l) * qs)
        calls += 1
        assert_out_close(got, ref, kv_dtype, f"crafted, after the second plan, layer {l}")
    assert_scores_close(p.gpu.get_scores(), p.orc.score, n + 1, _mass(cfg, calls))
    p.close()


@pytest.mark.parametrize("mode", ["wait", "stream"])
def test_sequence_with_no_live_position_gives_zero_output(mode):
    """A forced plan that evicts every position of one sequence: that sequence's output is exactly zero (not 0/0) and
    its scores stay as they were; the other sequence is unaffected."""
    from gpu_common import assert_out_close, assert_scores_close
    cfg = small_config(n_layers=2, batch=2, n_q_heads=10, n_kv_heads=2, head_dim=128, kv_dtype="bf16", context=200,
                       decode_steps=1, sigma=1.0)
    p = _pair(cfg, prefetch_mode=mode)
    n = cfg.context
    for l in range(cfg.n_layers):
        p.attend(l, p.wl.step_q(0, l))
    before = p.gpu.get_scores()[0, :n].copy()
    tiers = np.zeros((cfg.batch, n), np.uint8)
    tiers[0, :] = 3
    tiers[1, 50:120] = 1
    p.force_tiers(tiers)
    for l in range(cfg.n_layers):
        got, ref = p.attend(l, p.wl.step_q(1, l))
        assert np.all(got[0] == 0.0) and np.all(ref[0] == 0.0)
        assert_out_close(got[1:], ref[1:], "bf16", f"layer {l}")
    assert np.array_equal(p.gpu.get_scores()[0, :n], before)
    assert_scores_close(p.gpu.get_scores(), p.orc.score, n, _mass(cfg, 2 * cfg.n_layers))
    p.close()


@pytest.mark.parametrize("kv_dtype,D,Hq,Hkv", [("bf16", 128, 10, 2), ("f32", 64, 8, 2)])
def test_streamed_t1_agrees_with_its_all_t0_twin_to_rounding(kv_dtype, D, Hq, Hkv):
    """The documented exception to Prop. 1's bit identity: in streamed mode the T1 rows of a layer are served by a
    second launch with tiles and splits of its own, so the binary32 summation order depends on the placement.  The
    rows themselves are exact, so the run with rows in T1 and its twin with the same rows left in T0 must still
    agree to rounding: outputs within 1e-5 of each head's max-norm and scores within 1e-5 relative, two hundred times
    inside the method's own tolerances (the resident modes are held to bit equality by
    test_prop1_t1_placement_is_bit_invisible)."""
    from gpu_common import Pair
    cfg = small_config(n_layers=3, batch=2, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, kv_dtype=kv_dtype,
                       context=900, decode_steps=6, sigma=1.2)
    rng = np.random.default_rng(9)
    n = cfg.context
    tiers = _random_tiers(rng, cfg.batch, n, frac=(0.3, 0.5, 0.15, 0.05))
    twin = np.where(tiers == 1, 0, tiers).astype(np.uint8)
    outs = []
    for tt in (tiers, twin):
        print(f"[case] stream vs twin {kv_dtype} t1_rows={(tt == 1).sum()}", flush=True)
        p = Pair(cfg, prefetch_mode="stream")
        p.gpu.set_tiers(tt)
        p.gpu.migrate()
        res = []
        for step in range(cfg.decode_steps):
            for l in range(cfg.n_layers):
                k, v = p.wl.step_kv(step, l)
                p.gpu.append(l, k, v)
                res.append(p.gpu.attend_and_score(l, p.wl.step_q(step, l)).double().cpu().numpy())
        outs.append((np.stack(res), p.gpu.get_scores()[:, :n + cfg.decode_steps].astype(np.float64)))
        p.close()
    (o1, s1), (o0, s0) = outs
    scale = np.maximum(np.abs(o0).max(axis=-1, keepdims=True), 1e-6)
    assert (np.abs(o1 - o0) / scale).max() <= 1e-5
    total = cfg.decode_steps / 1.0          # Eq. 1's scale: each step adds one unit per sequence
    assert np.all(np.abs(s1 - s0) <= 1e-5 * s0 + 1e-9 * total / n)
