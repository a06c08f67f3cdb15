"""Pins for the CPU oracle: each test ties a piece of oracle/ to something the paper or the
mathematics fixes independently of the oracle's own code (closed forms, invariants, a library
routine on a special case, brute force on tiny inputs).  None of these touches the GPU path."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import tkv_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(1234)


# ---------------------------------------------------------------- attention: closed forms
def test_softmax_mass_is_one():
    K = rng.normal(size=(37, 16)) * 3
    q = rng.normal(size=16)
    live = rng.random(37) > 0.3
    a = O.attention_weights(q, K, live, 0.25)
    assert abs(a.sum() - 1.0) < 1e-14
    assert np.all(a[~live] == 0.0) and np.all(a[live] > 0.0)


def test_identical_keys_give_uniform_weights_and_mean_value():
    K = np.tile(rng.normal(size=(1, 8)), (11, 1))
    V = rng.normal(size=(11, 8))
    o, a = O.attend_head(rng.normal(size=8), K, V, np.ones(11, bool), 0.3)
    assert np.allclose(a, 1.0 / 11, atol=1e-15)
    assert np.allclose(o, V.mean(axis=0), atol=1e-14)


def test_two_token_case_is_a_sigmoid():
    # x_1 = a * scale, x_2 = 0  =>  alpha_1 = 1 / (1 + exp(-a * scale))
    a_, scale = 2.7, 1.0 / math.sqrt(4)
    q = np.array([a_, 0, 0, 0.0])
    K = np.array([[1.0, 0, 0, 0], [0, 0, 0, 0]])
    V = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0]])
    o, a = O.attend_head(q, K, V, np.ones(2, bool), scale)
    s = 1.0 / (1.0 + math.exp(-a_ * scale))
    assert abs(a[0] - s) < 1e-15 and abs(a[1] - (1 - s)) < 1e-15
    assert np.allclose(o, [s, 1 - s, 0, 0], atol=1e-15)


def test_basis_probe_pins_operand_roles():
    # keys = c_i * e_i, values = e_{pi(i)}: logits are q_i * c_i * scale and the output is a
    # permuted softmax of them.  A transposed operand, a swapped K/V or a dropped scale fails.
    d = 6
    c = np.array([0.5, -1.0, 2.0, 1.5, -0.25, 3.0])
    pi = np.array([3, 0, 5, 1, 4, 2])
    K = np.diag(c)
    V = np.eye(d)[pi]
    q = rng.normal(size=d)
    scale = 0.37
    x = q * c * scale
    want_a = np.exp(x) / np.exp(x).sum()
    o, a = O.attend_head(q, K, V, np.ones(d, bool), scale)
    assert np.allclose(a, want_a, atol=1e-15)
    want_o = np.zeros(d)
    want_o[pi] = want_a
    assert np.allclose(o, want_o, atol=1e-15)


def test_gqa_head_mapping_is_h_div_G():
    B, Hq, Hkv, n, d = 1, 6, 2, 5, 4
    K = rng.normal(size=(B, Hkv, n, d))
    V = np.zeros((B, Hkv, n, d))
    V[:, 0] = 1.0
    V[:, 1] = 2.0
    q = rng.normal(size=(B, Hq, d))
    out, _ = O.attend_gqa(q, K, V, np.ones((B, n), bool), 0.5)
    assert np.allclose(out[0, :3], 1.0) and np.allclose(out[0, 3:], 2.0)


def test_full_cache_matches_float64_sdpa():
    # special case with no eviction: a library routine (torch SDPA, float64, K/V expanded over the group)
    B, Hq, Hkv, n, d = 2, 8, 2, 67, 32
    G = Hq // Hkv
    K = rng.normal(size=(B, Hkv, n, d)) * np.exp(rng.normal(size=(B, 1, n, 1)))
    V = rng.normal(size=(B, Hkv, n, d))
    q = rng.normal(size=(B, Hq, d))
    out, alpha = O.attend_gqa(q, K, V, np.ones((B, n), bool), 1.0 / math.sqrt(d))
    tq = torch.from_numpy(q)[:, :, None, :]
    tk = torch.from_numpy(K).repeat_interleave(G, dim=1)
    tv = torch.from_numpy(V).repeat_interleave(G, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, :, 0, :].numpy()
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)
    assert np.allclose(alpha.sum(-1), 1.0, atol=1e-13)


# ---------------------------------------------------------------- Eq. 3, Eq. 4, Prop. 1
def test_eviction_is_softmax_over_survivors_eq3():
    n, d = 40, 8
    K, V, q = rng.normal(size=(n, d)) * 2, rng.normal(size=(n, d)), rng.normal(size=d)
    live = np.ones(n, bool)
    live[rng.choice(n, 9, replace=False)] = False
    o, a = O.attend_head(q, K, V, live, 0.35)
    o_ref, a_ref = O.attend_head(q, K[live], V[live], np.ones(live.sum(), bool), 0.35)
    assert np.allclose(o, o_ref, atol=1e-15) and np.allclose(a[live], a_ref, atol=1e-16)
    # and it is the full softmax renormalised by the surviving mass (Z'/Z)
    _, a_full = O.attend_head(q, K, V, np.ones(n, bool), 0.35)
    assert np.allclose(a[live], a_full[live] / a_full[live].sum(), atol=1e-15)


def test_error_bound_eq4_holds():
    for trial in range(50):
        n, d = 60, 16
        K, V, q = rng.normal(size=(n, d)) * 2, rng.normal(size=(n, d)) * 3, rng.normal(size=d)
        ev = np.zeros(n, bool)
        ev[rng.choice(n, rng.integers(1, 20), replace=False)] = True
        o_full, a_full = O.attend_head(q, K, V, np.ones(n, bool), 0.25)
        o_hat, _ = O.attend_head(q, K, V, ~ev, 0.25)
        assert np.linalg.norm(o_hat - o_full) <= O.eviction_error_bound(a_full, V, ev) + 1e-14


def _mk_cache(L=2, B=2, Hq=4, Hkv=2, d=16, n=48, **kw):
    c = O.OracleCache(L, B, Hq, Hkv, d, max_tokens=n + 8, kv_dtype="f32", k_sink=2, k_window=4, **kw)
    data = {}
    for l in range(L):
        k = rng.normal(size=(B, n, Hkv, d)).astype(np.float32)
        v = rng.normal(size=(B, n, Hkv, d)).astype(np.float32)
        c.append(l, k, v)
        data[l] = (k, v)
    return c, data


def test_prop1_offloading_is_exact():
    c1, data = _mk_cache()
    c2 = O.OracleCache(2, 2, 4, 2, 16, max_tokens=56, kv_dtype="f32", k_sink=2, k_window=4)
    for l, (k, v) in data.items():
        c2.append(l, k, v)
    tiers = np.zeros((2, 48), np.uint8)
    tiers[:, 5:40:2] = O.T1
    tiers[:, 7] = O.T3
    all_t0 = np.where(tiers == O.T1, O.T0, tiers)
    c1.set_tiers(tiers); c1.migrate()
    c2.set_tiers(all_t0); c2.migrate()
    for l in range(2):
        q = rng.normal(size=(2, 4, 16))
        assert np.array_equal(c1.attend_and_score(l, q), c2.attend_and_score(l, q))
    assert np.array_equal(c1.score, c2.score)


def test_score_total_closed_form():
    # each head's weights sum to 1 over the live set, so every layer call adds Hq * score_scale
    # to the sequence's total; with score_scale = 1/(L*Hq) a step adds exactly 1 (Eq. 1).
    c, _ = _mk_cache()
    tiers = np.zeros((2, 48), np.uint8)
    tiers[:, 10:20] = O.T3
    tiers[:, 20:30] = O.T2
    c.set_tiers(tiers); c.migrate()
    steps = 3
    for _ in range(steps):
        for l in range(2):
            c.attend_and_score(l, rng.normal(size=(2, 4, 16)))
    assert np.allclose(c.score.sum(axis=1), steps, atol=1e-12)
    assert np.all(c.score[:, 10:20] == 0.0)
    c2, _ = _mk_cache(score_scale=1.0)
    c2.attend_and_score(0, rng.normal(size=(2, 4, 16)))
    assert np.allclose(c2.score.sum(axis=1), 4.0, atol=1e-12)


def test_score_uniform_case():
    c = O.OracleCache(1, 1, 4, 2, 8, max_tokens=10, kv_dtype="f32", score_scale=1.0)
    k = np.tile(rng.normal(size=(1, 1, 2, 8)), (1, 10, 1, 1)).astype(np.float32)
    c.append(0, k, k)
    c.attend_and_score(0, rng.normal(size=(1, 4, 8)))
    assert np.allclose(c.score[0], 4.0 / 10, atol=1e-15)


# ---------------------------------------------------------------- storage rounding, codec
def test_bf16_rounding_matches_library_and_ties_to_even():
    x = (rng.normal(size=5000) * np.exp(rng.normal(size=5000) * 4)).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(O.round_to_bf16(x), ref)
    ties = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8), 1 + 2.0 ** -8 + 2.0 ** -20], np.float32)
    assert np.array_equal(O.round_to_bf16(ties), np.array([1.0, 1 + 2.0 ** -6, -1.0, 1 + 2.0 ** -7], np.float32))


def test_int8_hand_example_ties_to_even():
    x = np.zeros(16, np.float32)
    x[:7] = [127.0, -63.5, 0.5, 1.5, 2.5, -126.6, 3.49]
    codes, scale = O.quant_int8_row(x)
    assert scale == np.float32(1.0)
    assert list(codes[:7]) == [127, -64, 0, 2, 2, -127, 3]
    assert np.array_equal(O.dequant_int8_row(codes, scale), codes.astype(np.float64))


def test_int8_properties():
    x = (rng.normal(size=(200, 128)) * np.exp(rng.normal(size=(200, 1)) * 3)).astype(np.float32)
    x[17] = 0.0
    codes, scale = O.quant_int8_row(x)
    xh = O.dequant_int8_row(codes, scale)
    assert codes.dtype == np.int8 and np.abs(codes.astype(int)).max() <= 127
    assert scale[17] == 0 and np.all(codes[17] == 0) and np.all(xh[17] == 0)
    rows = np.arange(200) != 17
    amax = np.argmax(np.abs(x), axis=1)
    assert np.all(np.abs(codes[np.arange(200), amax].astype(int))[rows] == 127)
    assert np.all(np.abs(x - xh)[rows] <= (scale[rows, None].astype(np.float64) * (0.5 + 1e-6)))
    assert np.all(np.sign(codes[rows]) * np.sign(x[rows]) >= 0)


def test_int4_hand_example_and_fp16_scale():
    x = np.zeros(64, np.float32)
    x[:5] = [7.0, 3.5, -2.5, 0.49, -6.6]          # group 0: scale 1
    x[32] = np.float32(7.0 * (1 + 2.0 ** -12))      # group 1: a/7 = 1 + 2^-12 -> binary16 1.0
    x[33] = 0.5
    codes, scale = O.quant_int4_g32(x)
    assert list(scale) == [1.0, 1.0]
    assert list(codes[:5]) == [7, 4, -2, 0, -7]
    assert codes[32] == 7 and codes[33] == 0
    p = O.pack_int4(codes)
    assert p[0] == (7 | (4 << 4)) and p[1] == ((-2 & 0xF) | 0) and p[2] == ((-7 & 0xF))


def test_int4_properties():
    x = (rng.normal(size=(100, 128)) * np.exp(rng.normal(size=(100, 1)) * 2)).astype(np.float32)
    x[3, 32:64] = 0.0
    x[4, :32] = 1e-9                                   # scale underflows binary16 -> zero codes
    codes, scale = O.quant_int4_g32(x)
    assert np.abs(codes.astype(int)).max() <= 7
    assert scale.shape == (100, 4)
    assert np.array_equal(scale, scale.astype(np.float16).astype(np.float32))
    assert np.all(codes[3, 32:64] == 0) and scale[3, 1] == 0
    assert scale[4, 0] == 0 and np.all(codes[4, :32] == 0)
    xh = O.dequant_int4_g32(codes, scale)
    ok = np.repeat(scale > 0, 32, axis=1)
    # |x/scale| can exceed 7 by the binary16 rounding of the scale (clipped), so the bound is
    # scale/2 inside the range plus that rounding slack (2^-11 relative on 7*scale)
    bound = np.repeat(scale, 32, axis=1).astype(np.float64) * (0.5 + 7 * 2.0 ** -11 + 1e-6)
    assert np.all(np.abs(x - xh)[ok] <= bound[ok])


def test_codec_subnormal_scales_by_hand():
    """Edges of the two encoders, expected values worked out by hand.
    int4: a/7 below 2^-25 rounds to a zero binary16 scale (zero codes); a = 2^-22 gives a/7 = 0.571 * 2^-24, which rounds
    to the smallest binary16 subnormal 2^-24, so the codes are x / 2^-24 and the largest element does NOT map to 7.
    int8: a = 2^-125 gives the binary32 subnormal scale rne(2^-125 / 127): 2^-125 / 127 = 132104.06 * 2^-149, i.e.
    the bit pattern 132104; x / scale is then 127 * 2^k (slightly below, the scale having been rounded down...)
    for x = 2^(-125+k): codes 127, 64 (63.5 + eps rounds up), -32, 4."""
    x = np.zeros(64, np.float32)
    x[0:3] = [2.0 ** -24, -(2.0 ** -24), 2.0 ** -24]
    x[32:36] = [2.0 ** -22, 2.0 ** -23, -(2.0 ** -24), 3 * 2.0 ** -24]
    codes, scale = O.quant_int4_g32(x)
    assert list(scale) == [0.0, 2.0 ** -24]
    assert np.all(codes[:32] == 0) and list(codes[32:36]) == [4, 2, -1, 3]
    y = np.zeros(16, np.float32)
    y[3:8] = [2.0 ** -125, 2.0 ** -126, -(2.0 ** -127), 2.0 ** -130, 2.0 ** -133]
    codes, scale = O.quant_int8_row(y)
    assert np.float32(scale).view(np.uint32) == 132104
    assert list(codes[3:8]) == [127, 64, -32, 4, 0]


def test_promotion_value_is_binary32_product_rounded_to_storage():
    codes = np.array([[127, -3, 0, 55]], np.int8)
    scale = np.array([0.0123456789], np.float32)
    got = O.t2_decode_to_storage(codes, scale, "int8_row", "bf16")
    want = torch.from_numpy(codes.astype(np.float32) * scale).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got, want)
    got32 = O.t2_decode_to_storage(codes, scale, "int8_row", "f32")
    assert np.array_equal(got32, codes.astype(np.float32) * scale)
    got16 = O.t2_decode_to_storage(codes, scale, "int8_row", "f16")
    want16 = torch.from_numpy(codes.astype(np.float32) * scale).to(torch.float16).to(torch.float32).numpy()
    assert np.array_equal(got16, want16)
    # binary16 rounding: ties to even, by hand (1 + 2^-11 is halfway between 1 and 1 + 2^-10; 1 + 3*2^-11 between
    # 1 + 2^-10 and 1 + 2^-9), and the largest finite value
    x = np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 65504.0, 2.0 ** -25], np.float32)
    assert np.array_equal(O.round_to_storage(x, "f16"), np.array([1.0, 1.0 + 2.0 ** -9, 65504.0, 0.0], np.float32))


# ---------------------------------------------------------------- tier sizes and ranking
def test_tier_counts_exact_floors():
    for m in [0, 1, 7, 64, 999, 1000, 3964, 16268, 123457]:
        for pol in [(300000, 520000, 150000, 30000), (500000, 300000, 150000, 50000), (333333, 333333, 333333, 1),
                    (1000000, 0, 0, 0), (0, 0, 0, 1000000)]:
            n0, n1, n2, n3 = O.tier_counts(m, pol)
            assert n3 == math.floor(Fraction(pol[3], 10 ** 6) * m)
            assert n2 == math.floor(Fraction(pol[2], 10 ** 6) * m)
            assert n0 == math.floor(Fraction(pol[0], 10 ** 6) * m)
            assert n0 + n1 + n2 + n3 == m and n1 >= 0


def test_tier_counts_against_algorithm1_golden():
    # The fixture holds Algorithm 1's own floors evaluated by hand.  This build expresses the
    # bands as fractions of |U| (f0 = beta*(1-r), f3 = r, no T2): n_evict must agree exactly and
    # n_hbm to within one token (floor(beta*(m - floor(r m))) vs floor(beta (1-r) m)).
    with open(os.path.join(GOLDEN, "alg1_counts.txt")) as f:
        rows = [tuple(int(t) for t in ln.split()) for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 8
    for m, beta, r, n_hbm, n_ddr, n_evict in rows:
        assert n_hbm + n_ddr + n_evict == m
        f3 = r * 10000
        f0 = beta * (100 - r) * 100
        n0, n1, n2, n3 = O.tier_counts(m, (f0, 10 ** 6 - f0 - f3, 0, f3))
        assert n3 == n_evict and n2 == 0
        assert abs(n0 - n_hbm) <= 1 and abs(n1 - n_ddr) <= 1


def test_alg1_rule_reproduces_the_golden_floors_exactly():
    # Algorithm 1's floors, evaluated by hand in the fixture, with r = f3 and beta = f0 / (1 - f3)
    with open(os.path.join(GOLDEN, "alg1_counts.txt")) as f:
        rows = [tuple(int(t) for t in ln.split()) for ln in f if ln.strip() and not ln.startswith("#")]
    for m, beta, r, n_hbm, n_ddr, n_evict in rows:
        f3 = r * 10000
        f0 = beta * (100 - r) * 100
        assert O.tier_counts_alg1(m, (f0, 10 ** 6 - f0 - f3, 0, f3)) == (n_hbm, n_ddr, 0, n_evict)


def test_alg1_rule_compounds_and_partitions():
    # event after event on a fixed candidate set the live part shrinks by floor(r * live): the recurrence written
    # out with exact fractions, against the function; the four bands always partition the candidates
    pol = (400000, 350000, 150000, 100000)
    m, ev = 3000, 0
    for _ in range(12):
        n0, n1, n2, n3 = O.tier_counts_alg1(m, pol, ev)
        live = m - ev
        new = math.floor(Fraction(1, 10) * live)
        surv = live - new
        assert n3 == ev + new
        assert n0 == math.floor(Fraction(400000, 900000) * surv) and n2 == math.floor(Fraction(150000, 900000) * surv)
        assert n0 + n1 + n2 + n3 == m and n1 >= 0
        ev = n3
    # 3000 -> 2700 -> 2430 -> 2187 -> 1969 -> 1773 -> 1596 -> 1437 -> 1294 -> 1165 -> 1049 -> 945 -> 851 alive
    assert ev == 3000 - 851
    # no eviction: the rule reduces to plain floors of the fractions; everything evicted: nothing else
    assert O.tier_counts_alg1(1000, (500000, 300000, 200000, 0), 0) == (500, 300, 200, 0)
    assert O.tier_counts_alg1(1000, (0, 0, 0, 1000000), 0) == (0, 0, 0, 1000)
    assert O.tier_counts_alg1(10, (500000, 300000, 150000, 50000), 10) == (0, 0, 0, 10)


def test_alg1_rule_in_the_classifier_evicts_the_lowest_live_scores():
    # two events on 200 candidates with distinct scores: the second event evicts floor(0.1 * 180) = 18 more, and
    # they are the 18 lowest scores among the positions still alive
    rng = np.random.default_rng(3)
    n = 200 + 4 + 8
    s = rng.permutation(n).astype(np.float32) + 1.0
    pol = (450000, 450000, 0, 100000)
    t1 = O.classify_sequence(s, np.zeros(n, np.uint8), n, 0, 4, 8, pol, count_rule=1)
    assert (t1 == 3).sum() == 20 and (t1 == 0).sum() == 90 + 12 and (t1 == 1).sum() == 90
    t2 = O.classify_sequence(s, t1, n, 0, 4, 8, pol, count_rule=1)
    assert (t2 == 3).sum() == 38 and np.all(t2[t1 == 3] == 3)
    cand = np.arange(4, n - 8)
    alive = cand[t1[cand] != 3]
    lowest = alive[np.argsort(s[alive])[:18]]
    assert np.all(t2[lowest] == 3)
    assert (t2 == 0).sum() == 81 + 12 and (t2 == 1).sum() == 81


def test_tier_counts_keep_evicted():
    assert O.tier_counts(100, (500000, 300000, 150000, 50000), n_already_evicted=3) == (50, 30, 15, 5)
    assert O.tier_counts(100, (500000, 300000, 150000, 50000), n_already_evicted=12) == (50, 30, 8, 12)
    assert O.tier_counts(100, (500000, 300000, 150000, 50000), n_already_evicted=25) == (50, 25, 0, 25)
    assert O.tier_counts(100, (500000, 300000, 150000, 50000), n_already_evicted=70) == (30, 0, 0, 70)


def _brute_force_tiers(score32, tier_prev, n, n_prompt, k_sink, k_window, pol):
    """Rank of a candidate = number of candidates with a smaller (live, bits, position) key,
    by O(m^2) counting -- no sort."""
    lo, hi = n_prompt + k_sink, n - k_window
    out = np.zeros(n, np.uint8)
    if hi <= lo:
        return out
    m = hi - lo
    bits = score32.view(np.uint32)
    ev = int(sum(tier_prev[i] == 3 for i in range(lo, hi)))
    n3 = max((pol[3] * m) // 10 ** 6, ev)
    n2 = (pol[2] * m) // 10 ** 6
    n0 = (pol[0] * m) // 10 ** 6
    n1 = m - n0 - n2 - (pol[3] * m) // 10 ** 6
    over = n3 - (pol[3] * m) // 10 ** 6
    for name in ("n2", "n1", "n0"):
        take = min(over, locals()[name])
        if name == "n2": n2 -= take
        elif name == "n1": n1 -= take
        else: n0 -= take
        over -= take
    for i in range(lo, hi):
        ki = (tier_prev[i] != 3, int(bits[i]), i)
        rank = sum((tier_prev[j] != 3, int(bits[j]), j) < ki for j in range(lo, hi))
        out[i] = 3 if rank < n3 else 2 if rank < n3 + n2 else 1 if rank < n3 + n2 + n1 else 0
    return out


@pytest.mark.parametrize("seed", range(6))
def test_classify_matches_brute_force_with_ties_and_evicted(seed):
    r = np.random.default_rng(seed)
    n = int(r.integers(20, 120))
    n_prompt, k_sink, k_window = int(r.integers(0, 5)), int(r.integers(0, 5)), int(r.integers(0, 12))
    score = r.choice(np.array([0.0, 0.125, 0.5, 0.5000001, 1.0, 3.25], np.float32), size=n)  # many ties
    if seed % 2:
        score = (r.random(n) ** 4).astype(np.float32)
    tier_prev = np.zeros(n, np.uint8)
    lo, hi = n_prompt + k_sink, n - k_window
    if hi > lo and seed >= 2:
        ev = r.choice(np.arange(lo, hi), size=min(hi - lo, int(r.integers(1, 15))), replace=False)
        tier_prev[ev] = 3
    pol = [(500000, 300000, 150000, 50000), (300000, 520000, 150000, 30000), (250000, 250000, 250000, 250000)][seed % 3]
    got = O.classify_sequence(score, tier_prev, n, n_prompt, k_sink, k_window, pol)
    want = _brute_force_tiers(score, tier_prev, n, n_prompt, k_sink, k_window, pol)
    assert np.array_equal(got, want)
    # structural facts: protected -> T0, evicted stay evicted, band sizes
    if hi > lo:
        assert np.all(got[:lo] == 0) and np.all(got[hi:] == 0)
        assert np.all(got[tier_prev == 3] == 3)
        n0, n1, n2, n3 = O.tier_counts(hi - lo, pol, int(np.sum(tier_prev[lo:hi] == 3)))
        cand = got[lo:hi]
        assert [(cand == t).sum() for t in range(4)] == [n0, n1, n2, n3]
    else:
        assert np.all(got == 0)


def test_classify_ranks_by_score_and_lower_position_loses_ties():
    # 10 candidates, no protection; scores ascending except a tie between positions 2 and 6
    score = np.array([0.9, 0.1, 0.4, 0.8, 0.2, 0.7, 0.4, 0.3, 0.6, 0.5], np.float32)
    pol = (300000, 300000, 200000, 200000)      # n0=3 n1=3 n2=2 n3=2
    got = O.classify_sequence(score, np.zeros(10, np.uint8), 10, 0, 0, 0, pol)
    # ascending: 1(.1) 4(.2) | 7(.3) 2(.4) | 6(.4) 9(.5) 8(.6) | 5(.7) 3(.8) 0(.9)
    assert list(got) == [0, 3, 2, 0, 3, 0, 1, 2, 1, 1]


def test_compact_lists_partition_and_order():
    tier = rng.integers(0, 4, size=200).astype(np.uint8)
    lists = O.compact_lists(tier, 150)
    allpos = np.concatenate(lists)
    assert sorted(allpos.tolist()) == list(range(150))
    for t, lst in enumerate(lists):
        assert np.all(np.diff(lst) > 0) and np.all(tier[lst] == t)


# ---------------------------------------------------------------- migrate
def test_migrate_round_trips_and_t2_semantics():
    c, data = _mk_cache(L=1, B=1, n=32)
    k0 = c.K[0].copy()
    t = np.zeros((1, 32), np.uint8)
    t[0, 5:15] = O.T1
    c.set_tiers(t); c.migrate()
    assert np.array_equal(c.K[0], k0)
    c.set_tiers(np.zeros((1, 32), np.uint8)); c.migrate()
    assert np.array_equal(c.K[0], k0)
    t2 = np.zeros((1, 32), np.uint8)
    t2[0, 8:12] = O.T2
    c.set_tiers(t2); c.migrate()
    kc, ks, vc, vs = c.t2[0][(0, 9)]
    assert np.array_equal(c.K[0][0, :, 9], O.dequant_int8_row(kc, ks))
    assert not np.array_equal(c.K[0][0, :, 9], k0[0, :, 9])
    kq = c.K[0].copy()
    c.set_tiers(t2); c.migrate()                      # T2 -> T2: codes kept, no re-quantisation
    assert np.array_equal(c.K[0], kq)
    c.set_tiers(np.zeros((1, 32), np.uint8)); c.migrate()   # promotion keeps the lossy value
    assert np.array_equal(c.K[0][0, :, 9].astype(np.float32),
                          (kc.astype(np.float32) * ks[:, None]).astype(np.float32))
    t3 = np.zeros((1, 32), np.uint8)
    t3[0, 20] = O.T3
    c.set_tiers(t3); c.migrate()
    assert np.all(c.K[0][0, :, 20] == 0)
    c.set_tiers(np.zeros((1, 32), np.uint8))
    with pytest.raises(RuntimeError):
        c.migrate()


def test_cache_classify_then_attend_skips_evicted():
    c, _ = _mk_cache(L=1, B=1, n=40)
    c.attend_and_score(0, rng.normal(size=(1, 4, 16)))
    new = c.classify((400000, 300000, 200000, 100000))
    c.migrate()
    s_before = c.score.copy()
    c.attend_and_score(0, rng.normal(size=(1, 4, 16)))
    ev = new[0, :40] == O.T3
    assert ev.sum() == (40 - 6) // 10
    assert np.array_equal(c.score[0, :40][ev], s_before[0, :40][ev])
    assert np.all(c.score[0, :40][~ev] > s_before[0, :40][~ev])


# ---------------------------------------------------------------- value-aware scorer (scoring ablation)
def test_vatp_hand_worked_case():
    # one head, two positions with the same key: weights 1/2 and 1/2; value rows (3, 4) and (0, 2) have
    # norms 5 and 2, so the increments are 2.5 and 1 (score_scale 1)
    c = O.OracleCache(1, 1, 1, 1, 2, max_tokens=4, kv_dtype="f32", score_scale=1.0, scorer="vatp", k_sink=0, k_window=0)
    k = np.array([[[[1.0, 0.0]], [[1.0, 0.0]]]], np.float32)          # [B=1, n=2, Hkv=1, d=2]
    v = np.array([[[[3.0, 4.0]], [[0.0, 2.0]]]], np.float32)
    c.append(0, k, v)
    c.attend_and_score(0, np.array([[[0.7, -0.2]]]))
    assert np.allclose(c.score[0, :2], [2.5, 1.0], atol=1e-15)


def test_vatp_with_unit_value_rows_is_the_attention_score():
    ca = O.OracleCache(2, 2, 4, 2, 16, max_tokens=40, kv_dtype="f32", score_scale=1.0)
    cv = O.OracleCache(2, 2, 4, 2, 16, max_tokens=40, kv_dtype="f32", score_scale=1.0, scorer="vatp")
    for l in range(2):
        k = rng.normal(size=(2, 30, 2, 16))
        v = rng.normal(size=(2, 30, 2, 16))
        v /= np.linalg.norm(v, axis=-1, keepdims=True)
        ca.append(l, k, v); cv.append(l, k, v)
    for l in range(2):
        q = rng.normal(size=(2, 4, 16))
        assert np.array_equal(ca.attend_and_score(l, q), cv.attend_and_score(l, q))   # outputs do not depend on the scorer
    assert np.allclose(ca.score, cv.score, rtol=1e-13, atol=0)


def test_vatp_scaling_one_value_row_scales_that_positions_increment_only():
    def run(scale_pos7):
        c = O.OracleCache(1, 1, 4, 2, 8, max_tokens=16, kv_dtype="f32", score_scale=0.25, scorer="vatp")
        r = np.random.default_rng(5)
        k = r.normal(size=(1, 12, 2, 8)); v = r.normal(size=(1, 12, 2, 8))
        v[0, 7] *= scale_pos7
        c.append(0, k, v)
        c.attend_and_score(0, r.normal(size=(1, 4, 8)))
        return c.score[0, :12].copy()
    s1, s3 = run(1.0), run(-3.0)
    assert np.allclose(s3[7], 3.0 * s1[7], rtol=1e-13)
    others = np.arange(12) != 7
    assert np.allclose(s3[others], s1[others], rtol=1e-13)          # the weights do not depend on V


def test_vatp_matches_brute_force_loops_with_gqa_and_eviction():
    B, Hq, Hkv, d, n = 2, 6, 2, 4, 9
    G = Hq // Hkv
    r = np.random.default_rng(11)
    c = O.OracleCache(1, B, Hq, Hkv, d, max_tokens=n, kv_dtype="f32", score_scale=0.5, scorer="vatp", k_sink=0, k_window=0)
    k = r.normal(size=(B, n, Hkv, d)); v = r.normal(size=(B, n, Hkv, d))
    c.append(0, k, v)
    tiers = np.zeros((B, n), np.uint8); tiers[:, 2] = O.T3; tiers[1, 5] = O.T3
    c.set_tiers(tiers); c.migrate()
    q = r.normal(size=(B, Hq, d))
    c.attend_and_score(0, q)
    for b in range(B):
        want = [0.0] * n
        for h in range(Hq):
            kvh = h // G
            live = [i for i in range(n) if tiers[b, i] != O.T3]
            x = {i: sum(q[b, h, e] * k[b, i, kvh, e] for e in range(d)) / math.sqrt(d) for i in live}
            z = sum(math.exp(x[i]) for i in live)
            for i in live:
                want[i] += 0.5 * (math.exp(x[i]) / z) * math.sqrt(sum(v[b, i, kvh, e] ** 2 for e in range(d)))
        assert np.allclose(c.score[b], want, rtol=1e-12, atol=1e-15)
    assert c.score[0, 2] == 0.0 and c.score[1, 5] == 0.0


def test_vatp_norm_is_the_appended_rows_and_survives_compression():
    # a row that goes to T2 keeps the norm it was appended with (this build's reading)
    c = O.OracleCache(1, 1, 2, 1, 8, max_tokens=8, kv_dtype="bf16", score_scale=1.0, scorer="vatp", k_sink=0, k_window=0)
    r = np.random.default_rng(3)
    k = O.round_to_bf16(r.normal(size=(1, 6, 1, 8)).astype(np.float32)); v = O.round_to_bf16(r.normal(size=(1, 6, 1, 8)).astype(np.float32))
    c.append(0, k, v)
    before = c.vnorm[0].copy()
    tiers = np.zeros((1, 6), np.uint8); tiers[0, 1] = O.T2
    c.set_tiers(tiers); c.migrate()
    assert np.array_equal(c.vnorm[0], before)
    assert np.allclose(before[0, 0, :6], np.linalg.norm(v[0, :, 0].astype(np.float64), axis=-1), rtol=1e-15)


# ---------------------------------------------------------------- redundancy-penalised scorers (scoring ablation)
def test_key_redundancy_by_hand():
    # rows: e1, 2*e1 (cosine 1 with its neighbour), e2 (cosine 0), -e2 (cosine -1 -> clamped to 0),
    # (3, 4) after (0, -1): cosine -0.8 -> 0; (4, 3) after (3, 4): 24/25; a zero row and the row after it: 0
    K = np.array([[1, 0], [2, 0], [0, 1], [0, -1], [3, 4], [4, 3], [0, 0], [1, 1]], np.float64)
    rho = O.key_redundancy(K)
    assert np.allclose(rho, [0, 1, 0, 0, 0, 24 / 25, 0, 0], atol=1e-15)
    # with the row in front of the first one given: cosine of (1, 0) and (1, 1) is 1/sqrt(2)
    rho2 = O.key_redundancy(K, k_before=np.array([1.0, 1.0]))
    assert np.isclose(rho2[0], 1 / math.sqrt(2), rtol=1e-15) and np.allclose(rho2[1:], rho[1:])


def test_key_redundancy_matches_brute_force_and_ignores_row_scale():
    r = np.random.default_rng(17)
    K = r.normal(size=(2, 3, 11, 6))
    rho = O.key_redundancy(K)
    for b in range(2):
        for h in range(3):
            for i in range(11):
                if i == 0:
                    want = 0.0
                else:
                    dot = sum(K[b, h, i, e] * K[b, h, i - 1, e] for e in range(6))
                    na = math.sqrt(sum(K[b, h, i, e] ** 2 for e in range(6))); nb = math.sqrt(sum(K[b, h, i - 1, e] ** 2 for e in range(6)))
                    want = max(0.0, dot / (na * nb))
                assert abs(rho[b, h, i] - want) < 1e-14
    K2 = K * r.uniform(0.1, 9.0, size=K.shape[:-1] + (1,))          # positive factor per row: cosines unchanged
    assert np.allclose(O.key_redundancy(K2), rho, rtol=1e-12, atol=1e-15)
    assert rho.min() >= 0.0 and rho.max() <= 1.0 + 1e-15


def test_redundancy_scorer_hand_worked_case():
    # one head, three positions with equal logits (weights 1/3 each); redundancies 0, 1, 0.5; weight 0.6:
    # increment_i = 1/3 - 0.6 * rho_i / 3  ->  1/3, 2/15, 7/30
    alpha = np.full((1, 1, 3), 1 / 3)
    rho = np.array([[[0.0, 1.0, 0.5]]])
    live = np.ones((1, 3), bool)
    inc = O.score_increment_redundancy(alpha, rho, live, 1.0, 0.6)
    assert np.allclose(inc[0], [1 / 3, 2 / 15, 7 / 30], atol=1e-15)
    # the combined scorer with value norms 3, 1, 2: 1 - 0, 1/3 - 0.2, 2/3 - 0.1
    inc = O.score_increment_redundancy(alpha, rho, live, 1.0, 0.6, vnorm=np.array([[[3.0, 1.0, 2.0]]]))
    assert np.allclose(inc[0], [1.0, 1 / 3 - 0.2, 2 / 3 - 0.1], atol=1e-15)
    # an evicted position receives nothing, and the others' penalty is spread over the two that are left
    live = np.array([[True, False, True]])
    alpha = np.array([[[0.5, 0.0, 0.5]]])
    inc = O.score_increment_redundancy(alpha, rho, live, 2.0, 0.6)
    assert np.allclose(inc[0], [2 * 0.5, 0.0, 2 * (0.5 - 0.6 * 0.5 / 2)], atol=1e-15)


def test_redundancy_scorer_reduces_to_the_plain_ones_and_has_the_closed_form_mass():
    r = np.random.default_rng(23)
    B, Hq, Hkv, n = 2, 6, 2, 13
    x = r.normal(size=(B, Hq, n))
    live = r.random((B, n)) < 0.8
    live[:, 0] = True
    a = np.where(live[:, None, :], np.exp(x), 0.0)
    alpha = a / a.sum(-1, keepdims=True)
    rho = r.random((B, Hkv, n)); vn = r.random((B, Hkv, n)) + 0.5
    # weight 0: Eq. 1, and the value-aware scorer
    assert np.allclose(O.score_increment_redundancy(alpha, rho, live, 0.25, 0.0), O.score_increment(alpha, 0.25), rtol=1e-14, atol=0)
    assert np.allclose(O.score_increment_redundancy(alpha, rho, live, 0.25, 0.0, vnorm=vn), O.score_increment_vatp(alpha, vn, 0.25), rtol=1e-14, atol=0)
    # total added per sequence: score_scale * (Hq - weight * G * sum over kv heads of the mean redundancy of the live positions)
    G = Hq // Hkv
    inc = O.score_increment_redundancy(alpha, rho, live, 0.25, 0.7)
    for b in range(B):
        mean_rho = sum(rho[b, h][live[b]].mean() for h in range(Hkv))
        assert np.isclose(inc[b].sum(), 0.25 * (Hq - 0.7 * G * mean_rho), rtol=1e-13)
    assert np.all(inc[~live] == 0.0)


def test_redundancy_cache_appending_in_pieces_is_appending_at_once():
    # the neighbour of a piece's first row is the last row appended before it, as appended -- even if that
    # position has been compressed or evicted in the meantime
    r = np.random.default_rng(29)
    k = O.round_to_bf16(r.normal(size=(2, 10, 2, 8)).astype(np.float32)); v = O.round_to_bf16(r.normal(size=(2, 10, 2, 8)).astype(np.float32))
    c1 = O.OracleCache(1, 2, 4, 2, 8, max_tokens=16, kv_dtype="bf16", scorer="redundancy", k_sink=0, k_window=0)
    c1.append(0, k, v)
    c2 = O.OracleCache(1, 2, 4, 2, 8, max_tokens=16, kv_dtype="bf16", scorer="combined", k_sink=0, k_window=0)
    c2.append(0, k[:, :4], v[:, :4])
    tiers = np.zeros((2, 4), np.uint8); tiers[0, 3] = O.T3; tiers[1, 3] = O.T2
    c2.set_tiers(tiers); c2.migrate()
    c2.append(0, k[:, 4:9], v[:, 4:9]); c2.append(0, k[:, 9:], v[:, 9:])
    assert np.array_equal(c1.rho[0], c2.rho[0])
    assert np.allclose(c1.rho[0][:, :, :10], O.key_redundancy(k.transpose(0, 2, 1, 3).astype(np.float64)), rtol=0, atol=0)


def test_score_order_is_the_order_of_the_values():
    r = np.random.default_rng(31)
    vals = np.concatenate([r.normal(size=300) * 10.0 ** r.integers(-30, 5, size=300), [0.0, -0.0, 1e-45, -1e-45, 3.0e38, -3.0e38]]).astype(np.float32)
    bits = vals.view(np.uint32)
    keys = [O.score_order(int(u)) for u in bits]
    order = sorted(range(len(vals)), key=lambda i: keys[i])
    sorted_vals = vals[order].astype(np.float64)
    assert np.all(np.diff(sorted_vals) >= 0.0)
    assert O.score_order(0x80000000) + 1 == O.score_order(0x00000000)          # -0 directly below +0
    # non-negative scores (Eq. 1) rank exactly as their bit patterns do
    nn = np.abs(vals).view(np.uint32)
    assert sorted(range(len(nn)), key=lambda i: (O.score_order(int(nn[i])), i)) == sorted(range(len(nn)), key=lambda i: (int(nn[i]), i))


def test_classify_with_scores_below_zero_matches_a_plain_sort():
    r = np.random.default_rng(37)
    n = 60
    score = (r.normal(size=n) * 0.1).astype(np.float32)
    score[10] = score[20]                                             # a tie: the lower position ranks lower
    tier_prev = np.zeros(n, np.uint8); tier_prev[[5, 6]] = O.T3
    ppm = (300_000, 400_000, 200_000, 100_000)
    got = O.classify_sequence(score, tier_prev, n, 0, 2, 8, ppm)
    lo, hi = 2, n - 8
    m = hi - lo
    n0, n1, n2, n3 = O.tier_counts(m, ppm, 2)
    cand = sorted(range(lo, hi), key=lambda i: (tier_prev[i] != O.T3, float(score[i]), i))
    want = np.zeros(n, np.uint8)
    for rank, i in enumerate(cand):
        want[i] = O.T3 if rank < n3 else O.T2 if rank < n3 + n2 else O.T1 if rank < n3 + n2 + n1 else O.T0
    assert np.array_equal(got, want)
    assert (got[[5, 6]] == O.T3).all()


# ---------------------------------------------------------------- multi-token queries (causal chunk)
def test_chunk_of_one_is_the_single_token_call():
    c1, data = _mk_cache()
    c2 = O.OracleCache(2, 2, 4, 2, 16, max_tokens=56, kv_dtype="f32", k_sink=2, k_window=4)
    for l, (k, v) in data.items():
        c2.append(l, k, v)
    q = rng.normal(size=(2, 4, 16))
    assert np.array_equal(c1.attend_and_score(0, q), c2.attend_and_score_chunk(0, q[:, None])[:, 0])
    assert np.array_equal(c1.score, c2.score)


def test_chunk_equals_token_by_token_decode():
    # T tokens appended one at a time, each attended right after its append, against the same tokens appended
    # first and attended as one causal chunk: outputs and scores must be the same numbers
    B, Hq, Hkv, d, n0, T = 2, 4, 2, 8, 20, 5
    r = np.random.default_rng(21)
    k0, v0 = r.normal(size=(B, n0, Hkv, d)), r.normal(size=(B, n0, Hkv, d))
    kn, vn = r.normal(size=(B, T, Hkv, d)), r.normal(size=(B, T, Hkv, d))
    q = r.normal(size=(B, T, Hq, d))
    tiers = np.zeros((B, n0), np.uint8); tiers[:, 3] = O.T3; tiers[0, 7] = O.T2; tiers[1, 9] = O.T1
    def fresh():
        c = O.OracleCache(1, B, Hq, Hkv, d, max_tokens=n0 + T, kv_dtype="f32", score_scale=1.0, k_sink=0, k_window=0)
        c.append(0, k0, v0)
        c.set_tiers(tiers); c.migrate()
        return c
    a = fresh()
    outs = []
    for j in range(T):
        a.append(0, kn[:, j:j + 1], vn[:, j:j + 1])
        outs.append(a.attend_and_score(0, q[:, j]))
    b = fresh()
    b.append(0, kn, vn)
    got = b.attend_and_score_chunk(0, q)
    assert np.array_equal(got, np.stack(outs, axis=1))
    assert np.array_equal(a.score, b.score)


def test_chunk_matches_float64_sdpa_with_a_causal_mask():
    B, Hq, Hkv, d, n, T = 2, 6, 2, 16, 33, 7
    r = np.random.default_rng(22)
    c = O.OracleCache(1, B, Hq, Hkv, d, max_tokens=n, kv_dtype="f32", score_scale=1.0)
    k, v = r.normal(size=(B, n, Hkv, d)), r.normal(size=(B, n, Hkv, d))
    c.append(0, k, v)
    q = r.normal(size=(B, T, Hq, d))
    got = c.attend_and_score_chunk(0, q)
    G = Hq // Hkv
    tq = torch.from_numpy(q).permute(0, 2, 1, 3)                                   # [B, Hq, T, d]
    tk = torch.from_numpy(k).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)       # [B, Hq, n, d]
    tv = torch.from_numpy(v).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
    mask = torch.zeros((T, n), dtype=torch.bool)
    for j in range(T):
        mask[j, : n - T + j + 1] = True
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask).permute(0, 2, 1, 3).numpy()
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)
    # every query adds one unit of weight per head; the last position is seen by the last query alone
    assert np.allclose(c.score.sum(axis=1), T * Hq, rtol=1e-12)
    assert np.all(c.score[:, n - 1] < Hq)
