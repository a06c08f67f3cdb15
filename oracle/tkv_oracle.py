"""CPU oracle for tiered-KV decode attention ("Not All Thoughts Need HBM", Sec. 3).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain, obviously-correct
definition of what the GPU hot path computes.  It is imported by tests, by the
smoke check and by the benchmark's CPU-baseline leg -- never by the product
path, and it imports nothing from the product package.

Everything floating point is float64 (numpy), except where the method itself
fixes a precision:
  * the T2 codec (quantise / dequantise) is defined in IEEE-754 binary32 with
    round-to-nearest-even and true division, so that codes and scales are
    bit-reproducible (the paper only says "e.g. 8-bit quantization", Sec. 3.2;
    the concrete formats are this build's reading);
  * the classifier compares the float32 bit patterns of the scores, so that a
    tier assignment is a pure integer function of a float32 score array.

Parity pins (see tests/test_oracle_pins.py): softmax mass, Prop. 1, Eq. 3,
Eq. 4, closed forms for tiny hand-made caches, float64
scaled_dot_product_attention for the full-cache case, brute-force sorting for
ranks, codec round-trip bounds, hand-worked and brute-force cases for the
value-aware scorer.  No function here is "parity unpinned".

Notation follows the paper: L layers, H query heads (Hq), Hkv key/value heads,
G = Hq/Hkv, d head dim, s_i cumulative score of position i, tiers T0..T3,
protected set P, candidates U, Delta = re-tiering interval.
"""
from __future__ import annotations

import numpy as np

T0, T1, T2, T3 = 0, 1, 2, 3
PPM = 1_000_000


# ----------------------------------------------------------------------------
# storage-precision helpers (bf16 rounding written out on the bit pattern)
# ----------------------------------------------------------------------------
def round_to_bf16(x32: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16 (ties to even), returned as float32.

    bfloat16 is the upper 16 bits of binary32; rounding adds 0x7FFF plus the
    lowest kept bit and truncates.  Inputs are finite by contract.
    """
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    u = x32.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x32.shape)


def round_to_fp16(x32: np.ndarray) -> np.ndarray:
    """float32 -> nearest IEEE binary16 (ties to even), returned as float32."""
    return np.asarray(x32, dtype=np.float32).astype(np.float16).astype(np.float32)


def round_to_storage(x32: np.ndarray, kv_dtype: str) -> np.ndarray:
    if kv_dtype == "f32":
        return np.asarray(x32, dtype=np.float32)
    if kv_dtype == "bf16":
        return round_to_bf16(x32)
    if kv_dtype == "f16":
        return round_to_fp16(x32)
    raise ValueError(kv_dtype)


# ----------------------------------------------------------------------------
# attention over a live set  (Eq. 2, Eq. 3)
# ----------------------------------------------------------------------------
def attention_weights(q: np.ndarray, K: np.ndarray, live: np.ndarray, softmax_scale: float) -> np.ndarray:
    """Softmax attention weights of ONE query head over the live positions.

    q [d], K [n, d], live [n] bool.  alpha_i = exp(x_i - max) / sum_live exp(x_j - max),
    x_i = (q . k_i) * softmax_scale, and alpha_i = 0 for evicted positions: the
    softmax is renormalised over the survivors (Eq. 3, with Z').
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    n = K.shape[0]
    alpha = np.zeros(n, dtype=np.float64)
    idx = np.nonzero(live)[0]
    if idx.size == 0:
        return alpha
    x = (K[idx] @ q) * float(softmax_scale)
    e = np.exp(x - x.max())
    alpha[idx] = e / e.sum()
    return alpha


def attend_head(q, K, V, live, softmax_scale):
    """o = sum_i alpha_i v_i for one head (Eq. 2 restricted to survivors, Eq. 3)."""
    alpha = attention_weights(q, K, live, softmax_scale)
    return alpha @ np.asarray(V, dtype=np.float64), alpha


def attend_gqa(q, K, V, live, softmax_scale):
    """All heads of one layer.

    q [B, Hq, d]; K, V [B, Hkv, n, d] (effective values: stored rows for T0/T1,
    dequantised rows for T2); live [B, n] bool.
    Query head h reads kv-head h // G (grouped-query attention).
    Returns out [B, Hq, d] and alpha [B, Hq, n].
    """
    q = np.asarray(q, dtype=np.float64)
    B, Hq, d = q.shape
    Hkv, n = K.shape[1], K.shape[2]
    G = Hq // Hkv
    assert G * Hkv == Hq
    out = np.zeros((B, Hq, d), dtype=np.float64)
    alpha = np.zeros((B, Hq, n), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            o, a = attend_head(q[b, h], K[b, h // G], V[b, h // G], live[b], softmax_scale)
            out[b, h] = o
            alpha[b, h] = a
    return out, alpha


def score_increment(alpha: np.ndarray, score_scale: float) -> np.ndarray:
    """One layer's contribution to the cumulative scores (Eq. 1).

    alpha [B, Hq, n] -> [B, n]: score_scale * sum over query heads.  With
    score_scale = 1/(L*H) the sum over the L layer calls of a step is Eq. 1's
    double average; evicted positions have alpha = 0 and so keep their score.
    """
    return float(score_scale) * alpha.sum(axis=1)


def value_norms(V: np.ndarray) -> np.ndarray:
    """Euclidean norm of every value row: V [..., d] -> [...]."""
    V = np.asarray(V, dtype=np.float64)
    return np.sqrt((V * V).sum(axis=-1))


def score_increment_vatp(alpha: np.ndarray, vnorm: np.ndarray, score_scale: float) -> np.ndarray:
    """One layer's contribution under the value-aware scorer of the scoring ablation
    (Sec. "Ablation: Importance Scoring Methods"): every head's attention weight on a
    position is multiplied by the norm of the value row that head reads there.

    alpha [B, Hq, n], vnorm [B, Hkv, n] -> [B, n]:
    score_scale * sum_h alpha[b, h, i] * vnorm[b, h // G, i].
    The paper names "value vector norms" without saying which norm or which copy of
    the row; this build's reading: Euclidean, of the row as appended (a position's
    norm does not change when its row is later compressed).
    """
    alpha = np.asarray(alpha, dtype=np.float64)
    vnorm = np.asarray(vnorm, dtype=np.float64)
    B, Hq, n = alpha.shape
    G = Hq // vnorm.shape[1]
    inc = np.zeros((B, n), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            inc[b] += alpha[b, h] * vnorm[b, h // G]
    return float(score_scale) * inc


def key_redundancy(K: np.ndarray, k_before: np.ndarray = None) -> np.ndarray:
    """Redundancy of every key row with respect to its neighbour (the "Redundancy" scorer of
    Sec. "Ablation: Importance Scoring Methods": tokens with high cosine similarity to
    neighbours are penalised; the paper gives no formula).  This build's reading:

        rho_i = max(0, <k_i, k_{i-1}> / (||k_i|| ||k_{i-1}||)),

    the cosine similarity of a position's key row with the key row of the position before it
    (the neighbour that exists when the token is appended), of the same layer and kv head,
    clamped below at 0; 0 for the first position and whenever either row is all zero.
    Taken once, from the rows as appended; it stays with the position like the value norm.

    K [..., n, d]; k_before [..., d] is the row in front of K[..., 0, :] (None: there is none).
    Returns [..., n]."""
    K = np.asarray(K, dtype=np.float64)
    n = K.shape[-2]
    rho = np.zeros(K.shape[:-1], dtype=np.float64)
    for i in range(n):
        if i == 0:
            if k_before is None:
                continue
            prev = np.asarray(k_before, dtype=np.float64)
        else:
            prev = K[..., i - 1, :]
        cur = K[..., i, :]
        dot = (cur * prev).sum(axis=-1)
        den = np.sqrt((cur * cur).sum(axis=-1)) * np.sqrt((prev * prev).sum(axis=-1))
        cos = np.where(den > 0.0, dot / np.where(den > 0.0, den, 1.0), 0.0)
        rho[..., i] = np.maximum(cos, 0.0)
    return rho


def score_increment_redundancy(alpha: np.ndarray, rho: np.ndarray, live: np.ndarray, score_scale: float,
                               weight: float, vnorm: np.ndarray = None) -> np.ndarray:
    """One layer's contribution under the redundancy-penalised scorers of the scoring ablation
    ("Redundancy (attn - redundancy)" and, with vnorm, "Combined (attn x val - redundancy)").
    This build's reading: per query head, the attention weight on a position (times the value
    norm for the combined scorer) minus weight * rho / n_live, rho being the position's key
    redundancy in the kv head that query head reads and n_live the number of positions the
    query attends to; so a head's attention mass (1) and its penalty mass (at most `weight`)
    are on the same scale at any cache length.  Evicted positions receive nothing.

    alpha [B, Hq, n], rho [B, Hkv, n], live [B, n] bool, vnorm [B, Hkv, n] or None -> [B, n]:
    score_scale * sum_h (alpha[b,h,i] * (vnorm[b,h//G,i] or 1) - weight * rho[b,h//G,i] / n_live[b])."""
    alpha = np.asarray(alpha, dtype=np.float64)
    rho = np.asarray(rho, dtype=np.float64)
    B, Hq, n = alpha.shape
    G = Hq // rho.shape[1]
    inc = np.zeros((B, n), dtype=np.float64)
    for b in range(B):
        n_live = int(np.sum(live[b]))
        for h in range(Hq):
            gain = alpha[b, h] * (vnorm[b, h // G] if vnorm is not None else 1.0)
            pen = float(weight) * rho[b, h // G] / max(n_live, 1)
            inc[b] += np.where(live[b], gain - pen, 0.0)
    return float(score_scale) * inc


def eviction_error_bound(alpha_full: np.ndarray, V: np.ndarray, evicted: np.ndarray) -> float:
    """Right-hand side of Eq. 4: 2 * sum_{i in E} alpha_i ||v_i||."""
    V = np.asarray(V, dtype=np.float64)
    return float(2.0 * np.sum(alpha_full[evicted] * np.linalg.norm(V[evicted], axis=1)))


# ----------------------------------------------------------------------------
# T2 codec, defined in binary32
# ----------------------------------------------------------------------------
def quant_int8_row(x: np.ndarray):
    """Symmetric int8 with one absmax scale per row (last axis).

    a = max|x|; scale = a / 127 (binary32 division); code = clip(rne(x / scale), -127, 127);
    a == 0 gives scale 0 and all-zero codes.  Returns (codes int8, scale float32 [...]).
    """
    x = np.asarray(x, dtype=np.float32)
    a = np.max(np.abs(x), axis=-1).astype(np.float32)
    scale = (a / np.float32(127.0)).astype(np.float32)
    safe = np.where(scale > 0, scale, np.float32(1.0)).astype(np.float32)
    r = np.rint((x / safe[..., None]).astype(np.float32))
    codes = np.clip(r, -127, 127)
    codes = np.where(scale[..., None] > 0, codes, 0).astype(np.int8)
    return codes, scale


def dequant_int8_row(codes: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """x_hat = code * scale, exact in float64 (7-bit integer times binary32)."""
    return codes.astype(np.float64) * np.asarray(scale, dtype=np.float64)[..., None]


INT4_GROUP = 32


def quant_int4_g32(x: np.ndarray):
    """Symmetric int4, groups of 32 along the last axis, binary16 scales.

    Per group: a = max|x|; scale = fp16_rne(a / 7) with a/7 in binary32;
    code = clip(rne(x / float32(scale)), -7, 7); a scale that is zero (a == 0,
    or a/7 below half the smallest binary16 subnormal) gives all-zero codes.
    Returns (codes int8 in [-7, 7] with shape of x, scales float32-valued
    binary16 numbers with shape [..., d/32]).
    """
    x = np.asarray(x, dtype=np.float32)
    d = x.shape[-1]
    assert d % INT4_GROUP == 0
    xg = x.reshape(x.shape[:-1] + (d // INT4_GROUP, INT4_GROUP))
    a = np.max(np.abs(xg), axis=-1).astype(np.float32)
    scale = round_to_fp16((a / np.float32(7.0)).astype(np.float32))
    safe = np.where(scale > 0, scale, np.float32(1.0)).astype(np.float32)
    r = np.rint((xg / safe[..., None]).astype(np.float32))
    codes = np.clip(r, -7, 7)
    codes = np.where(scale[..., None] > 0, codes, 0).astype(np.int8)
    return codes.reshape(x.shape), scale


def dequant_int4_g32(codes: np.ndarray, scale: np.ndarray) -> np.ndarray:
    d = codes.shape[-1]
    cg = codes.reshape(codes.shape[:-1] + (d // INT4_GROUP, INT4_GROUP)).astype(np.float64)
    return (cg * np.asarray(scale, dtype=np.float64)[..., None]).reshape(codes.shape)


def pack_int4(codes: np.ndarray) -> np.ndarray:
    """Two's-complement nibbles, element 2j in the low nibble of byte j."""
    c = codes.astype(np.int16) & 0xF
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def t2_encode(x32: np.ndarray, t2_format: str):
    if t2_format == "int8_row":
        return quant_int8_row(x32)
    if t2_format == "int4_g32":
        return quant_int4_g32(x32)
    raise ValueError(t2_format)


def t2_decode(codes, scale, t2_format: str) -> np.ndarray:
    if t2_format == "int8_row":
        return dequant_int8_row(codes, scale)
    return dequant_int4_g32(codes, scale)


def t2_decode_to_storage(codes, scale, t2_format: str, kv_dtype: str) -> np.ndarray:
    """Value a promoted T2 row is stored as: binary32 product, then rounded to the KV dtype."""
    if t2_format == "int8_row":
        p = codes.astype(np.float32) * np.asarray(scale, dtype=np.float32)[..., None]
    else:
        d = codes.shape[-1]
        cg = codes.reshape(codes.shape[:-1] + (d // INT4_GROUP, INT4_GROUP)).astype(np.float32)
        p = (cg * np.asarray(scale, dtype=np.float32)[..., None]).reshape(codes.shape)
    return round_to_storage(p.astype(np.float32), kv_dtype)


# ----------------------------------------------------------------------------
# tier assignment (Sec. 3.3, Algorithm 1 "tier management")
# ----------------------------------------------------------------------------
def candidate_range(n: int, n_prompt: int, k_sink: int, k_window: int):
    """U = [n_prompt + k_sink, n - k_window): everything else is protected (Sec. 3.2)."""
    lo = n_prompt + k_sink
    hi = n - k_window
    if hi <= lo:
        return lo, lo
    return lo, hi


def tier_counts(m: int, policy_ppm, n_already_evicted: int = 0):
    """Sizes (n0, n1, n2, n3) of the four bands among m candidates.

    Fractions are parts-per-million of |U| (total-fraction reading of the
    eviction ratio): n3, n2, n0 by floor, T1 takes the remainder.  Evicted
    positions never come back: if more are already evicted than n3 allows,
    n3 grows to that count at the expense of n2, then n1, then n0.
    """
    f0, f1, f2, f3 = (int(v) for v in policy_ppm)
    assert f0 + f1 + f2 + f3 == PPM
    n3 = (f3 * m) // PPM
    n2 = (f2 * m) // PPM
    n0 = (f0 * m) // PPM
    n1 = m - n0 - n2 - n3
    extra = n_already_evicted - n3
    if extra > 0:
        n3 += extra
        take = min(extra, n2); n2 -= take; extra -= take
        take = min(extra, n1); n1 -= take; extra -= take
        take = min(extra, n0); n0 -= take; extra -= take
        assert extra == 0
    return n0, n1, n2, n3


def tier_counts_alg1(m: int, policy_ppm, n_already_evicted: int = 0):
    """Sizes (n0, n1, n2, n3) by Algorithm 1 read literally (tier management step).

    The candidate set the algorithm ranks is what is still in the cache:
    live = m - n_already_evicted.  n_evict = floor(r * live) of them are removed
    at THIS event (so eviction compounds from event to event), and of the
    survivors n_hbm = floor(beta * (live - n_evict)) stay in HBM.  In the four
    parts-per-million fractions r = f3 and beta = f0 / (1 - f3); the compressed
    band, which Algorithm 1 does not have, takes floor(f2 / (1 - f3) * survivors)
    in the same way, and T1 the remainder.
    """
    f0, f1, f2, f3 = (int(v) for v in policy_ppm)
    assert f0 + f1 + f2 + f3 == PPM
    live = m - n_already_evicted
    n_evict = (f3 * live) // PPM
    survivors = live - n_evict
    if f3 == PPM:
        n_hbm = n_cmp = 0
    else:
        n_hbm = (f0 * survivors) // (PPM - f3)
        n_cmp = (f2 * survivors) // (PPM - f3)
    return n_hbm, survivors - n_hbm - n_cmp, n_cmp, n_already_evicted + n_evict


def score_order(bits: int) -> int:
    """Unsigned 32-bit integer that orders binary32 bit patterns like the values they encode
    (-0 directly below +0; NaNs are not scores)."""
    return (~bits & 0xFFFFFFFF) if (bits & 0x80000000) else (bits | 0x80000000)


def classify_sequence(score_f32: np.ndarray, tier_prev: np.ndarray, n: int,
                      n_prompt: int, k_sink: int, k_window: int, policy_ppm, count_rule: int = 0) -> np.ndarray:
    """New tier of each of the n positions of one sequence.

    Candidates are ranked ascending by the key (live, score_order, position):
    live = 0 for an already evicted position; score_order puts binary32 scores in
    the order of their values (total order on the bit patterns: for a score with
    the sign bit clear the pattern with that bit set, else the complemented
    pattern; for the non-negative scores of Eq. 1 this is the order of the
    patterns themselves).  Penalised scorers can go below zero.  Lowest n3 -> T3, next
    n2 -> T2, next n1 -> T1, top n0 -> T0; protected positions -> T0.
    The sort is written out with Python's sorted() on explicit tuples.
    """
    s = np.ascontiguousarray(score_f32[:n], dtype=np.float32)
    bits = s.view(np.uint32)
    lo, hi = candidate_range(n, n_prompt, k_sink, k_window)
    tier_new = np.zeros(n, dtype=np.uint8)
    m = hi - lo
    if m == 0:
        return tier_new
    evicted = int(np.sum(tier_prev[lo:hi] == T3))
    n0, n1, n2, n3 = (tier_counts_alg1 if count_rule == 1 else tier_counts)(m, policy_ppm, evicted)
    keys = [((0 if tier_prev[i] == T3 else 1), score_order(int(bits[i])), i) for i in range(lo, hi)]
    order = [k[2] for k in sorted(keys)]
    for rank, i in enumerate(order):
        if rank < n3:
            tier_new[i] = T3
        elif rank < n3 + n2:
            tier_new[i] = T2
        elif rank < n3 + n2 + n1:
            tier_new[i] = T1
        else:
            tier_new[i] = T0
    return tier_new


def compact_lists(tier_row: np.ndarray, n: int):
    """Per tier, ascending list of positions (stream compaction of the tier array)."""
    return [np.nonzero(tier_row[:n] == t)[0].astype(np.int32) for t in (T0, T1, T2, T3)]


# ----------------------------------------------------------------------------
# the whole cache: Algorithm 1's state and loop body
# ----------------------------------------------------------------------------
class OracleCache:
    """State of Algorithm 1 for a batch of B equally long sequences.

    K[l], V[l]: [B, Hkv, max_tokens, d] float64 holding the *effective* value of
    every row: the stored (kv_dtype-representable) value for T0/T1 rows, the
    dequantised value for T2 rows; rows of evicted positions are zeroed.
    tier [B, max_tokens] uint8, score [B, max_tokens] float64.
    One score and one tier per (sequence, position), shared by layers and heads.
    """

    def __init__(self, n_layers, batch, n_q_heads, n_kv_heads, head_dim, max_tokens,
                 kv_dtype="bf16", t2_format="int8_row", n_prompt=0, k_sink=4, k_window=128,
                 score_scale=None, softmax_scale=None, layers=None, scorer="attention", redundancy_weight=1.0):
        self.L, self.B, self.Hq, self.Hkv, self.d = n_layers, batch, n_q_heads, n_kv_heads, head_dim
        self.G = n_q_heads // n_kv_heads
        assert self.G * n_kv_heads == n_q_heads
        self.max_tokens = max_tokens
        self.kv_dtype, self.t2_format = kv_dtype, t2_format
        self.n_prompt, self.k_sink, self.k_window = n_prompt, k_sink, k_window
        self.score_scale = (1.0 / (n_layers * n_q_heads)) if score_scale is None else float(score_scale)
        self.softmax_scale = (1.0 / np.sqrt(head_dim)) if not softmax_scale else float(softmax_scale)
        # `layers` lets a caller hold only a subset of the layers (bounded CPU timing samples).
        self.layers = list(range(n_layers)) if layers is None else list(layers)
        shape = (batch, n_kv_heads, max_tokens, head_dim)
        self.K = {l: np.zeros(shape, dtype=np.float64) for l in self.layers}
        self.V = {l: np.zeros(shape, dtype=np.float64) for l in self.layers}
        self.t2 = {l: {} for l in self.layers}          # (b, pos) -> (kcodes, kscale, vcodes, vscale), all kv heads
        self.length = {l: 0 for l in self.layers}
        self.tier = np.zeros((batch, max_tokens), dtype=np.uint8)
        self.tier_pending = None
        self.score = np.zeros((batch, max_tokens), dtype=np.float64)
        # "attention": Eq. 1.  The others are the variants of the scoring ablation: "vatp" (attention x value
        # norm), "redundancy" (attention - redundancy), "combined" (attention x value norm - redundancy).
        assert scorer in ("attention", "vatp", "redundancy", "combined")
        self.scorer = scorer
        self.redundancy_weight = float(redundancy_weight)
        self.vnorm = {l: np.zeros(shape[:3], dtype=np.float64) for l in self.layers} if scorer in ("vatp", "combined") else None
        self.last_k = {}
        self.rho = {l: np.zeros(shape[:3], dtype=np.float64) for l in self.layers} if scorer in ("redundancy", "combined") else None
        # sum of the magnitudes of what was added and what was taken off (the scale of a penalised score's rounding)
        self.score_mag = np.zeros((batch, max_tokens), dtype=np.float64)

    # -- Algorithm 1: the cache grows by the generated token --------------------
    def append(self, layer, k, v):
        """k, v [B, n_new, Hkv, d], values representable in kv_dtype.  New tokens are T0."""
        k = np.asarray(k, dtype=np.float64)
        v = np.asarray(v, dtype=np.float64)
        n0 = self.length[layer]
        n_new = k.shape[1]
        if n0 + n_new > self.max_tokens:
            raise OverflowError("append beyond max_tokens")
        if self.rho is not None:
            # against the row appended just before, as it was appended (it may have been compressed or evicted since)
            before = self.last_k[layer] if n0 > 0 else None
            self.rho[layer][:, :, n0:n0 + n_new] = key_redundancy(k.transpose(0, 2, 1, 3), before)
            self.last_k[layer] = k[:, -1].copy()
        self.K[layer][:, :, n0:n0 + n_new] = k.transpose(0, 2, 1, 3)
        self.V[layer][:, :, n0:n0 + n_new] = v.transpose(0, 2, 1, 3)
        if self.vnorm is not None:
            self.vnorm[layer][:, :, n0:n0 + n_new] = value_norms(v.transpose(0, 2, 1, 3))
        self.length[layer] = n0 + n_new
        self.tier[:, n0:n0 + n_new] = T0

    # -- forward pass + score update of one layer -------------------------------
    def attend_and_score(self, layer, q):
        n = self.length[layer]
        live = self.tier[:, :n] != T3
        out, alpha = attend_gqa(q, self.K[layer][:, :, :n], self.V[layer][:, :, :n], live, self.softmax_scale)
        self._add_scores(layer, alpha, live, n)
        return out

    def _add_scores(self, layer, alpha, live, n):
        """The layer call's contribution to the first n positions' scores, by the configured scorer."""
        if self.scorer == "vatp":
            inc = score_increment_vatp(alpha, self.vnorm[layer][:, :, :n], self.score_scale)
            mag = inc
        elif self.scorer in ("redundancy", "combined"):
            vn = self.vnorm[layer][:, :, :n] if self.scorer == "combined" else None
            inc = score_increment_redundancy(alpha, self.rho[layer][:, :, :n], live, self.score_scale,
                                             self.redundancy_weight, vn)
            gain = score_increment_redundancy(alpha, self.rho[layer][:, :, :n], live, self.score_scale, 0.0, vn)
            mag = gain + (gain - inc)
        else:
            inc = score_increment(alpha, self.score_scale)
            mag = inc
        self.score[:, :n] += inc
        self.score_mag[:, :n] += mag

    def attend_and_score_chunk(self, layer, q):
        """Several query tokens at once: q [B, T, Hq, d] belongs to the last T appended positions,
        query j to position n - T + j.  Each attends causally, i.e. to the positions up to and
        including its own (Eq. 2 sums i = 1..t for the token at t), and each adds its weights to
        the scores (Eq. 1), in the order j = 0..T-1: the same as T single-token steps whose
        appends had all been done beforehand.  Returns out [B, T, Hq, d]."""
        q = np.asarray(q, dtype=np.float64)
        n = self.length[layer]
        T = q.shape[1]
        if T < 1 or T > n:
            raise ValueError("chunk length")
        out = np.zeros(q.shape, dtype=np.float64)
        for j in range(T):
            m = n - T + j + 1
            live = self.tier[:, :m] != T3
            o, alpha = attend_gqa(q[:, j], self.K[layer][:, :, :m], self.V[layer][:, :, :m], live, self.softmax_scale)
            self._add_scores(layer, alpha, live, m)
            out[:, j] = o
        return out

    # -- tier management ----------------------------------------------------------
    def classify(self, policy_ppm, score_f32=None, count_rule=0):
        """Plan new tiers.  `score_f32` (e.g. the GPU's array) replaces the oracle's own
        scores rounded to binary32, so the assignment can be checked bit-exactly."""
        ns = set(self.length.values())
        if len(ns) != 1:
            raise RuntimeError("layers differ in length")
        n = ns.pop()
        s32 = self.score.astype(np.float32) if score_f32 is None else np.asarray(score_f32, dtype=np.float32)
        new = np.zeros_like(self.tier)
        for b in range(self.B):
            new[b, :n] = classify_sequence(s32[b], self.tier[b], n, self.n_prompt, self.k_sink,
                                           self.k_window, policy_ppm, count_rule)
        self.tier_pending = new
        return new

    def set_tiers(self, tiers):
        """Force a plan (teacher forcing, invariant tests); apply with migrate()."""
        t = np.zeros_like(self.tier)
        t[:, :tiers.shape[1]] = tiers
        self.tier_pending = t

    def migrate(self):
        """Apply the pending plan: T0<->T1 keeps bits; ->T2 encodes the current stored row;
        T2->T0/T1 stores the decoded value rounded to kv_dtype; T2->T2 keeps its codes;
        ->T3 deletes the row.  Scores are never reset."""
        if self.tier_pending is None:
            raise RuntimeError("no pending plan")
        new = self.tier_pending
        ns = set(self.length.values())
        n = ns.pop()
        for b in range(self.B):
            for i in range(n):
                old_t, new_t = int(self.tier[b, i]), int(new[b, i])
                if old_t == new_t:
                    continue
                if old_t == T3:
                    raise RuntimeError("evicted position cannot return")
                for l in self.layers:
                    if new_t == T3:
                        self.K[l][b, :, i] = 0.0
                        self.V[l][b, :, i] = 0.0
                        self.t2[l].pop((b, i), None)
                    elif new_t == T2:
                        kc, ks = t2_encode(self.K[l][b, :, i].astype(np.float32), self.t2_format)
                        vc, vs = t2_encode(self.V[l][b, :, i].astype(np.float32), self.t2_format)
                        self.t2[l][(b, i)] = (kc, ks, vc, vs)
                        self.K[l][b, :, i] = t2_decode(kc, ks, self.t2_format)
                        self.V[l][b, :, i] = t2_decode(vc, vs, self.t2_format)
                    elif old_t == T2:
                        kc, ks, vc, vs = self.t2[l].pop((b, i))
                        self.K[l][b, :, i] = t2_decode_to_storage(kc, ks, self.t2_format, self.kv_dtype)
                        self.V[l][b, :, i] = t2_decode_to_storage(vc, vs, self.t2_format, self.kv_dtype)
                    # T0 <-> T1: placement only, the stored bits do not change (Prop. 1)
        self.tier[:, :n] = new[:, :n]
        self.tier_pending = None

    def index_lists(self, seq):
        n = next(iter(self.length.values()))
        return compact_lists(self.tier[seq], n)
