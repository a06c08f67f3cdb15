"""Helpers for the GPU parity tests: run the HIP path (through the C ABI) and the CPU oracle side by side
on the same seeded synthetic inputs, and the tolerance definitions."""
import numpy as np
import torch

import paper_2605_09490_amd as tkv
from oracle import tkv_oracle as O
from tkv_synth import Workload

TOL_OUT = {"bf16": 2e-3, "f16": 2e-3, "f32": 1e-5}
TOL_SCORE_REL = 1e-4


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


class Pair:
    """One GPU cache and one oracle cache fed with identical stored values."""

    def __init__(self, cfg, prefetch_mode="wait", preload=True, scorer="attention", redundancy_weight=1.0, **gpu_kw):
        self.cfg = cfg
        self.wl = Workload(cfg, device="cuda")
        self.score_scale = cfg.score_scale if cfg.score_scale is not None else 1.0 / (cfg.n_layers * cfg.n_q_heads)
        self.gpu = tkv.TieredKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.max_tokens,
                                kv_dtype=cfg.kv_dtype, t2_format=cfg.t2_format, n_prompt=cfg.n_prompt,
                                k_sink=cfg.k_sink, k_window=cfg.k_window, score_scale=self.score_scale,
                                prefetch_mode=prefetch_mode, scorer=scorer, redundancy_weight=redundancy_weight, **gpu_kw)
        self.orc = O.OracleCache(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.max_tokens,
                                 kv_dtype=cfg.kv_dtype, t2_format=cfg.t2_format, n_prompt=cfg.n_prompt,
                                 k_sink=cfg.k_sink, k_window=cfg.k_window, score_scale=self.score_scale, scorer=scorer,
                                 redundancy_weight=redundancy_weight)
        self.steps_done = 0
        if preload:
            for l in range(cfg.n_layers):
                k, v = self.wl.context_kv(l)
                self.append(l, k, v)

    def append(self, layer, k, v):
        self.gpu.append(layer, k, v)
        self.orc.append(layer, to_f64(k), to_f64(v))

    def attend(self, layer, q):
        out = self.gpu.attend_and_score(layer, q)
        ref = self.orc.attend_and_score(layer, to_f64(q))
        return to_f64(out), ref

    def attend_chunk(self, layer, q):
        out = self.gpu.attend_and_score_chunk(layer, q)
        ref = self.orc.attend_and_score_chunk(layer, to_f64(q))
        return to_f64(out), ref

    def force_tiers(self, tiers):
        self.gpu.set_tiers(tiers)
        self.gpu.migrate()
        self.orc.set_tiers(tiers)
        self.orc.migrate()

    def close(self):
        self.gpu.close()


def assert_out_close(got, ref, kv_dtype, what=""):
    """max |o_gpu - o_ref| <= tol * max-norm of the head's reference vector (the binary32 output; a 16-bit output is
    checked elsewhere as exactly one rounding of it)."""
    tol = TOL_OUT[kv_dtype]
    scale = np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1e-6)
    err = np.abs(got - ref)
    worst = (err / scale).max()
    assert np.all(err <= tol * scale), f"{what}: attention output off by {worst:.3e} of the head max-norm (tol {tol})"
    return worst


def assert_t2_rows_exact(p, tiers, layers=None, seqs=None, kv_heads=None, what=""):
    """Codes and scales of every T2 row of the chosen (layer, sequence, kv head) sets, K and V, bit for bit against the
    oracle's binary32 encoder (integer work: no tolerance).  tiers [B, n] is the plan in force.  Returns the number of
    rows compared."""
    cfg = p.cfg
    layers = range(cfg.n_layers) if layers is None else layers
    seqs = range(cfg.batch) if seqs is None else seqs
    kv_heads = range(cfg.n_kv_heads) if kv_heads is None else kv_heads
    rows = 0
    for b in seqs:
        for pos in np.nonzero(tiers[b] == 2)[0]:
            pos = int(pos)
            for l in layers:
                oc = p.orc.t2[l][(b, pos)]
                for which in (0, 1):
                    for kvh in kv_heads:
                        codes, scales = p.gpu.get_t2_row(l, b, kvh, pos, which)
                        ref_codes, ref_scale = oc[2 * which][kvh], oc[2 * which + 1][kvh]
                        tag = f"{what}: T2 row layer {l} seq {b} kv head {kvh} pos {pos} {'KV'[which]}"
                        if cfg.t2_format == "int8_row":
                            assert np.array_equal(codes, ref_codes), tag + " codes"
                            assert scales.view(np.uint32)[0] == np.float32(ref_scale).view(np.uint32), tag + " scale"
                        else:
                            assert np.array_equal(codes, O.pack_int4(ref_codes)), tag + " codes"
                            assert np.array_equal(scales, np.asarray(ref_scale, np.float32).astype(np.float16).view(np.uint16)), tag + " scales"
                        rows += 1
    return rows


def assert_scores_close(got32, ref64, n, total_mass, what="", mag64=None):
    """|s_gpu - s_ref| <= 1e-4 * s_ref + 1e-9 * (total mass added so far) / n  (the floor only guards
    weights that underflowed).  A penalised score is a difference: there the relative part is taken of mag64, the sum
    of the magnitudes of what was added and what was taken off (the oracle tracks it), which is s_ref itself for the
    scorers that only add."""
    got = got32[:, :n].astype(np.float64)
    ref = ref64[:, :n]
    bound = TOL_SCORE_REL * (ref if mag64 is None else mag64[:, :n]) + 1e-9 * total_mass / max(n, 1)
    bad = np.abs(got - ref) > bound
    assert not bad.any(), (f"{what}: {bad.sum()} scores off, worst rel "
                           f"{(np.abs(got - ref) / np.maximum(ref, 1e-300)).max():.3e}")
