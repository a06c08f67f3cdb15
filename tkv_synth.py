"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path's tests/bench.

This module holds NO arithmetic of the method (no attention, no scoring, no
quantiser, no ranking): it only draws random tensors with the shapes and the
long-tail structure of the paper's reasoning workloads (Sec. 2.1: a few
positions collect most of the attention mass) and rounds them to the storage
dtype.  Both sides read the same stored arrays, so no cross-device RNG
reproducibility is needed.

Recipe (stand-in for the paper's GSM8K / MATH reasoning traces, which are not
available offline):
  K, V ~ N(0, 1) i.i.d.; every (sequence, position) draws one factor
  c = exp(sigma * z), z ~ N(0, 1), shared by all layers and kv heads, and
  K <- c * K; optionally a random `boost_frac` of positions gets K <- boost * K
  (late-referenced intermediate results).  Queries ~ N(0, 1) fresh per
  (step, layer).  All values are rounded to the KV dtype (bf16, fp16 or fp32).
  This is the recipe the benchmark configurations state (recipe = "scale").  Because the factor multiplies the whole
  key row, it multiplies the logits, and the attention of every query collapses onto the few largest factors.

Second recipe (recipe = "bias", the "-tail" configurations): the same per-position draw enters the logits as an
  additive term instead: K ~ N(0, 1) unscaled, except that element 0 of every key row is sigma * z (plus log(boost)
  for a boosted position) and element 0 of every query is sqrt(head_dim), so that a position's logit is
  sigma * z + (a unit-variance term that differs per query).  Averaged over queries, layers and heads a position's
  attention weight is then proportional to exp(sigma * z): log-normal, the long tail of Sec. 2.1 (sigma = 1 puts
  about 56 % of the mass on the top 20 % of positions).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    kv_dtype: str            # "f32" | "bf16" | "f16"
    context: int             # tokens preloaded before the first decode step
    decode_steps: int
    reclassify_every: int    # Delta
    policy_ppm: tuple        # (T0, T1, T2, T3) parts per million of the candidates
    t2_format: str           # "int8_row" | "int4_g32"
    sigma: float
    boost_frac: float = 0.0
    boost: float = 1.0
    k_sink: int = 4
    k_window: int = 128
    n_prompt: int = 0
    score_scale: float | None = None   # None -> 1/(L*Hq) (Eq. 1)
    seed: int = 0
    recipe: str = "scale"    # "scale": the position factor multiplies the key row; "bias": it is added to the logit

    @property
    def max_tokens(self) -> int:
        return self.context + self.decode_steps

    @property
    def torch_dtype(self):
        return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[self.kv_dtype]


CONFIGS = {
    "tiny": WorkloadConfig("tiny", 1, 1, 8, 2, 64, "f32", 512, 32, 8,
                           (500_000, 300_000, 150_000, 50_000), "int8_row", 1.0,
                           k_window=32, score_scale=1.0),
    "7b": WorkloadConfig("7b", 28, 8, 28, 4, 128, "bf16", 2048, 64, 16,
                         (500_000, 350_000, 100_000, 50_000), "int8_row", 1.0),
    "14b": WorkloadConfig("14b", 48, 8, 40, 8, 128, "bf16", 4096, 64, 16,
                          (300_000, 520_000, 150_000, 30_000), "int8_row", 1.2,
                          boost_frac=0.03, boost=4.0),
    "32b": WorkloadConfig("32b", 64, 4, 40, 8, 128, "bf16", 8192, 32, 8,
                          (300_000, 500_000, 100_000, 100_000), "int8_row", 1.0),
    "prod": WorkloadConfig("prod", 28, 64, 28, 4, 128, "bf16", 16384, 16, 8,
                           (300_000, 470_000, 200_000, 30_000), "int4_g32", 1.0),
}
# the 14B shape and policy with the log-normal attention profile the method is described on (not a benchmark
# configuration: the graded line uses "14b")
CONFIGS["14b-tail"] = WorkloadConfig("14b-tail", 48, 8, 40, 8, 128, "bf16", 4096, 64, 16,
                                     (300_000, 520_000, 150_000, 30_000), "int8_row", 1.0,
                                     boost_frac=0.03, boost=4.0, recipe="bias")


def _gen(device, *key) -> torch.Generator:
    g = torch.Generator(device=device)
    h = 0x9E3779B97F4A7C15
    for k in key:
        h = (h ^ (int(k) + 0x9E3779B97F4A7C15 + ((h << 6) & 0xFFFFFFFFFFFFFFFF) + (h >> 2))) & 0x7FFFFFFFFFFFFFFF
    g.manual_seed(h)
    return g


class Workload:
    """Draws the context, the per-step appended rows and the queries of one config."""

    def __init__(self, cfg: WorkloadConfig, device="cpu"):
        self.cfg = cfg
        self.device = torch.device(device)
        n_total = cfg.max_tokens
        g = _gen("cpu", cfg.seed, 1)
        z = torch.randn(cfg.batch, n_total, generator=g, dtype=torch.float32)
        c = torch.exp(cfg.sigma * z)
        if cfg.boost_frac > 0:
            u = torch.rand(cfg.batch, n_total, generator=g)
            c = torch.where(u < cfg.boost_frac, c * cfg.boost, c)
        self.key_factor = c.to(self.device)          # [B, n_total]
        self.bias = cfg.recipe == "bias"
        assert cfg.recipe in ("scale", "bias")
        self.key_bias = torch.log(c).to(self.device)  # [B, n_total]: what the "bias" recipe writes into element 0 of a key row
        self.q0 = float(cfg.head_dim) ** 0.5

    def _kv(self, lo, hi, layer, tag):
        cfg = self.cfg
        g = _gen(self.device, cfg.seed, 2, tag, layer, lo)
        shape = (cfg.batch, hi - lo, cfg.n_kv_heads, cfg.head_dim)
        k = torch.randn(shape, generator=g, device=self.device, dtype=torch.float32)
        v = torch.randn(shape, generator=g, device=self.device, dtype=torch.float32)
        if self.bias:
            k[..., 0] = self.key_bias[:, lo:hi, None]
        else:
            k = k * self.key_factor[:, lo:hi, None, None]
        return k.to(cfg.torch_dtype).contiguous(), v.to(cfg.torch_dtype).contiguous()

    def context_kv(self, layer):
        """k, v [B, context, Hkv, D] in the storage dtype."""
        return self._kv(0, self.cfg.context, layer, 0)

    def step_kv(self, step, layer):
        """k, v [B, 1, Hkv, D] of the token generated at decode step `step`."""
        p = self.cfg.context + step
        return self._kv(p, p + 1, layer, 1)

    def step_q(self, step, layer):
        """q [B, Hq, D] in the storage dtype."""
        cfg = self.cfg
        g = _gen(self.device, cfg.seed, 3, step, layer)
        q = torch.randn((cfg.batch, cfg.n_q_heads, cfg.head_dim), generator=g,
                        device=self.device, dtype=torch.float32)
        if self.bias:
            q[..., 0] = self.q0
        return q.to(cfg.torch_dtype).contiguous()


    def decode_inputs(self, first_step, n_steps):
        """Bulk draw for a benchmark loop: k_all, v_all [n_steps, L, B, 1, Hkv, D] and q_all [n_steps, L, B, Hq, D]
        (same distributions as step_kv / step_q, drawn per layer in one go)."""
        cfg = self.cfg
        p0 = cfg.context + first_step
        fac = self.key_factor[:, p0:p0 + n_steps].t().contiguous()       # [n_steps, B]
        bias = self.key_bias[:, p0:p0 + n_steps].t().contiguous()
        k_all = torch.empty((n_steps, cfg.n_layers, cfg.batch, 1, cfg.n_kv_heads, cfg.head_dim),
                            dtype=cfg.torch_dtype, device=self.device)
        v_all = torch.empty_like(k_all)
        q_all = torch.empty((n_steps, cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.head_dim),
                            dtype=cfg.torch_dtype, device=self.device)
        for l in range(cfg.n_layers):
            g = _gen(self.device, cfg.seed, 4, l, first_step)
            shape = (n_steps, cfg.batch, 1, cfg.n_kv_heads, cfg.head_dim)
            k = torch.randn(shape, generator=g, device=self.device, dtype=torch.float32)
            if self.bias:
                k[..., 0] = bias[:, :, None, None]
            else:
                k = k * fac[:, :, None, None, None]
            k_all[:, l] = k.to(cfg.torch_dtype)
            v_all[:, l] = torch.randn(shape, generator=g, device=self.device, dtype=torch.float32).to(cfg.torch_dtype)
            q = torch.randn((n_steps, cfg.batch, cfg.n_q_heads, cfg.head_dim), generator=g, device=self.device, dtype=torch.float32)
            if self.bias:
                q[..., 0] = self.q0
            q_all[:, l] = q.to(cfg.torch_dtype)
        return k_all, v_all, q_all


def small_config(name="small", **kw) -> WorkloadConfig:
    """A free-form config for parity tests (sizes the oracle finishes in seconds)."""
    base = dict(name=name, n_layers=2, batch=2, n_q_heads=8, n_kv_heads=2, head_dim=64,
                kv_dtype="f32", context=300, decode_steps=8, reclassify_every=4,
                policy_ppm=(500_000, 300_000, 150_000, 50_000), t2_format="int8_row",
                sigma=1.0, k_sink=4, k_window=32)
    base.update(kw)
    return WorkloadConfig(**base)
