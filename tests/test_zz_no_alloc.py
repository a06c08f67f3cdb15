"""The entry point that allocates nothing, tkv_attend_and_score_noalloc, against tkv_attend_and_score: the same
kernels with their scratch in the library's fixed device array, so outputs and scores must agree bit for bit.
Two calls in a row share the array, the second on a smaller cache (the array then still holds the first call's
logits and partials behind the part the second call uses)."""
import numpy as np
import pytest
import torch

from tkv_synth import Workload, small_config

pytestmark = pytest.mark.gpu


def _twin_caches(cfg, mode, tiers):
    """Two caches with identical contents and the same forced plan: one for each entry point."""
    import paper_2605_09490_amd as tkv
    wl = Workload(cfg, device="cuda")
    ss = 1.0 / (cfg.n_layers * cfg.n_q_heads)
    caches = []
    for _ in range(2):
        g = tkv.TieredKV(cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.max_tokens,
                         kv_dtype=cfg.kv_dtype, t2_format=cfg.t2_format, k_sink=cfg.k_sink, k_window=cfg.k_window,
                         score_scale=ss, prefetch_mode=mode)
        for l in range(cfg.n_layers):
            g.append(l, *wl.context_kv(l))
        g.set_tiers(tiers)
        g.migrate()
        caches.append(g)
    return wl, caches


def _tiers(rng, B, n):
    t = rng.choice(4, size=(B, n), p=(0.4, 0.3, 0.2, 0.1)).astype(np.uint8)
    t[:, :4] = 0
    t[:, n - 8:] = 0
    return t


@pytest.mark.parametrize("mode", ["wait", "lazy"])
def test_noalloc_entry_point_matches_the_allocating_one(mode):
    import paper_2605_09490_amd as tkv
    rng = np.random.default_rng(17)
    big = small_config(name="big", n_layers=2, batch=3, n_q_heads=10, n_kv_heads=2, head_dim=128, kv_dtype="bf16",
                       context=900, decode_steps=2, sigma=1.0)
    small = small_config(name="small", n_layers=2, batch=2, n_q_heads=8, n_kv_heads=2, head_dim=64, kv_dtype="f32",
                         context=150, decode_steps=2, t2_format="int4_g32", sigma=1.0)
    sets = []
    for cfg in (big, small):
        print(f"[case] noalloc {mode} {cfg.name}", flush=True)
        sets.append((cfg, *_twin_caches(cfg, mode, _tiers(rng, cfg.batch, cfg.context))))
    # the calls of the fixed-scratch variant come in a row: first the larger cache, then the smaller one
    for step in range(2):
        for cfg, wl, (ref_c, new_c) in sets:
            for l in range(cfg.n_layers):
                k, v = wl.step_kv(step, l)
                ref_c.append(l, k, v)
                new_c.append(l, k, v)
                q = wl.step_q(step, l)
                want = ref_c.attend_and_score(l, q)
                got = torch.full_like(want, float("nan"))
                new_c.attend_and_score_noalloc(l, q, got)
                assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), (cfg.name, step, l)
    for cfg, wl, (ref_c, new_c) in sets:
        n = cfg.context + 2
        assert np.array_equal(new_c.get_scores()[:, :n].view(np.uint32), ref_c.get_scores()[:, :n].view(np.uint32)), cfg.name
        ref_c.close(); new_c.close()
    # a cache whose call needs more scratch than the fixed array holds is refused with a clear error, nothing launched
    wide = tkv.TieredKV(1, 8, 64, 8, 128, 16384, kv_dtype="bf16", t0_rows=64, staging_rows=64, t2_rows=64, host_rows=64)
    k = torch.zeros((8, 1, 8, 128), dtype=torch.bfloat16, device="cuda")
    wide.append(0, k, k)
    q = torch.zeros((8, 64, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((8, 64, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(tkv.TkvError) as e:
        wide.attend_and_score_noalloc(0, q, out)
    assert e.value.status == tkv.TKV_ECAPACITY and "bytes of scratch" in str(e.value)
    wide.attend_and_score(0, q, out)          # the allocating entry point still serves it
    wide.close()
