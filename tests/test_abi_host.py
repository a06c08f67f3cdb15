"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares, and the
host-only logic (configuration validation, band sizes) behaves.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2605_09490_amd as tkv
from paper_2605_09490_amd import binding
from oracle import tkv_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    src = open(os.path.join(ROOT, "include", "tkv.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(tkv_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    lib = tkv.load_library()
    names = _declared_symbols()
    assert "tkv_create" in names and "tkv_attend_and_score" in names and "tkv_migrate" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.SYMBOLS) == names


def test_config_struct_matches_header_field_order():
    src = open(os.path.join(ROOT, "include", "tkv.h")).read()
    body = src[src.index("typedef struct {", src.index("tkv_prefetch_mode;")):]
    body = body[:body.index("} tkv_config;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip().replace("typedef struct {", "")
        if not decl:
            continue
        m = re.match(r"(?:void\*?|void)\s*\(\*(\w+)\)", decl)
        if m:
            fields.append(m.group(1))
            continue
        names = decl.split(None, 1)[1] if " " in decl else ""
        fields += [n.strip().lstrip("*") for n in names.split(",")]
    assert fields == [f[0] for f in binding.tkv_config._fields_]


def test_create_rejects_bad_configs_before_touching_the_device():
    lib = tkv.load_library()

    def status(**kw):
        cfg = binding.tkv_config()
        base = dict(n_layers=1, batch=1, n_q_heads=8, n_kv_heads=2, head_dim=64, max_tokens=64, kv_dtype=0, t2_format=0)
        base.update(kw)
        for k, v in base.items():
            setattr(cfg, k, v)
        h = C.c_void_p()
        st = lib.tkv_create(C.byref(cfg), C.byref(h))
        assert not h.value
        return st

    assert status(head_dim=96) == tkv.TKV_EINVAL
    assert status(n_q_heads=7) == tkv.TKV_EINVAL
    assert status(n_q_heads=18, n_kv_heads=2) == tkv.TKV_EINVAL      # group of 9
    assert status(max_tokens=0) == tkv.TKV_EINVAL
    assert status(max_tokens=1 << 24) == tkv.TKV_EINVAL
    assert status(kv_dtype=7) == tkv.TKV_EINVAL
    assert status(t2_format=2) == tkv.TKV_EINVAL
    assert status(k_window=-1) == tkv.TKV_EINVAL
    assert status(prefetch_mode=5) == tkv.TKV_EINVAL
    assert status(scorer=4) == tkv.TKV_EINVAL
    assert status(scorer=2, redundancy_weight=-1.0) == tkv.TKV_EINVAL
    assert lib.tkv_create(None, None) == tkv.TKV_EINVAL
    assert b"tkv_create" in lib.tkv_last_error(None)
    lib.tkv_destroy(None)


def test_tier_counts_agree_with_oracle_and_reject_bad_policy():
    rng = np.random.default_rng(0)
    for _ in range(200):
        m = int(rng.integers(0, 40000))
        cut = np.sort(rng.integers(0, 10 ** 6 + 1, size=3))
        pol = (int(cut[0]), int(cut[1] - cut[0]), int(cut[2] - cut[1]), int(10 ** 6 - cut[2]))
        ev = int(rng.integers(0, m + 1)) if rng.random() < 0.3 else 0
        assert tkv.tier_counts(pol, m, ev) == O.tier_counts(m, pol, ev)
        assert tkv.tier_counts(pol, m, ev, count_rule=1) == O.tier_counts_alg1(m, pol, ev)
    with pytest.raises(tkv.TkvError):
        tkv.tier_counts((1, 2, 3, 4), 10)
    with pytest.raises(tkv.TkvError):
        tkv.tier_counts((250000, 250000, 250000, 250000), 10, 0, count_rule=5)


def test_host_code_under_sanitizers_host_only_part():
    """The library's host code built with AddressSanitizer and UndefinedBehaviorSanitizer (host side only) and driven by
    tests/native/host_sanitize_check.cpp: here the part that needs no GPU (configuration validation, band sizes, NULL
    handles).  The full scenario runs in the GPU suite."""
    import subprocess
    from paper_2605_09490_amd import build
    exe = build.HOST_CHECK
    if not os.path.exists(exe):
        build.build_host_check()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:protect_shadow_gap=0", UBSAN_OPTIONS="halt_on_error=1")
    r = subprocess.run([exe, "--host-only"], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host sanitizer check passed" in r.stdout
