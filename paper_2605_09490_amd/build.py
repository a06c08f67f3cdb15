"""Builds libtkv.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtkv.so")
# (source, extra flags, object name); the attention kernels are one source compiled in seven parts that build in parallel
UNITS = [("attn_kernels.hip", [f"-DTKV_ATTN_PART={p}"], f"attn_kernels_{p}.o") for p in range(7)]
UNITS += [("tkv_host.hip", [], "tkv_host.o"), ("tier_kernels.hip", [], "tier_kernels.o")]
# packed-fp32 VALU forms are switched off on purpose (the compiler would otherwise emit them from plain float code)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for p in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if p and (os.path.isabs(p) and os.path.exists(p) or not os.path.isabs(p)):
            return p
    return "hipcc"


def build(verbose: bool = False) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(unit):
        src, extra, name = unit
        obj = os.path.join(objdir, name)
        cmd = [hipcc, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(ln for ln in r.stderr.splitlines() if "packed-fp32-ops" not in ln)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(len(UNITS), os.cpu_count() or 4)) as ex:
        objs = list(ex.map(compile_one, UNITS))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


HOST_CHECK = os.path.join(HERE, "_build", "host_sanitize_check")


def build_host_check(verbose: bool = False) -> str:
    """A second build of the host code (tkv_host.hip) with AddressSanitizer and UndefinedBehaviorSanitizer on the host
    side only, linked with the ordinary kernel objects and the scenario driver tests/native/host_sanitize_check.cpp.
    Uses the kernel objects build() leaves in _build/ (and runs it first if they are not there)."""
    objdir = os.path.join(HERE, "_build")
    if not all(os.path.exists(os.path.join(objdir, n)) for _, _, n in UNITS):
        build()
    hipcc = _hipcc()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    host_obj = os.path.join(objdir, "tkv_host_san.o")
    drv_obj = os.path.join(objdir, "host_sanitize_check.o")
    drv_src = os.path.join(os.path.dirname(HERE), "tests", "native", "host_sanitize_check.cpp")
    for cmd in ([hipcc, *FLAGS, "-g", *san, "-c", os.path.join(CSRC, "tkv_host.hip"), "-o", host_obj],
                [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", *san, "-x", "hip", "-c", drv_src, "-o", drv_obj]):
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + r.stderr)
    objs = [os.path.join(objdir, n) for _, _, n in UNITS if n != "tkv_host.o"]
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                        drv_obj, host_obj, *objs, "-o", HOST_CHECK], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(HOST_CHECK, file=sys.stderr)
    return HOST_CHECK


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_host_check(verbose=True))
