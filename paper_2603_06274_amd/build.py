"""Builds libstem_hip.so (the C-ABI library) for gfx950 with hipcc, in-tree.

Run as `python -m paper_2603_06274_amd.build`.  Cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libstem_hip.so")

SOURCES = ["stem_api.cpp", "stem_pool.hip", "stem_scores.hip", "stem_select.hip", "stem_attn.hip", "stem_static.hip"]

# -packed-fp32-ops: keep the compiler from forming v_pk_*_f32 out of plain float code.
COMMON = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-I" + os.path.join(ROOT, "include"),
          "-I" + CSRC, "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wall", "-Wno-unused-command-line-argument"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc(), *COMMON, *extra, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, res.stdout, res.stderr))
    warnings = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if warnings.strip():
        sys.stderr.write(warnings + "\n")
    return obj


def check_wait_states(extra=()) -> None:
    """The attention kernel places some matrix instructions (and the wait states they need) by hand:
    compile it to assembly once more and verify the distances in what the compiler made of it."""
    from . import wait_states
    asm_path = os.path.join(OBJ, "stem_attn.s")
    cmd = [hipcc(), *COMMON, *extra, "--cuda-device-only", "-S", "-x", "hip", os.path.join(CSRC, "stem_attn.hip"),
           "-o", asm_path]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc -S failed for stem_attn.hip:\n%s\n%s" % (res.stdout, res.stderr))
    with open(asm_path) as f:
        asm = f.read()
    names = wait_states.kernels(asm, "sparse_attn_kernel")
    if len(names) < 6:
        raise RuntimeError("expected the six attention kernels in %s, found %d" % (asm_path, len(names)))
    for name in names:
        broken = wait_states.check_kernel(asm, name)
        if broken:
            raise RuntimeError("wait states missing in %s:\n  %s" % (name, "\n  ".join(broken[:20])))


def build(extra_flags=(), verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        checked = ex.submit(check_wait_states, list(extra_flags))
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
        checked.result()
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (res.stdout, res.stderr))
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(sys.argv[1:])
