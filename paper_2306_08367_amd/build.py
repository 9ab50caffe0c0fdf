"""Builds liblq.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblq.so")
OBJDIR = os.path.join(HERE, "_build")
SOURCES = ["lq_api.hip", "gemm.hip", "fused.hip", "fused_rowbatch.hip", "fused_rowbatch_wide_a.hip", "fused_rowbatch_wide_b.hip", "fused_rowbatch_wide_c.hip", "fused_rowbatch_wide_d.hip", "fused_coltile_a.hip", "fused_coltile_b.hip", "fused_coltile_c.hip", "fused_bf16.hip", "fused_tile.hip", "fused_deep.hip", "fused_deep_b.hip", "fused_deep_c.hip", "fused_deep_bf16.hip", "fused_lds.hip", "gather.hip", "yardstick.hip", "groupby.hip", "groupby_many.hip", "groupby_wide.hip", "groupby_agg_fast.hip", "tree.hip", "keymap.hip", "keymap64.hip", "domain.hip"]
ARCH = "gfx950"
# Packed-fp32 instruction selection is switched off for all device code.
FLAGS = ["-O3", "-std=c++17", "-fPIC", f"--offload-arch={ARCH}", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP library cannot be built")
    return exe


def _fresh(obj: str, src: str) -> bool:
    """True when `obj` is newer than its source and every header it may include."""
    if not os.path.exists(obj):
        return False
    t = os.path.getmtime(obj)
    deps = [os.path.join(CSRC, src), os.path.abspath(__file__)]
    deps += [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    inc = os.path.join(ROOT, "include")
    deps += [os.path.join(inc, f) for f in os.listdir(inc)]
    return all(os.path.getmtime(d) < t for d in deps)


def _compile(src: str, only_changed: bool = False) -> str:
    obj = os.path.join(OBJDIR, os.path.splitext(src)[0] + ".o")
    if only_changed and _fresh(obj, src):
        return obj
    cmd = [hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # hipcc's host pass warns that it does not know the packed-fp32 feature: harmless.
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True, only_changed: bool = False) -> str:
    """Compile every source and link liblq.so.  Rebuilds everything unless `only_changed` is set
    (a developer's shortcut: objects newer than their source and all headers are kept)."""
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda src: _compile(src, only_changed), SOURCES))
    cmd = [hipcc(), "-shared", "-fPIC", f"--offload-arch={ARCH}", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build(only_changed="--changed" in sys.argv[1:])
