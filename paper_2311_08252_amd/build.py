"""Compiles the HIP sources in csrc/ into librest_gfx950.so next to this file (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librest_gfx950.so")
# the same sources with -DREST_BOUNDS_CHECK: data- and plan-dependent indices are clamped into their arrays and a
# violation makes the call return REST_BOUNDS_VIOLATION (the parity suite runs under it with REST_LIBRARY=checked)
LIB_CHECKED = os.path.join(HERE, "librest_gfx950_checked.so")
SOURCES = ["api.hip", "attention.hip", "retrieve.hip", "accept.hip", "build_index.hip", "kvcache.hip", "sample.hip", "index_io.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# per-source extras: keep the MFMA accumulators of the attention kernel in ordinary vector registers; the
# compiler's default choice shuttles all 128 of them through the accumulation file on every loop trip
# sampling: the definition of a token's weight is a fixed sequence of separately rounded fp64 operations, so no
# multiplication may be fused with an addition there
EXTRA = {"attention.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"], "sample.hip": ["-ffp-contract=off"]}


def build(verbose: bool = False, checked: bool = False) -> str:
    objs = []
    procs = []
    bdir = os.path.join(HERE, "_build", "checked" if checked else "product")
    os.makedirs(bdir, exist_ok=True)
    lib = LIB_CHECKED if checked else LIB
    for src in SOURCES:
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        cmd = ["hipcc", "-c", os.path.join(CSRC, src), "-o", obj] + [f for f in FLAGS if f != "-shared"] + EXTRA.get(src, [])
        if checked:
            cmd.append("-DREST_BOUNDS_CHECK")
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(ln for ln in out.splitlines() if "packed-fp32-ops" not in ln)
        if pr.returncode != 0:
            failed = True
            sys.stderr.write(f"[build] {src} failed:\n{out}\n")
        elif verbose and out.strip():
            sys.stderr.write(f"[build] {src}:\n{out}\n")
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs)
    return lib


if __name__ == "__main__":
    print(build(verbose=True))
    print(build(verbose=True, checked=True))
