"""Builds the HIP library in-tree: paper_1705_07860_amd/libob.so (gfx950 only).

`python -m paper_1705_07860_amd.build` or `build()`; hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libob.so"
SOURCES = ["ob_prims.hip", "ob_sched.hip", "ob_exec.hip", "ob_api.hip"]
HEADERS = ["ob_internal.h", "ob_ctx.h", "../../include/ob.h"]

# Packed fp32 instructions are switched off for all device code (the compiler would otherwise
# form them from ordinary float arithmetic).
# Leading scalar and pointer kernel arguments are preloaded into scalar registers at wave start
# (the step kernels put what they need first there), so their first loads do not wait for a
# read of the argument block.
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-kernarg-preload-count=16"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def build(force: bool = True, verbose: bool = False) -> Path:
    """Compiles every source to an object and links the shared library.  With force=False an
    up-to-date library is kept."""
    srcs = [CSRC / s for s in SOURCES]
    deps = srcs + [(CSRC / h).resolve() for h in HEADERS]
    if not force and LIB.exists() and all(LIB.stat().st_mtime >= d.stat().st_mtime for d in deps):
        return LIB
    if LIB.exists():
        LIB.unlink()    # a failed build must not leave an older library behind to be loaded by mistake
    objdir = HERE / "_build"
    objdir.mkdir(exist_ok=True)
    procs = []
    objs = []
    for s in srcs:
        o = objdir / (s.stem + ".o")
        objs.append(o)
        cmd = [_hipcc(), *FLAGS, "-c", str(s), "-o", str(o)]
        if verbose:
            print(" ".join(cmd))
        procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for s, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0 or verbose:
            sys.stderr.write(out)
        elif out.strip():
            # keep real warnings visible, drop the host pass's note about the unknown target feature
            lines = [ln for ln in out.splitlines() if "packed-fp32-ops" not in ln]
            if any("warning" in ln or "error" in ln for ln in lines):
                sys.stderr.write("\n".join(lines) + "\n")
        failed |= p.returncode != 0
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", *map(str, objs), "-o", str(LIB)]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
