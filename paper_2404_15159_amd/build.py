"""Build libmixlora.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2404_15159_amd.build

Cross-compiles without a GPU.  Objects go to csrc/_build/ (git-ignored); the shared library is
written next to this file, where binding.py looks for it.
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libmixlora.so")
SOURCES = ("gemm.hip", "router.hip", "elementwise.hip", "grads.hip", "fused.hip", "fused_pg.hip", "probe.hip",
           "linear.hip", "optim.hip", "dora.hip", "prof.hip", "api.hip")

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # packed fp32 VALU forms are not to be generated on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str, obj: str) -> None:
    cmd = [hipcc(), *FLAGS, "-c", src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")


def build(verbose: bool = True) -> str:
    bdir = os.path.join(CSRC, "_build")
    os.makedirs(bdir, exist_ok=True)
    jobs = [(os.path.join(CSRC, s), os.path.join(bdir, s.replace(".hip", ".o"))) for s in SOURCES]
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        for fut in [ex.submit(_compile, s, o) for s, o in jobs]:
            fut.result()
    tmp = OUT + ".tmp"
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [o for _, o in jobs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    os.replace(tmp, OUT)
    if verbose:
        print(f"built {OUT} ({os.path.getsize(OUT) >> 10} KiB)")
    return OUT


if __name__ == "__main__":
    build()
