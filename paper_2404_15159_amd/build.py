"""Build libmixlora.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2404_15159_amd.build

Cross-compiles without a GPU.  Objects go to csrc/_build/ (git-ignored); the shared library is
written next to this file, where binding.py looks for it.

    python -m paper_2404_15159_amd.build --sanitize-host

builds a second library, csrc/_build/san/libmixlora_san.so, whose HOST code carries
AddressSanitizer and UndefinedBehaviorSanitizer checks (the device code is unchanged), for the
CPU-only argument and layout tests:

    MIXLORA_LIB=paper_2404_15159_amd/csrc/_build/san/libmixlora_san.so \
    LD_PRELOAD=$(/opt/rocm/lib/llvm/bin/clang -print-file-name=libclang_rt.asan-x86_64.so) \
    ASAN_OPTIONS=detect_leaks=0:verify_asan_link_order=0 python -m pytest tests/test_abi_cpu.py
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


SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def _compile(src: str, obj: str, extra=()) -> None:
    cmd = [hipcc(), *FLAGS, *extra, "-c", src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")


def build(verbose: bool = True, sanitize_host: bool = False) -> str:
    bdir = os.path.join(CSRC, "_build", "san") if sanitize_host else os.path.join(CSRC, "_build")
    out = os.path.join(bdir, "libmixlora_san.so") if sanitize_host else OUT
    extra = SAN_FLAGS if sanitize_host else []
    os.makedirs(bdir, exist_ok=True)
    jobs = [(os.path.join(CSRC, s), os.path.join(bdir, s.replace(".hip", ".o"))) for s in SOURCES]
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        for fut in [ex.submit(_compile, s, o, extra) for s, o in jobs]:
            fut.result()
    tmp = out + ".tmp"
    link_extra = ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"] if sanitize_host else []
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *link_extra, "-o", tmp] + [o for _, o in jobs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    os.replace(tmp, out)
    if verbose:
        print(f"built {out} ({os.path.getsize(out) >> 10} KiB)")
    return out


if __name__ == "__main__":
    build(sanitize_host="--sanitize-host" in sys.argv[1:])
