"""Builds libmcr.so (the C-ABI library) from csrc/ with hipcc for gfx950.

    python -m paper_2303_08374_amd.build [--changed]
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmcr.so")
OBJ_DIR = os.path.join(HERE, "_build")

# the reductions' kernels are instantiated per element type, the slowest units first
SOURCES = ["mcr_allreduce_f32.hip", "mcr_allreduce_bf16.hip", "mcr_reduce_scatter_f32.hip", "mcr_reduce_scatter_bf16.hip",
           "mcr_fuse.hip", "mcr_allreduce_f16.hip", "mcr_allreduce_i32.hip", "mcr_reduce_scatter_f16.hip",
           "mcr_reduce_scatter_i32.hip", "mcr_copy.hip", "mcr_fused.hip", "mcr_moe.hip", "mcr_allreduce.hip",
           "mcr_reduce_scatter.hip", "mcr_api.hip"]

# -packed-fp32-ops is switched off on purpose: the compiler otherwise forms packed
# binary32 instructions from ordinary float code.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the device-only target feature and says so: harmless
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out.strip():
        print(out, file=sys.stderr)
    return obj


def _up_to_date(src: str) -> bool:
    """The object is newer than the source, every header next to it and the public header."""
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    if not os.path.exists(obj):
        return False
    deps = [os.path.join(CSRC, src), os.path.join(HERE, "..", "include", "mcr.h")]
    deps += [os.path.join(CSRC, h) for h in os.listdir(CSRC) if h.endswith(".hpp")]
    return all(os.path.getmtime(d) < os.path.getmtime(obj) for d in deps)


def build(jobs: int = 8, only_changed: bool = False) -> str:
    """Compiles every source (only_changed: every source whose object is out of date) and links."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    todo = [s for s in SOURCES if not (only_changed and _up_to_date(s))]
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(_compile, todo))
    objs = [os.path.join(OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(only_changed="--changed" in sys.argv[1:]))
