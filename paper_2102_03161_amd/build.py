"""Builds libpt.so (the C-ABI library) from csrc/*.hip for gfx950 with hipcc.

Usage: python -m paper_2102_03161_amd.build [--force]
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpt.so")
SOURCES = ["gemm.hip", "gemm_dma.hip", "attention.hip", "attention_mfma.hip", "rowops.hip", "optim.hip", "pt.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-Wall", "-Wno-unused-function",
         # keep fp32 vector math scalar per lane: no packed-fp32 instruction selection
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# Per-file additions.  The attention kernels keep long-lived MFMA accumulators next to short-lived score tiles;
# with the default AGPR form of the MFMA result the compiler shuttles the long-lived ones between register
# files every iteration, so these kernels are built with MFMA results in ordinary VGPRs.
EXTRA_FLAGS = {"attention_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def _compile(src: str, obj: str) -> None:
    cmd = [_hipcc(), *FLAGS, *EXTRA_FLAGS.get(os.path.basename(src), []), "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")


def build(force: bool = True, jobs: int = 4) -> str:
    """Compiles every source (always, unless force=False and the library is newer than all inputs)."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    deps = srcs + [os.path.join(CSRC, h) for h in ("common.h", "kernels.h", "gemm_epilogue.h", "ln_bwd_rows.h", "libpt.map")] + [os.path.join(HERE, "..", "include", "pt.h")]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    objs = [os.path.join(objdir, os.path.basename(s) + ".o") for s in srcs]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(lambda a: _compile(*a), zip(srcs, objs)))
    r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC",
                        "-Wl,--version-script=" + os.path.join(CSRC, "libpt.map"), "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv or True))
