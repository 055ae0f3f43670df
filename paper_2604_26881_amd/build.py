"""Builds libmoe_hip.so (the gfx950 kernels and the C entry points) in-tree with hipcc."""
from __future__ import annotations

import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

try:
    from . import mfma_hazards
except ImportError:      # run as a script
    import mfma_hazards

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libmoe_hip.so")
OBJDIR = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "route.hip", "permute.hip", "combine.hip", "expert_tile.hip", "expert_stream_lds.hip", "mfma_probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # the global->LDS copy sets m0 itself (the instruction takes its LDS address from there); the compiler
         # reports every such asm statement because it does not track m0 across inline asm
         "-Wno-inline-asm",
         # packed-fp32 instructions are switched off for all device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def source_id() -> str:
    """SHA-256 over the library's sources (csrc/ and the C headers), by file name and content.  The
    build stamps it into the library (moe_build_id); the binding refuses a library whose stamp is not
    the id of the sources beside it, and stored profiler counters carry the id of the kernels they
    were taken on."""
    h = hashlib.sha256()
    files = [os.path.join(CSRC, n) for n in sorted(os.listdir(CSRC))]
    files += [os.path.join(os.path.dirname(HERE), "include", n) for n in ("moe.h", "moe_tuning.h")]
    for path in files:
        with open(path, "rb") as f:
            h.update(os.path.basename(path).encode() + b"\0" + f.read())
    return h.hexdigest()


def _compile(src: str) -> str:
    stem = os.path.splitext(src)[0]
    obj = os.path.join(OBJDIR, stem + ".o")
    # -save-temps=obj leaves the device assembly beside the object: the MFMA kernels' own code is checked
    # for result registers touched before the matrix pipe has written them (mfma_hazards.py)
    cmd = [HIPCC, *FLAGS, "-save-temps=obj", "-c", os.path.join(CSRC, src), "-o", obj]
    if src == "api.hip":
        cmd.append(f'-DMOE_BUILD_ID="{source_id()}"')
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    asm = os.path.join(OBJDIR, f"{stem}-hip-amdgcn-amd-amdhsa-gfx950.s")
    if not os.path.exists(asm):
        raise RuntimeError(f"hipcc left no device assembly for {src} (expected {asm})")
    bad = mfma_hazards.check_file(asm)
    for n in os.listdir(OBJDIR):     # the other intermediate files are of no further use (several MB per source)
        if n.startswith(stem + "-") or n.startswith(stem + ".hip-"):
            os.remove(os.path.join(OBJDIR, n))
    if bad:
        raise RuntimeError(f"{src}: the emitted code touches MFMA results before they are written back:\n  " + "\n  ".join(bad))
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", OUT],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", OUT)
    return OUT


if __name__ == "__main__":
    build(verbose=True)
