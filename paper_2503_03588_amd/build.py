"""Builds libpowattn.so (the C-ABI library) for gfx950 with hipcc, in-tree.

Run as `python -m paper_2503_03588_amd.build`.  Every .hip file under csrc/ is
compiled to an object in csrc/_build/ and the objects are linked into
paper_2503_03588_amd/libpowattn.so.
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libpowattn.so")
ARCH = "gfx950"

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", f"--offload-arch={ARCH}",
    "-Wall", "-Wno-unused-function",
    # the asynchronous-copy helpers name M0 as clobbered; the compiler notes that it is a reserved register
    # (one it never hands out itself), which is the point of naming it
    "-Wno-inline-asm",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the prefill step is one fully unrolled instruction stream of 32 matrix instructions; the default size
    # limit for loops with an unroll pragma is too small for it
    "-mllvm", "-pragma-unroll-threshold=200000",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str, obj: str, extra) -> None:
    cmd = [hipcc(), *HIPCC_FLAGS, *extra, "-c", src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{res.stdout}\n{res.stderr}")
    noise = "'-packed-fp32-ops' is not a recognized feature"
    for line in res.stderr.splitlines():
        if line.strip() and noise not in line:
            print(line, file=sys.stderr)


def build(verbose: bool = True, extra_flags=()) -> str:
    """Compile and link unconditionally; returns the path of the library."""
    bdir = os.path.join(CSRC, "_build")
    os.makedirs(bdir, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(bdir, os.path.basename(s)[:-4] + ".o") for s in srcs]
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
        futs = [pool.submit(_compile, s, o, list(extra_flags)) for s, o in zip(srcs, objs)]
        for f in futs:
            f.result()
    tmp = OUT + ".tmp"
    cmd = [hipcc(), "-shared", "-fPIC", f"--offload-arch={ARCH}", *objs, "-o", tmp]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}\n{res.stderr}")
    os.replace(tmp, OUT)
    if verbose:
        print(f"built {OUT} from {len(srcs)} sources")
    return OUT


def build_microbench(verbose: bool = True):
    """The two machine micro-benchmarks (stand-alone executables that bench.py runs for its `measured_peaks`)."""
    mdir = os.path.join(HERE, "microbench")
    bdir = os.path.join(mdir, "bin")
    os.makedirs(bdir, exist_ok=True)
    outs = []
    for name in ("mfma_peak", "stream_decode"):
        out = os.path.join(bdir, name)
        cmd = [hipcc(), "-O3", "-std=c++17", f"--offload-arch={ARCH}", "-Wno-unused-value", "-Wno-unused-result",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               os.path.join(mdir, name + ".hip"), "-o", out]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed for {name}:\n{res.stdout}\n{res.stderr}")
        outs.append(out)
    if verbose:
        print(f"built {len(outs)} micro-benchmarks in {bdir}")
    return outs


if __name__ == "__main__":
    build()
    build_microbench()
