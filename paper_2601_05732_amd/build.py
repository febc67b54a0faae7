"""Builds libmhcl.so (HIP, gfx950 only) next to this file with hipcc, and the stand-alone
memory-system probe (probe/memsys_probe.hip -> memsys_probe) that `bench.py --memsys` runs."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libmhcl.so")
OBJ_DIR = os.path.join(_HERE, "_build")
PROBE_SRC = os.path.join(_HERE, "probe", "memsys_probe.hip")
PROBE = os.path.join(_HERE, "memsys_probe")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # hipcc -O3 may otherwise fuse scalar fp32 code into packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def build_library(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(OBJ_DIR, os.path.basename(s) + ".o") for s in srcs]

    def compile_one(pair):
        src, obj = pair
        cmd = [HIPCC, *FLAGS, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        return src, r

    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        for src, r in ex.map(compile_one, zip(srcs, objs)):
            # the host pass warns that it does not know the packed-fp32 feature: harmless
            err = "\n".join(l for l in r.stderr.splitlines()
                            if "packed-fp32-ops" not in l and l.strip())
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
            if err and verbose:
                print(err, file=sys.stderr)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    build_probe(verbose)
    return LIB


def build_probe(verbose: bool = False) -> str:
    """The traffic-skeleton executable (no part of the library; it links nothing of it)."""
    cmd = [HIPCC, *[f for f in FLAGS if f != "-fPIC"], PROBE_SRC, "-o", PROBE]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {PROBE_SRC}:\n{r.stderr}")
    return PROBE


if __name__ == "__main__":
    print(build_library(verbose=True))
