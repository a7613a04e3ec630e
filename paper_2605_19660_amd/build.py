"""Build the HIP library in-tree for gfx950:  python -m paper_2605_19660_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "liboscar_hip.so")

COMMON = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
          # packed fp32 VALU forms are kept out of every device code object
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-command-line-argument"]
# per-file extras: the encoder's fp32 operation order is part of the format
SOURCES = {
    "oscar_api.hip": [],
    "oscar_quantize.hip": ["-ffp-contract=off"],
    "oscar_quantize_allheads.hip": ["-ffp-contract=off"],
    "oscar_quantize_switched.hip": ["-ffp-contract=off"],
    "oscar_decode.hip": [],
    "oscar_decode_mfma.hip": [],
    "oscar_decode_mfma_zpmin.hip": [],
    "oscar_bf16_decode.hip": [],
    "oscar_probe.hip": [],
}


def _compile(name: str, extra: list[str], verbose: bool, tag: str = "") -> str:
    src = os.path.join(CSRC, name)
    obj = os.path.join(OBJ, name.replace(".hip", tag + ".o"))
    cmd = ["hipcc", *COMMON, *extra, "-c", src, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {name}:\n{err}")
    if verbose and err.strip():
        print(err, flush=True)
    return obj


def _link(lib: str, objs: list[str], verbose: bool) -> str:
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return lib


def build(verbose: bool = False, jobs: int = 6) -> str:
    os.makedirs(OBJ, exist_ok=True)
    present = {n: e for n, e in SOURCES.items() if os.path.exists(os.path.join(CSRC, n))}
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda kv: _compile(kv[0], kv[1], verbose), present.items()))
    return _link(LIB, objs, verbose)


# The same library with phase time stamps in the matrix-core decode kernel (phase_profile.py):
# only the two translation units of that kernel are compiled again.
STAMPED = ("oscar_decode_mfma.hip", "oscar_decode_mfma_zpmin.hip")
LIB_STAMPS = os.path.join(HERE, "liboscar_hip_stamps.so")


def build_stamps(verbose: bool = False, jobs: int = 6) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(
            lambda kv: _compile(kv[0], kv[1] + ["-DOSCAR_DECODE_STAMPS"], verbose, "_stamps")
            if kv[0] in STAMPED else _compile(kv[0], kv[1], verbose), SOURCES.items()))
    return _link(LIB_STAMPS, objs, verbose)


if __name__ == "__main__":
    quiet = "-q" in sys.argv
    print(build_stamps(verbose=not quiet) if "--stamps" in sys.argv else build(verbose=not quiet))
