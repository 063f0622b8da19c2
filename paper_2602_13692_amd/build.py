"""Builds the HIP library for gfx950 with hipcc (in-tree, next to this file)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libta_hip.so")
SOURCES = ["ta_api.hip", "ta_decode.hip", "ta_decode_fp8.hip", "ta_prefill.hip", "ta_restore.hip", "ta_sched.cpp", "ta_sim.cpp"]
# measurement aids of the benchmark: a library of their own, nothing of the hot path is in it
PROBE_LIB = os.path.join(HERE, "libta_probe.so")
PROBE_SOURCES = ["ta_probe.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
    # packed fp32 VALU forms stay off for every kernel in this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # matrix-core results that vector instructions consume (the attention scores) are written to
    # vector registers directly instead of accumulation registers plus a copy per value
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every HIP source into libta_hip.so (and the probes into libta_probe.so); raises on failure."""
    _compile(SOURCES, LIB, verbose, extra_flags)
    _compile(PROBE_SOURCES, PROBE_LIB, verbose, extra_flags)
    return LIB


def _run(cmd, verbose) -> None:
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    out = "\n".join(l for l in res.stdout.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def _compile(sources, lib, verbose, extra_flags) -> str:
    """One object per source (compiled side by side), then one link."""
    from concurrent.futures import ThreadPoolExecutor

    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    flags = [f for f in FLAGS if f != "-shared"]
    objs = [os.path.join(obj_dir, os.path.splitext(s)[0] + ".o") for s in sources]
    cmds = [["hipcc", *flags, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c",
             os.path.join(CSRC, s), "-o", o] for s, o in zip(sources, objs)]
    with ThreadPoolExecutor(max_workers=min(len(cmds), 8)) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden", *objs, "-o", lib], verbose)
    return lib


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
