"""Build libgoom.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgoom.so")
SOURCES = ["goom_api.hip", "goom_codec.hip", "goom_chain.hip", "goom_reset.hip", "goom_lmme_exact.hip", "goom_chain_f32_goom.hip",
           "goom_chain_f32_fact.hip", "goom_chain_f64_goom.hip", "goom_chain_f64_fact.hip", "goom_chain_f64_io32.hip", "goom_affine.hip", "goom_large.hip", "goom_large_f64.hip", "goom_lmme128.hip", "goom_chain256.hip", "goom_chain_small.hip", "goom_chain_ragged.hip", "goom_backward.hip", "goom_lmme_backward.hip", "goom_scan_backward.hip", "goom_lmme_tall.hip", "goom_affine_seq.hip"]
HEADERS = ["goom_internal.h", "goom_chain_kernel.h", "goom_chain_fast.h", "goom_codec_tables.h", "goom_large_scan.h", os.path.join("..", "..", "include", "goom.h")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    # packed fp32 instructions are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def _stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return any(os.path.getmtime(p) > t for p in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    """Compile every source and link the shared library.  Returns its path."""
    if not force and not _stale():
        return LIB
    objs = []
    procs = []
    for s in SOURCES:
        o = os.path.join(CSRC, s.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, "-DGOOM_BUILDING", "-c", os.path.join(CSRC, s), "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(o)
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
        if verbose and out.strip():
            print(out)
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
