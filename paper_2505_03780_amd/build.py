"""Build the HIP library for gfx950: one hipcc process per translation unit, then a link.

Run as ``python -m paper_2505_03780_amd.build`` or through ``__graft_entry__.build()``.
hipcc cross-compiles without a GPU.  The shared object lands next to this file so that
it travels with the source tree.
"""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libattn_gfx950.so")
SOURCES = ["attn_api.hip", "prefill_f32.hip", "prefill_bf16.hip", "prefill_bf16_ring.hip", "prefill_f16_ring.hip", "prefill_f16.hip", "decode_bf16.hip", "decode_f16.hip", "rmsnorm.hip", "kv_write.hip"]
# the benchmark's measurement aids: a library of their own, outside the attention ABI
PROBE_LIB = os.path.join(HERE, "libprobe_gfx950.so")
# Packed fp32 instructions (v_pk_fma_f32 and friends) are switched off on purpose: some of their forms
# have given wrong results on this hardware, and the kernels do not depend on them.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# The MFMA kernels never do arithmetic on NaN (garbage rows are replaced by selects before any use),
# so the compiler may skip the canonicalising v_max it otherwise puts in front of every fmaxf.
EXTRA = {"prefill_bf16_ring.hip": ["-fno-honor-nans"], "prefill_f16_ring.hip": ["-fno-honor-nans"]}


def _compile(src: str) -> str:
    obj = os.path.join(BUILD, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stderr[-4000:]))
    return obj


def build(verbose: bool = False) -> str:
    """Build the library."""
    os.makedirs(BUILD, exist_ok=True)
    lib = LIB
    with cf.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = lib + ".tmp.%d" % os.getpid()
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr[-4000:])
    os.replace(tmp, lib)
    probe_obj = _compile("probe.hip")
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PROBE_LIB + ".tmp", probe_obj], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr[-4000:])
    os.replace(PROBE_LIB + ".tmp", PROBE_LIB)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
