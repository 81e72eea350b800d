"""Compile the HIP sources under csrc/ into libkvc_hip.so for gfx950 (in-tree).

hipcc cross-compiles without a GPU.  Run as ``python -m paper_2503_13773_amd.build``.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libkvc_hip.so")
SOURCES = ["kvc_api.hip", "kv_block_copy.hip", "kv_cache_append.hip", "paged_attention_valu.hip",
           "paged_attention_mfma.hip", "paged_attention_mfma_stream.hip", "paged_attention_prefill.hip", "paged_attention_prefill32.hip",
           "paged_attention_merge.hip"]
# packed-fp32 instructions are switched off on purpose for this target
# The atomic optimizer is switched off: it rewrites an atomic add issued by one lane into a
# wavefront-wide reduction that reads the result back at once, which makes the balanced
# attention kernel wait for its arrival counters instead of consuming tiles meanwhile.
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str, extra) -> str:
    obj = os.path.join(PKG, "_build", os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    return obj


def build_library(extra_flags=(), verbose: bool = False) -> str:
    os.makedirs(os.path.join(PKG, "_build"), exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print("built", LIB)
    return LIB


POLICY_LIB = os.path.join(PKG, "libkvc_policy.so")


def build_policy_library(verbose: bool = False, out: str = "", extra_flags=()) -> str:
    """The host-side policy core (plain C++, no GPU code).  `out` / `extra_flags` build a variant
    elsewhere (the sanitizer run of the CPU tests)."""
    target = out or POLICY_LIB
    cmd = ["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-fvisibility=hidden", "-Wall", "-Werror", *extra_flags,
           "-I", os.path.join(ROOT, "include"), os.path.join(CSRC, "policy", "kvc_policy.cpp"),
           "-o", target]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"g++ failed on kvc_policy.cpp:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print("built", target)
    return target


if __name__ == "__main__":
    build_library(sys.argv[1:], verbose=True)
    build_policy_library(verbose=True)
