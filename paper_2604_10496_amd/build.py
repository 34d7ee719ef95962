"""Builds libcq.so (the C-ABI library, gfx950 only) in-tree with hipcc.

    python -m paper_2604_10496_amd.build        # compile every .hip under csrc/ and link

hipcc cross-compiles without a GPU.  Objects go to _build/ (git-ignored); the shared library is
written next to this file so that it travels with the source tree.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(ROOT, "include")
BUILD_DIR = os.path.join(ROOT, "_build")
LIB_PATH = os.path.join(PKG_DIR, "libcq.so")

HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", INCLUDE, "-I", CSRC,
]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _stale(src: str, obj: str) -> bool:
    if not os.path.exists(obj):
        return True
    deps = [os.path.join(CSRC, src), os.path.join(INCLUDE, "cq.h"), os.path.join(INCLUDE, "cq_measure.h")]
    deps += [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    return any(os.path.getmtime(d) > os.path.getmtime(obj) for d in deps)


def _split_resource_remarks(lines):
    """Separates hipcc's kernel-resource-usage remarks ({kernel: {field: value}}) from its other output."""
    usage, rest, cur, skip, held = {}, [], None, 0, []
    for l in lines:
        if skip:                      # the two source-excerpt lines clang prints under a remark
            skip -= 1
            continue
        if l.startswith("In file included from"):   # belongs to the diagnostic that follows
            held.append(l)
            continue
        if "[-Rpass-analysis=kernel-resource-usage]" not in l:
            rest.extend(held)
        held = []
        if "[-Rpass-analysis=kernel-resource-usage]" in l:
            body = l.split("remark:", 1)[1].rsplit("[-Rpass-analysis", 1)[0].strip()
            if body.startswith("Function Name:"):
                cur = body.split(":", 1)[1].strip()
                usage[cur] = {}
                skip = 2
            elif cur is not None and ":" in body:
                k, v = body.rsplit(":", 1)
                try:
                    usage[cur][k.strip()] = int(v)
                except ValueError:
                    pass
            continue
        rest.append(l)
    return usage, rest


def _compile(src: str, force: bool = True) -> str:
    obj = os.path.join(BUILD_DIR, src[:-4] + ".o")
    if not force and not _stale(src, obj):
        return obj
    cmd = [HIPCC, *FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    lines = [l for l in res.stderr.splitlines() if noise not in l]
    usage, err = _split_resource_remarks(lines)
    err = "\n".join(err)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    # Kernels that issue register loads from inline assembly and wait for them later (cq_async.h) must not spill:
    # a spill or reload of a register with a load in flight would store or restore a stale value.
    with open(os.path.join(CSRC, src)) as f:
        if "cq_async.h" in f.read():
            bad = [(k, u) for k, u in usage.items() if u.get("VGPRs Spill", 0) or u.get("ScratchSize [bytes/lane]", 0)]
            if bad:
                if os.path.exists(obj):
                    os.remove(obj)
                raise RuntimeError(f"{src}: kernels with asynchronous register loads spill: {bad}")
    if err.strip():
        print(err, file=sys.stderr)
    return obj


def build_library(verbose: bool = True, force: bool = True) -> str:
    """force=False recompiles only sources older than their object (development); the default compiles all."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as pool:
        objs = list(pool.map(lambda s: _compile(s, force), sources()))
    # no rpath to a particular ROCm: when torch is imported first its HIP runtime (same soname) is
    # already mapped and is the one this library binds to, so streams and pointers are shared.
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", LIB_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    if verbose:
        print(f"built {LIB_PATH}")
    return LIB_PATH


if __name__ == "__main__":
    build_library(force="--changed" not in sys.argv)
