"""Builds libghd.so and the stream probe (gfx950) in-tree with hipcc.  Run as a module or call build()."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libghd.so")
PROBE = os.path.join(HERE, "ghd_stream_probe")       # measurement tool (bench.py --stream-probe), its own program
PROBE_SOURCE = "stream_probe.hip"
SOURCES = ["api.hip", "fused.hip", "linear.hip", "linear_mt1.hip", "linear_mt2.hip", "linear_mt4.hip",
           "linear_mt8.hip", "qkv_attn_mt1.hip", "qkv_attn_mt2.hip", "qkv_attn_mt4.hip", "qkv_attn_mt8.hip",
           "accept.hip", "draft.hip", "coo.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # keep the compiler from forming packed-fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # per-kernel register and scratch use, checked below
         "-Rpass-analysis=kernel-resource-usage", "-fno-caret-diagnostics"]
# The persistent kernels must not use scratch memory: a launch of a kernel that has a private
# segment costs several microseconds more here, whatever the kernel does with it.
NO_SCRATCH = ("k_linear", "k_qkv_attn", "k_attention")


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [_hipcc()] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    lines = r.stderr.splitlines()
    err = "\n".join(l for l in lines if "packed-fp32-ops" not in l and "kernel-resource-usage" not in l
                    and not l.startswith("In file included from"))
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    name = ""
    for l in lines:
        if "Function Name:" in l:
            name = l.split("Function Name:")[1].split()[0]
        elif "ScratchSize [bytes/lane]:" in l:
            size = int(l.split("ScratchSize [bytes/lane]:")[1].split()[0])
            if size and any(k in name for k in NO_SCRATCH):
                raise RuntimeError("%s: kernel %s uses %d bytes of scratch per lane" % (src, name, size))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    cmd = [_hipcc()] + [f for f in FLAGS if f != "-fPIC" and not f.startswith("-Rpass")] + ["-o", PROBE, os.path.join(CSRC, PROBE_SOURCE)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (PROBE_SOURCE, r.stderr))
    if verbose:
        print("built", LIB)
        print("built", PROBE)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
