"""Build the HIP library (libmux.so) in-tree for gfx950 with hipcc.

`python -m paper_2404_02015_amd.build` or `build()` compiles every source under csrc/
(device code for gfx950 only) and links paper_2404_02015_amd/libmux.so.  hipcc
cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OUT = os.path.join(PKG, "libmux.so")
OBJ_DIR = os.path.join(ROOT, "_build")

SOURCES = ["mux_api.cpp", "mux_sched.cpp", "mux_stream.cpp", "mux_estimator.cpp", "mux_probes.hip", "mux_runner.hip", "mux_kv_append.hip", "mux_decode_attn.hip", "mux_prefill_attn.hip", "mux_static_scratch.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-inline-asm", "-fvisibility=hidden",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + FLAGS + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stderr))
    noise = "is not a recognized feature for this target"
    warn = "\n".join(l for l in r.stderr.splitlines() if l.strip() and noise not in l)
    if warn.strip():
        sys.stderr.write(warn + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = OUT + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s" % r.stderr)
    os.replace(tmp, OUT)
    if verbose:
        print("built", OUT)
    build_demo(verbose)
    return OUT


DEMO_SRC = os.path.join(PKG, "examples", "c_abi_demo.cpp")
DEMO = os.path.join(PKG, "examples", "c_abi_demo")


def build_demo(verbose: bool = True) -> str:
    """A small host program that uses the library through include/mux.h alone (run by the GPU tests)."""
    cmd = [HIPCC, "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wall", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I" + os.path.join(ROOT, "include"), DEMO_SRC,
           "-o", DEMO, "-L" + PKG, "-lmux", "-Wl,-rpath,$ORIGIN/.."]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for the C ABI demo:\n%s" % r.stderr)
    if verbose:
        print("built", DEMO)
    return DEMO


def is_stale() -> bool:
    if not os.path.exists(OUT):
        return True
    t = os.path.getmtime(OUT)
    if not os.path.exists(DEMO):
        return True
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "mux.h"), DEMO_SRC]
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    build()
