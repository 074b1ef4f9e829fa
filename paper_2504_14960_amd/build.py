"""Build libmoe_hip.so (gfx950) in-tree with hipcc.

    python -m paper_2504_14960_amd.build [--force]
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoe_hip.so")
SOURCES = ["api.hip", "router.hip", "permute.hip", "combine.hip", "grouped_gemm.hip", "gemm_pipe3.hip", "gemm_persist.hip", "gemm_persist_fp8.hip", "fp8_quant.hip", "ffn_backward.hip", "router_backward.hip", "probe.hip", "chunks.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # packed-fp32 VALU forms are switched off on this fleet
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]


def _deps(src: str):
    """Every header of csrc/ counts for every object: the sources include them in changing combinations,
    and a stale object is worse than a few seconds of rebuilding."""
    yield os.path.join(CSRC, src)
    for name in sorted(os.listdir(CSRC)):
        if name.endswith(".h"):
            yield os.path.join(CSRC, name)
    yield os.path.join(HERE, "..", "include", "moe.h")


def stale_sources():
    """Sources and headers newer than the built library (empty when the library is up to date)."""
    if not os.path.exists(LIB):
        return ["libmoe_hip.so is missing"]
    t = os.path.getmtime(LIB)
    files = [os.path.join(CSRC, n) for n in sorted(os.listdir(CSRC)) if n.endswith((".h", ".hip"))]
    files.append(os.path.join(HERE, "..", "include", "moe.h"))
    return [os.path.relpath(f, HERE) for f in files if os.path.getmtime(f) > t]


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in _deps(src)):
        return obj
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError(f"hipcc failed on {src}")
    warn = [ln for ln in r.stderr.splitlines() if "packed-fp32-ops" not in ln and ln.strip()]
    if warn:
        sys.stderr.write("\n".join(warn) + "\n")
    return obj


def build(force: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(len(SOURCES)) as pool:
        objs = list(pool.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB + ".tmp", *objs]
        subprocess.run(cmd, check=True)
        os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
