"""Builds the HIP library in-tree: paper_2505_05950_amd/libfloe_hip.so (gfx950 only)."""
from __future__ import annotations

import concurrent.futures as fut
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfloe_hip.so")
SOURCES = ["api.hip", "quantize.hip", "up_gemv.hip", "up_gemv_mfma.hip", "fused_layer.hip", "fused_int2.hip", "fused_int3.hip", "fused_int4.hip", "select.hip", "gate_down.hip", "gate_down_union.hip", "variants.hip", "router.hip", "stage.hip", "prefetch.hip", "static_scratch.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


# Instrumented build for tuning: every kernel that carries FLOE_TL marks stores a clock value per workgroup and mark into
# a buffer handed over through floe_debug_set_timeline_* (see FLOE_TL in csrc/floe_dev.h).  A library of its own
# (libfloe_hip_timeline.so); the product library never contains the marks.
LIB_TIMELINE = os.path.join(HERE, "libfloe_hip_timeline.so")
OBJ_TIMELINE = os.path.join(HERE, "_build_timeline")


def _compile(src: str, timeline: bool = False) -> str:
    obj = os.path.join(OBJ_TIMELINE if timeline else OBJ, src.replace(".hip", ".o"))
    cmd = [HIPCC] + FLAGS + (["-DFLOE_TIMELINE"] if timeline else []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{res.stdout}\n{res.stderr}")
    return obj


def build(verbose: bool = False, timeline: bool = False) -> str:
    os.makedirs(OBJ_TIMELINE if timeline else OBJ, exist_ok=True)
    lib = LIB_TIMELINE if timeline else LIB
    with fut.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda src: _compile(src, timeline), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}\n{res.stderr}")
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    import sys
    build(verbose=True, timeline="--timeline" in sys.argv[1:])
