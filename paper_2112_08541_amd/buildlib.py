"""Build the HIP library (libbgl.so, gfx950) and the input generator in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(_ROOT, "include")
LIB = os.path.join(_HERE, "libbgl.so")
HIP_SOURCES = ["bgl_api.hip", "bgl_sample.hip", "bgl_cache.hip", "bgl_host_tier.hip", "bgl_order.hip", "bgl_pipeline.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # keep hipcc from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I" + INCLUDE, "-I" + CSRC,
]


def build_hip(verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 and link libbgl.so (always recompiles)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in HIP_SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        text = out.decode()
        # the host pass does not know the packed-fp32 feature name; that warning is expected
        text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"--- {src} ---\n{text}\n")
        elif verbose and text.strip():
            print(text)
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


def build_all(verbose: bool = False) -> None:
    from . import inputs, policy_study
    inputs.build(force=True)
    policy_study.build(force=True)
    build_hip(verbose)


if __name__ == "__main__":
    build_all(verbose=True)
    print("built", LIB)
