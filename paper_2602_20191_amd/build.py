"""Builds libmbq.so (HIP, gfx950) in-tree with hipcc.  Run: python -m paper_2602_20191_amd.build"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmbq.so")
OBJ_DIR = os.path.join(HERE, "_build")

SOURCES = [
    # (file, extra flags)
    ("mbq_api.hip", []),
    ("mbq_encode.hip", ["-ffp-contract=off"]),   # the code recursion is specified unfused
    ("mbq_route.hip", ["-ffp-contract=off"]),
    ("mbq_act.hip", ["-ffp-contract=off"]),      # every step of the activation quantiser is one fp32 operation
    ("mbq_linear_simple.hip", []),
    ("mbq_linear_decode.hip", []),
    ("mbq_linear_decode16.hip", []),
    ("mbq_linear_decode_f4.hip", []),
    ("mbq_linear_decode_f4_ws.hip", []),
    ("mbq_linear_prefill.hip", []),
    ("mbq_bench.hip", []),
]

COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-DMBQ_BUILDING=1",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "is not a recognized feature for this target" not in l)
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False, save_temps: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    cc = hipcc()
    objs = []
    jobs = []
    for src, extra in SOURCES:
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [cc] + COMMON + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
        if save_temps:
            cmd += ["-save-temps=obj"]
        jobs.append(cmd)
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as pool:
        for out in pool.map(_run, jobs):
            if verbose and out.strip():
                print(out)
    _run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    path = build(verbose=True, save_temps="--save-temps" in sys.argv)
    print("built", path)
