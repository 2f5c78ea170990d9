"""Builds libwpsgd.so (HIP, gfx950) in-tree with hipcc.

    python -m paper_1708_04801_amd.build          # rebuild everything

The register-resident chain kernel is compiled once per (row storage, loss) pair; all
translation units are compiled in parallel and linked into one shared library that exports the
C ABI declared in include/wpsgd.h.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libwpsgd.so")

HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-ignored-attributes", "-Wno-inline-asm",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]

UNITS = [
    ("api", "api.hip", []),
    ("combine", "combine.hip", []),
    ("objective", "objective.hip", []),
    ("chain_dense_mem", "chain_dense_mem.hip", []),
    ("chain_delay", "chain_delay.hip", []),
    ("chain_csr", "chain_csr.hip", []),
    ("chain_csr_pair", "chain_csr_pair.hip", []),
    ("chain_dense_reg_f32_hinge", "chain_dense_reg.hip", ["-DWPSGD_TX_BF16=0", "-DWPSGD_LOSS=0"]),
    ("chain_dense_reg_f32_logistic", "chain_dense_reg.hip", ["-DWPSGD_TX_BF16=0", "-DWPSGD_LOSS=1"]),
    ("chain_dense_reg_bf16_hinge", "chain_dense_reg.hip", ["-DWPSGD_TX_BF16=1", "-DWPSGD_LOSS=0"]),
    ("chain_dense_reg_bf16_logistic", "chain_dense_reg.hip", ["-DWPSGD_TX_BF16=1", "-DWPSGD_LOSS=1"]),
]


def _compile(unit, extra):
    name, src, defs = unit
    obj = os.path.join(OBJ, name + ".o")
    cmd = [HIPCC, *FLAGS, *defs, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed for {name}:\n{' '.join(cmd)}\n{proc.stdout}\n{proc.stderr}")
    return obj, proc.stderr


def build_library(extra_flags=(), jobs=None, verbose=False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(len(UNITS), max(1, len(os.sched_getaffinity(0))))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        results = list(pool.map(lambda u: _compile(u, list(extra_flags)), UNITS))
    if verbose:
        for _, err in results:
            if err.strip():
                sys.stderr.write(err)
    objs = [o for o, _ in results]
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *objs, "-o", LIB]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError(f"link failed:\n{proc.stdout}\n{proc.stderr}")
    return LIB


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
