"""Builds the HIP library in-tree: csrc/*.hip -> libmedusa_hip.so (gfx950 only).

``python -m paper_2401_10774_amd.build`` or ``build_library()``.  hipcc cross-compiles
without a GPU present.  Objects go to a throw-away directory; only the shared library
stays next to this file.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libmedusa_hip.so")

SOURCES = ["tree.hip", "heads.hip", "gemm_big.hip", "rope.hip", "topk_tree.hip", "tree_attention.hip", "accept.hip", "kv_commit.hip"]

# Per-file code-generation options.  gemm_big.hip keeps MFMA accumulators in ordinary vector
# registers: with the compiler's default choice its large accumulator tile is copied between the
# two register files in every loop iteration (several hundred moves per 96 MFMAs).
PER_FILE_FLAGS = {"gemm_big.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


# Packed-fp32 VALU forms are switched off for every device compile.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; the HIP library cannot be built")


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), proc.stdout))
    return proc.stdout


def build_library(verbose: bool = False) -> str:
    hipcc = _hipcc()
    extra = os.environ.get("MEDUSA_HIPCC_EXTRA", "").split()      # tuning knobs, e.g. -DMEDUSA_GEMM_STAGES=3
    tmp = tempfile.mkdtemp(prefix="medusa_hip_build_")
    try:
        objs = [os.path.join(tmp, s.replace(".hip", ".o")) for s in SOURCES]

        def compile_one(pair):
            src, obj = pair
            return _run([hipcc, *HIPCC_FLAGS, *PER_FILE_FLAGS.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj])

        with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
            logs = list(ex.map(compile_one, zip(SOURCES, objs)))
        if verbose:
            for s, log in zip(SOURCES, logs):
                text = "\n".join(l for l in log.splitlines() if "packed-fp32-ops" not in l)
                if text.strip():
                    print("[%s]\n%s" % (s, text))
        out_tmp = os.path.join(tmp, "libmedusa_hip.so")
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out_tmp])
        shutil.move(out_tmp, LIB_PATH)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
