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


# Host-side sanitizers (AddressSanitizer + UndefinedBehaviorSanitizer) for the library's host code --
# argument checks, tree builders, GEMM planning -- in a second library that the CPU tests load in a
# child process (tests/test_host_sanitizer.py).  Device code is compiled as usual.
HOST_SANITIZER_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                        "-Xarch_host", "-fno-omit-frame-pointer", "-Xarch_host", "-fno-sanitize-recover=undefined", "-g"]


def sanitizer_runtime() -> str:
    """The shared AddressSanitizer runtime of hipcc's clang (to be preloaded into the Python process)."""
    import glob
    hits = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not hits:
        raise RuntimeError("no shared AddressSanitizer runtime found next to hipcc's clang")
    return hits[-1]


def build_library(verbose: bool = False, host_sanitizers: bool = False, out_path: str = None) -> str:
    hipcc = _hipcc()
    extra = HOST_SANITIZER_FLAGS if host_sanitizers else []
    out_path = out_path or LIB_PATH
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
        link_extra = ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"] if host_sanitizers else []
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *link_extra, *objs, "-o", out_tmp])
        shutil.move(out_tmp, out_path)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return out_path


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
