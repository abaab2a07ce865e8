"""The library's host code (argument checks, tree builders, GEMM planning, status strings) under
AddressSanitizer and UndefinedBehaviorSanitizer: a second build of the library with host-side
sanitizers (device code as usual) is loaded by the host-only tests in a child process that
preloads the sanitizer runtime.  Any report fails the test.  The sanitized library is rebuilt
only when a source is newer than it (about two minutes), so the suite stays quick."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT_DIR = os.path.join(ROOT, "_build", "hostsan")
LIB = os.path.join(OUT_DIR, "libmedusa_hip_hostsan.so")


def _stale():
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    srcs = glob.glob(os.path.join(ROOT, "paper_2401_10774_amd", "csrc", "*")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return any(os.path.getmtime(s) > built for s in srcs)


def test_host_code_under_address_and_undefined_behaviour_sanitizers():
    from paper_2401_10774_amd.build import build_library, sanitizer_runtime
    try:
        runtime = sanitizer_runtime()
    except RuntimeError as e:
        pytest.skip(str(e))
    if _stale():
        os.makedirs(OUT_DIR, exist_ok=True)
        build_library(host_sanitizers=True, out_path=LIB)
    env = dict(os.environ)
    env.update(MEDUSA_LIB_PATH=LIB, LD_PRELOAD=(runtime + " " + env.get("LD_PRELOAD", "")).strip(),
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=77", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1:exitcode=78")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
           os.path.join(ROOT, "tests", "test_abi.py"), os.path.join(ROOT, "tests", "test_sparse_tree.py")]
    proc = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    out = proc.stdout
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert proc.returncode == 0, out[-4000:]
    assert " passed" in out
