"""The library's host code (tile-map builder, argument validation, partition driver) under AddressSanitizer and
UndefinedBehaviorSanitizer: a second build of the same sources with both sanitizers on the host side, and the host
test file run against it in a child process.  No GPU is involved (sanitizers do not run on device code)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/llvm/bin/clang"


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    from paper_2602_01469_amd import build as _build
    if not os.path.exists(CLANG):
        pytest.skip("no ROCm clang: cannot locate the sanitizer runtime")
    runtime = subprocess.run([CLANG, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE,
                             text=True, check=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("AddressSanitizer runtime not found")
    lib = _build.build(sanitize_host_to=str(tmp_path / "libpeagle_attn_hostsan.so"))
    env = dict(os.environ)
    env["PEAGLE_ATTN_LIB"] = lib
    # the interpreter is not instrumented: the runtime comes first in the preload list (after whatever is there)
    env["LD_PRELOAD"] = " ".join(x for x in (env.get("LD_PRELOAD", ""), runtime) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=86"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=87"
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_tilemap_host.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True, timeout=1500)
    tail = r.stdout[-4000:]
    assert "AddressSanitizer" not in r.stdout and "runtime error:" not in r.stdout, tail
    assert r.returncode == 0, tail
    assert " passed" in r.stdout, tail
