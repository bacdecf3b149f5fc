"""The host code of the library (converters, schedule and composite builders, reordering, Matrix Market reader, the
C ABI's argument handling) and the C oracle under AddressSanitizer + UndefinedBehaviorSanitizer: the CPU-only
converter, reader and format tests run once more in a child process against `libasyncsparse_hostsan.so` (device
code built as always, every -fsanitize= applied to the host compilation only) and a sanitized build of the
oracle.  Sanitizers never run on the GPU.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/lib/llvm/bin/clang"


@pytest.mark.skipif(not os.path.exists(CLANG), reason="no clang with sanitizer runtimes in this image")
def test_host_code_under_address_and_undefined_behaviour_sanitizers():
    runtime = subprocess.check_output([CLANG, "--print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("no shared AddressSanitizer runtime")
    sys.path.insert(0, ROOT)
    from paper_2604_17834_amd import build as lib_build
    lib = lib_build.build(tag="hostsan")
    env = {k: v for k, v in os.environ.items() if not k.startswith("ASP_")}
    env.update({
        "ASP_LIBRARY": lib, "ASP_ORACLE_SANITIZE": "1",
        # the runtime has to be the first library of the process; Python itself is not instrumented, so leak
        # reports (its arenas) are off -- out-of-bounds, use-after-free and undefined behaviour stay fatal
        "LD_PRELOAD": runtime + ((":" + os.environ["LD_PRELOAD"]) if os.environ.get("LD_PRELOAD") else ""),
        "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=1:halt_on_error=1",
        "UBSAN_OPTIONS": "print_stacktrace=1:halt_on_error=1",
    })
    files = ["tests/test_library_host.py", "tests/test_library_reorder.py", "tests/test_oracle_formats.py",
             "tests/test_oracle_spmm.py"]
    out = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + files,
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = out.stdout[-3000:] + "\n" + out.stderr[-3000:]
    assert out.returncode == 0, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    assert " passed" in out.stdout
