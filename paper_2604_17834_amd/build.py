"""Build libasyncsparse.so (gfx950 only) in-tree with hipcc.

    python -m paper_2604_17834_amd.build              the library
    python -m paper_2604_17834_amd.build hostsan      libasyncsparse_hostsan.so: the same sources with the HOST code
                                                      under AddressSanitizer + UndefinedBehaviorSanitizer (device code
                                                      is built as always); for the CPU-only tests of the converters
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libasyncsparse.so")
MEASURE_LIB = os.path.join(PKG, "libasyncsparse_measure.so")   # the benchmark's probe kernels: not part of the product
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

SOURCES = ["asp_api.cpp", "asp_convert.cpp", "asp_reorder.cpp", "asp_bcsr.hip", "asp_bcsr_dma.hip", "asp_bcsr_wide.hip", "asp_bcsr_f32.hip", "asp_wcsr.hip", "asp_wcsr_bf16.hip"]
EXTRA = os.environ.get("ASP_EXTRA_FLAGS", "").split()
# host-side sanitizers: every -fsanitize= goes to the host compilation only
HOSTSAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-g", "-fno-omit-frame-pointer"]
HOSTSAN_LINK = ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan", "-fno-gpu-sanitize"]
COMMON = EXTRA + ["-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-result", "-Wno-inline-asm"]
# gfx950 only; packed-fp32 VALU forms are switched off for device code
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str, tag: str = "") -> str:
    obj = os.path.join(OBJ, src + (("." + tag) if tag else "") + ".o")
    cmd = [HIPCC, "-c", os.path.join(CSRC, src), "-o", obj] + COMMON + DEVICE + (HOSTSAN if tag == "hostsan" else [])
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False, tag: str = "") -> str:
    """tag "" builds the library; tag "hostsan" builds libasyncsparse_hostsan.so with sanitized host code."""
    assert tag in ("", "hostsan")
    os.makedirs(OBJ, exist_ok=True)
    lib = LIB if not tag else os.path.join(PKG, "libasyncsparse_%s.so" % tag)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, tag), SOURCES))
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib] + objs + (HOSTSAN_LINK if tag else [])
    subprocess.check_call(cmd)
    if not tag:
        mobj = _compile("asp_measure.hip")
        subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", MEASURE_LIB, mobj])
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build(verbose=True, tag=sys.argv[1] if len(sys.argv) > 1 else "")
