"""Build libepd_encode.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libepd_encode.so")

SOURCES = ["epd_api.hip", "mm_cache.hip", "simple_f32.hip", "gemm_bf16.hip", "gemm_mxfp8.hip", "attention_bf16.hip", "rowops_bf16.hip", "roof_probe.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-result",
    # packed fp32 VALU forms stay disabled for every device function
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


# Host-side sanitizer build (address + undefined behaviour) of the same sources: the device code is compiled
# as always, only the host half of every file is instrumented.  The result is a second library that nothing
# loads by default; see sanitized_env().
SAN_LIB = os.path.join(BUILD, "libepd_encode_san.so")
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-omit-frame-pointer", "-Xarch_host", "-g"]


def _compile(src: str, sanitize: bool = False) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + (".san.o" if sanitize else ".o"))
    cmd = [_hipcc(), *FLAGS, *(SAN_FLAGS if sanitize else []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stderr[-8000:]))
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s" % r.stderr[-8000:])
    if verbose:
        print("built", LIB, file=sys.stderr)
    return LIB


def build_sanitized(verbose: bool = True) -> str:
    """libepd_encode_san.so: host code under AddressSanitizer and UndefinedBehaviorSanitizer."""
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, True), SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined", "-shared-libsan",
           "-fno-gpu-sanitize", *objs, "-o", SAN_LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s" % r.stderr[-8000:])
    if verbose:
        print("built", SAN_LIB, file=sys.stderr)
    return SAN_LIB


def sanitized_env() -> dict:
    """Environment in which a Python process loads the sanitized library: the sanitizer runtime first in the
    preload list (in front of whatever is there already), the binding pointed at the library, leak checking off
    (the interpreter itself never frees everything)."""
    rt = subprocess.run([_hipcc(), "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    env = dict(os.environ)
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["EPD_LIB_PATH"] = SAN_LIB
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    return env


if __name__ == "__main__":
    if "--sanitize" in sys.argv:
        build_sanitized()
        if "--test" in sys.argv:   # the host-only test files under the sanitizers
            root = os.path.dirname(HERE)
            sys.exit(subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                                     os.path.join(root, "tests", "test_abi_host.py"),
                                     os.path.join(root, "tests", "test_mm_cache_host.py")], env=sanitized_env()).returncode)
    else:
        build()
