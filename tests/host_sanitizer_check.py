"""Builds libgptaq with AddressSanitizer + UndefinedBehaviorSanitizer on the HOST side only and runs the
argument-validation paths of every entry point under it (tests/host_sanitizer_driver.cpp).  No GPU is needed: each
call must return its error code before anything is launched.  Not collected by pytest (a full build of the
library takes a few minutes); run by hand:  python tests/host_sanitizer_check.py
"""
import os
import shutil
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from paper_2504_02692_amd import build as B  # noqa: E402

SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def main() -> int:
    out = tempfile.mkdtemp(prefix="gptaq_hostsan_")
    try:
        return run(out)
    finally:
        shutil.rmtree(out, ignore_errors=True)


def run(out: str) -> int:
    hipcc = B._hipcc()
    cxx = "/opt/rocm/lib/llvm/bin/clang++"            # the compiler hipcc drives: same sanitizer runtime as the library
    objs = []
    for src in B.SOURCES:
        obj = os.path.join(out, src.replace(".hip", ".o"))
        cmd = [hipcc, *B.FLAGS, *SAN, "-c", os.path.join(B.CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            print(r.stderr[-4000:])
            return 2
        objs.append(obj)
        print("compiled", src, flush=True)
    lib = os.path.join(out, "libgptaq_hostsan.so")
    exe = os.path.join(out, "driver")
    for cmd in ([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", lib, *objs],
                [cxx, "-std=c++17", "-fsanitize=address", "-fsanitize=undefined", "-g", "-I", os.path.join(ROOT, "include"),
                 os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), "-o", exe, "-L", out, "-lgptaq_hostsan", "-Wl,-rpath," + out]):
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            print(" ".join(cmd), "\n", r.stderr[-4000:])
            return 2
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env)
    print(r.stdout[-4000:], r.stderr[-4000:])
    return r.returncode


if __name__ == "__main__":
    sys.exit(main())
