"""Builds libfastforward.so (gfx950) from csrc/ with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libfastforward.so")
SOURCES = ["ff_api.hip", "ff_predict.hip", "ff_gemm.hip", "ff_gemv.hip", "ff_glue.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
    "-Wno-unused-command-line-argument",
]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 feature flag; that warning is harmless
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False, extra_flags=()) -> str:
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        return _run([HIPCC, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=min(5, len(SOURCES))) as ex:
        outs = list(ex.map(one, zip(SOURCES, objs)))
    outs.append(_run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]))
    if verbose:
        for o in outs:
            if o.strip():
                print(o)
    return LIB


def build_example() -> str:
    """csrc/ff_c_example.c: a plain-C caller of the ABI (gcc, HIP runtime, libfastforward; no Python)."""
    os.makedirs(OBJ, exist_ok=True)
    exe = os.path.join(OBJ, "ff_c_example")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    _run(["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(rocm, "include"),
          os.path.join(CSRC, "ff_c_example.c"), "-o", exe, "-L" + PKG, "-lfastforward", "-L" + os.path.join(rocm, "lib"),
          "-lamdhip64", "-Wl,-rpath,$ORIGIN/..", "-Wl,-rpath," + os.path.join(rocm, "lib")])
    return exe


def build_host_checks() -> str:
    """csrc/ff_host_checks.c and the whole library in one executable whose HOST code is built with
    AddressSanitizer and UndefinedBehaviorSanitizer (the device code is compiled as always)."""
    os.makedirs(OBJ, exist_ok=True)
    exe = os.path.join(OBJ, "ff_host_checks")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    objs = [os.path.join(OBJ, s.replace(".hip", ".san.o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        return _run([HIPCC, *FLAGS, *san, "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=min(5, len(SOURCES))) as ex:
        list(ex.map(one, zip(SOURCES, objs)))
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    clang = os.path.join(rocm, "lib", "llvm", "bin", "clang")
    cobj = os.path.join(OBJ, "ff_host_checks.san.o")
    _run([clang, "-std=c99", "-O1", "-g", "-Wall", "-Wextra", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
          "-fno-omit-frame-pointer", "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(rocm, "include"),
          "-c", os.path.join(CSRC, "ff_host_checks.c"), "-o", cobj])
    _run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", *objs, cobj, "-o", exe,
          "-Wl,-rpath," + os.path.join(rocm, "lib")])
    return exe


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
