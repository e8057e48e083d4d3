"""Build libmi355conv.so (HIP, gfx950 only) in-tree with hipcc.

Usage: ``python -m paper_2305_08819_amd.build [--force]``.  hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libmi355conv.so")
SOURCES = ["api.hip", "kernels_direct.hip", "kernel_gather_gemm.hip", "kernel_gather_elem.hip",
           "kernel_wgrad.hip", "kernel_wgrad_fast.hip", "kernel_small_ic.hip", "probe_mfma.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed-fp32 VALU forms are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _deps_mtime() -> float:
    paths = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    paths.append(os.path.join(os.path.dirname(PKG), "include", "mi355conv.h"))
    return max(os.path.getmtime(p) for p in paths)


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= _deps_mtime():
        return obj
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    noise = "is not a recognized feature for this target"
    warn = "\n".join(l for l in r.stderr.splitlines() if noise not in l).strip()
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def build_host_sanitized(out_dir: str) -> str:
    """A HOST-ONLY build of the library under AddressSanitizer + UndefinedBehaviorSanitizer: api.hip
    (argument checks, planner, dealing, launch set-up) compiled as plain C++ with g++, the kernel
    launchers replaced by stand-ins that report hipErrorNotSupported (host_only_stubs.cpp).  For the
    CPU test that runs the host-only ABI tests under the sanitizers; it holds no device code and is
    never used on a GPU."""
    os.makedirs(out_dir, exist_ok=True)
    lib = os.path.join(out_dir, "libmi355conv_hostsan.so")
    rocm = os.path.dirname(os.path.dirname(os.path.realpath(HIPCC)))
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-D__HIP_PLATFORM_AMD__",
           "-I" + os.path.join(rocm, "include"), "-x", "c++", os.path.join(CSRC, "api.hip"),
           os.path.join(CSRC, "host_only_stubs.cpp"), "-o", lib, "-L" + os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath," + os.path.join(rocm, "lib")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("host-only sanitizer build failed:\n%s" % r.stderr[-4000:])
    return lib


def build(force: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        tmp = LIB + ".tmp%d" % os.getpid()
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
