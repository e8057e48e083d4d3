"""Host-side sanitizer runs (CPU only, nothing here touches a GPU): the C oracle and the host half
of the library (argument checks, planner, dealing, launch set-up) are rebuilt with AddressSanitizer
and UndefinedBehaviorSanitizer, and the oracle pins / the host-only ABI tests run against those
builds in a child process that preloads the sanitizer runtimes."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _child_env(runtime_libs, extra):
    env = dict(os.environ)
    pre = [p for p in runtime_libs if p and os.path.exists(p)]
    if env.get("LD_PRELOAD"):          # keep whatever is preloaded already, behind the sanitizer runtime
        pre.append(env["LD_PRELOAD"])
    env["LD_PRELOAD"] = ":".join(pre)
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra)
    return env


def _gcc_file(name):
    return subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True, text=True).stdout.strip()


def test_oracle_pins_under_asan_ubsan(tmp_path):
    so = str(tmp_path / "liboracle_conv_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                           "-o", so, os.path.join(ROOT, "oracle", "conv_oracle.c")])
    env = _child_env([_gcc_file("libasan.so"), _gcc_file("libubsan.so")], {"ORACLE_CONV_LIB": so, "OMP_NUM_THREADS": "4"})
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "passed" in r.stdout


def test_host_api_under_asan_ubsan(tmp_path):
    """api.hip as plain C++ (no device code, launchers replaced by stand-ins) under the sanitizers:
    every host-only ABI test - argument checks, plans for thousands of shapes, the dealing."""
    from paper_2305_08819_amd import build
    lib = build.build_host_sanitized(str(tmp_path / "hostsan"))
    env = _child_env([_gcc_file("libasan.so"), _gcc_file("libubsan.so")], {"MI355CONV_LIB": lib})
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_abi_cpu.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "passed" in r.stdout
