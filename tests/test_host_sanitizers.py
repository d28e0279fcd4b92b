"""Host code under the address and undefined-behaviour sanitizers (CPU only).

The library's host side (graph construction, planner, executor: csrc/eg_graph.cpp, eg_planner.cpp, eg_exec.hip) and
the C oracle are built a second time with -fsanitize=address,undefined, and the suites that drive them without a GPU
run once more against those builds in a child process that has the matching sanitizer runtime loaded first.  A report
from either sanitizer aborts the child (halt_on_error, -fno-sanitize-recover), which fails the test.  Device code is
not instrumented (no GPU sanitizer is available), and leak checking is off: the interpreter itself never frees much
of what it allocates.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_suite(files, preload, env_extra):
    env = dict(os.environ)
    # the runtime must come first among the preloaded objects; whatever is preloaded already stays, behind it
    env["LD_PRELOAD"] = preload + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(env_extra)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + [os.path.join(ROOT, "tests", f) for f in files]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout[-3000:] + "\n" + r.stderr[-3000:])
    assert r.returncode == 0, f"suite under sanitizers failed (exit {r.returncode}):\n{tail}"
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error:" not in r.stderr, tail
    assert " passed" in r.stdout, tail
    return r.stdout


def _maps_of_child(code, preload, env_extra):
    env = dict(os.environ)
    env["LD_PRELOAD"] = preload + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0"
    env.update(env_extra)
    r = subprocess.run([sys.executable, "-c", code + "\nprint(open('/proc/self/maps').read())"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    return r.stdout


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers():
    from paper_2410_02682_amd import build
    lib = build.build_sanitized()
    # the child really runs the instrumented build with the runtime in place
    maps = _maps_of_child("from paper_2410_02682_amd import _lib; _lib.load()", build.sanitizer_runtime(), {"EINDECOMP_LIB": lib})
    assert "libeindecomp_san.so" in maps and "libclang_rt.asan" in maps
    out = _run_suite(["test_abi_host.py", "test_planner_host.py"], build.sanitizer_runtime(), {"EINDECOMP_LIB": lib})
    print(out.strip().splitlines()[-1])


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    from oracle import build
    lib = build.build_sanitized()
    maps = _maps_of_child("from oracle.einsum_ref import round_bf16; round_bf16(1.0)", build.sanitizer_runtime(), {"EINSUM_REF_LIB": lib})
    assert "libeinsum_ref_san.so" in maps and "libasan" in maps
    out = _run_suite(["test_oracle_pins.py", "test_oracle_graphs.py"], build.sanitizer_runtime(), {"EINSUM_REF_LIB": lib, "OMP_NUM_THREADS": "4"})
    print(out.strip().splitlines()[-1])
