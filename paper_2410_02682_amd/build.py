"""Builds libeindecomp.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(HERE, "libeindecomp.so")
OBJDIR = os.path.join(HERE, "_build")
SOURCES = ["eg_graph.cpp", "eg_planner.cpp", "eg_exec.hip", "k_simple.hip", "k_contract.hip", "k_contract_dma.hip", "k_attention.hip", "k_ceilings.hip"]
HEADERS = [os.path.join(CSRC, "eg_internal.h"), os.path.join(CSRC, "eg_device.h"), os.path.join(INCLUDE, "eindecomp.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE, "-I" + CSRC,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function",
         "-Wno-unknown-warning-option", "-Wno-unused-command-line-argument"]


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src, force):
    obj = os.path.join(OBJDIR, src + ".o")
    path = os.path.join(CSRC, src)
    if force or _stale(obj, [path] + HEADERS):
        cmd = ["hipcc", "-x", "hip", "-c", path, "-o", obj] + FLAGS
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        errs = [ln for ln in r.stderr.splitlines() if "warning" in ln and "packed-fp32-ops" not in ln]
        if errs:
            sys.stderr.write("\n".join(errs[:20]) + "\n")
    return obj


def build(force: bool = False) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or _stale(LIB, objs):
        cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    return LIB


SAN_LIB = os.path.join(OBJDIR, "san", "libeindecomp_san.so")
HOST_SOURCES = ["eg_graph.cpp", "eg_planner.cpp", "eg_exec.hip"]      # everything that runs on the host besides the launchers
SAN_HOST = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
            "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def build_sanitized() -> str:
    """The library with its host code (graph, planner, executor) under the address and undefined-behaviour sanitizers;
    device code and the kernel files are the ordinary build's.  For tests/test_host_sanitizers.py: a process that loads
    it must have clang's shared ASan runtime loaded first (LD_PRELOAD), see sanitizer_runtime()."""
    build()
    d = os.path.dirname(SAN_LIB)
    os.makedirs(d, exist_ok=True)

    def one(src):
        obj = os.path.join(d, src + ".o")
        cmd = ["hipcc", "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + [f for f in FLAGS if f != "-O3"] + ["-O1"] + SAN_HOST
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc (sanitized) failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        return obj

    with ThreadPoolExecutor(max_workers=3) as ex:
        objs = list(ex.map(one, HOST_SOURCES))
    objs += [os.path.join(OBJDIR, s + ".o") for s in SOURCES if s not in HOST_SOURCES]
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan", "-o", SAN_LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link (sanitized) failed:\n%s\n%s" % (r.stdout, r.stderr))
    return SAN_LIB


def sanitizer_runtime() -> str:
    r = subprocess.run(["hipcc", "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = r.stdout.strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        import glob
        found = sorted(glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
        if not found:
            raise RuntimeError("clang's shared ASan runtime was not found")
        path = found[-1]
    return path


if __name__ == "__main__":
    print(build_sanitized() if "--sanitize" in sys.argv else build(force="--force" in sys.argv))
