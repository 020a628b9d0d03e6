"""Build the HIP library (libqcache.so) in-tree for gfx950 with hipcc."""
import os
import shutil
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libqcache.so")

SOURCES = ["qc_api.cpp", "qc_util.hip", "qc_decode.hip", "qc_prefill_simple.hip", "qc_prefill_mfma.hip",
           "qc_select.hip", "qc_project.hip", "qc_prune.hip"]

# Packed fp32 instructions are kept out of the generated code on purpose.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def hipcc():
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l]
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(lines))
    if verbose and lines:
        print("\n".join(lines))


def build_library(verbose=False, extra_flags=()):
    """Compile every source (in parallel) and link libqcache.so; always recompiles."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(PKG_DIR, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"] + list(extra_flags) + [
        "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = []
    jobs = []
    for src in SOURCES:
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        objs.append(obj)
        jobs.append([hipcc()] + compile_flags + ["-c", os.path.join(CSRC, src), "-o", obj])
    with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 1, 8)) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB_PATH + ".tmp"], verbose)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


NATIVE_CALLER_SRC = os.path.join(ROOT, "tests", "c_abi_gpu_probe.cpp")
NATIVE_CALLER = os.path.join(ROOT, "tests", "c_abi_gpu_probe")


def build_native_caller(verbose=False):
    """The test program that calls the library with nothing but the HIP runtime (tests/c_abi_gpu_probe.cpp):
    host code only, linked against the library that sits in the package directory."""
    _run([hipcc(), "-O2", "-std=c++17", "-Wall", "-I", os.path.join(ROOT, "include"), NATIVE_CALLER_SRC,
          "-o", NATIVE_CALLER + ".tmp", "-L", PKG_DIR, "-l:" + os.path.basename(LIB_PATH),
          "-Wl,-rpath," + PKG_DIR, "-Wl,-rpath,$ORIGIN/../paper_2602_01901_amd"], verbose)
    os.replace(NATIVE_CALLER + ".tmp", NATIVE_CALLER)
    return NATIVE_CALLER


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_native_caller(verbose=True))
