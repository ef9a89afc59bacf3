"""Builds libhctr.so (HIP, gfx950) in-tree with hipcc.  No GPU is needed to build."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhctr.so")
SOURCES = ["runtime.cpp", "primitives.hip", "emb.hip", "hash.hip", "cache.hip", "etc.hip", "noalloc.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 instructions
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "hctr.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = False) -> str:
    """One hipcc per source file, side by side, then one link; every call compiles everything."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ, os.path.basename(src) + ".o")
        cmd = [hipcc] + FLAGS + ["-x", "hip", "-c"] + inc + [src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        done = subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
        # the host pass does not know the packed-fp32 feature and says so once per file: harmless
        text = "\n".join(l for l in done.stdout.decode(errors="replace").splitlines() if "packed-fp32-ops" not in l)
        if text.strip():
            print(text, flush=True)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        try:
            objs = list(pool.map(compile_one, sources()))
        except subprocess.CalledProcessError as e:
            sys.stderr.write(e.stdout.decode(errors="replace"))
            raise
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def build_host_sanitized(driver_src: str) -> str:
    """The library with its HOST code under AddressSanitizer and UndefinedBehaviorSanitizer (device code
    as usual), as _build/libhctr_san.so, and `driver_src` linked against it as _build/abi_sanitize_driver.
    Returns the driver's path.  For the CPU-side checks of the argument validation: the driver makes only
    calls that the host answers before any launch, so it runs without a GPU."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=all", "-g"]
    lib_san = os.path.join(OBJ, "libhctr_san.so")

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ, os.path.basename(src) + ".san.o")
        subprocess.run([hipcc] + [f for f in FLAGS if f != "-O3"] + ["-O1"] + san + ["-x", "hip", "-c"] + inc +
                       [src, "-o", obj], check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        objs = list(pool.map(compile_one, sources()))
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                           "-shared-libsan"] + objs + ["-o", lib_san])
    exe = os.path.join(OBJ, "abi_sanitize_driver")
    # the sanitizer runtime as a shared library, found through the run path (it lies in the compiler's tree)
    rt = subprocess.run([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], check=True, capture_output=True,
                        text=True).stdout.strip()
    if not os.path.isabs(rt):
        import glob
        found = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
        rt = found[0] if found else rt
    subprocess.check_call([hipcc, "-x", "c++", "-std=c++17", "-g", "-fsanitize=address", "-fsanitize=undefined",
                           "-fno-sanitize-recover=all", "-shared-libsan"] + inc + [driver_src, "-x", "none", lib_san,
                           "-Wl,-rpath," + OBJ, "-Wl,-rpath," + os.path.dirname(rt), "-o", exe])
    return exe


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
