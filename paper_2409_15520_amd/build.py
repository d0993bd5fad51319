"""Build libmpz.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2409_15520_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libmpz.so")
BUILD_DIR = os.path.join(PKG, "_build")

# -packed-fp32-ops off: the compiler must not form packed fp32 instructions on the test machines.
COMMON = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
# per-file extras: the noise stream is defined as unfused binary32 multiplies and adds
EXTRA = {"noise.hip": ["-ffp-contract=off"]}


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def build_library(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(BUILD_DIR, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(BUILD_DIR, src.replace(".hip", ".o"))
        cmd = [hipcc, *COMMON, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as ex:
        objs = list(ex.map(compile_one, sources()))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("linking libmpz.so failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


def build_host_sanitized(verbose: bool = True) -> str:
    """The same sources with AddressSanitizer and UndefinedBehaviorSanitizer on the HOST code only (argument
    validation, workspace carving, launch arithmetic); device code is compiled as usual.  Returns the path of
    _build/san/libmpz_san.so; load it with MPZ_LIBRARY=<path> and the ASan runtime preloaded (sanitizer_runtime())."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out_dir = os.path.join(BUILD_DIR, "san")
    os.makedirs(out_dir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    flags = [f if f != "-O3" else "-O1" for f in COMMON] + ["-g"] + san

    def compile_one(src):
        obj = os.path.join(out_dir, src.replace(".hip", ".o"))
        r = subprocess.run([hipcc, *flags, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc (host-sanitised) failed on {src}:\n{r.stderr}")
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as ex:
        objs = list(ex.map(compile_one, sources()))
    lib = os.path.join(out_dir, "libmpz_san.so")
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined", "-fno-gpu-sanitize",
                        "-shared-libsan", "-o", lib, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("linking libmpz_san.so failed:\n" + r.stderr)
    if verbose:
        print(f"built {lib}")
    return lib


def sanitizer_runtime() -> str:
    """Path of the shared ASan runtime of the ROCm clang (to LD_PRELOAD ahead of an uninstrumented python)."""
    clang = os.path.join(os.path.dirname(os.path.realpath(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"))), "..", "lib", "llvm",
                         "bin", "clang")
    r = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    return r.stdout.strip()


if __name__ == "__main__":
    if "--sanitize-host" in sys.argv:
        print(build_host_sanitized(), sanitizer_runtime())
    else:
        build_library()
