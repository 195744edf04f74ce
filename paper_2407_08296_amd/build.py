"""Builds libqgalore.so (HIP, gfx950 only) in-tree with hipcc: one object per source, compiled in parallel, then linked."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libqgalore.so")
SOURCES = ["qg_api.hip", "qg_quant.hip", "qg_adam.hip", "qg_gemm.hip", "qg_cossim.hip", "qg_diag.hip", "qg_refresh.hip", "qg_linear.hip", "qg_adam8.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                                   # fused multiply-adds only where written
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build(verbose: bool = False, extra_flags: list[str] | None = None, lib: str = LIB,
          link_flags: list[str] | None = None) -> str:
    """Compile every source (always: no up-to-date check) and link `lib`."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    flags = FLAGS + list(extra_flags or [])
    tag = os.path.splitext(os.path.basename(lib))[0]

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ, f"{tag}.{os.path.splitext(src)[0]}.o")
        cmd = [hipcc, *flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *(link_flags or []), *objs, "-o", lib]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return lib


def build_sanitized(driver_src: str, verbose: bool = False) -> str:
    """Host-side AddressSanitizer + UBSan build: the library with its HOST code instrumented (the sanitizer flags sit
    behind -Xarch_host; device code is compiled as usual) as _build/libqgalore_san.so, and `driver_src` (a host
    program that walks the ABI's validation paths) linked against it as _build/abi_sanitizer_driver.  Returns the
    driver's path; run it with LD_LIBRARY_PATH pointing at _build/."""
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    lib = build(verbose=verbose, extra_flags=san, lib=os.path.join(OBJ, "libqgalore_san.so"),
                link_flags=["-fsanitize=address", "-fsanitize=undefined"])
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    exe = os.path.join(OBJ, "abi_sanitizer_driver")
    cmd = [hipcc, "-x", "c++", "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined",
           "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"), driver_src,
           "-L", OBJ, "-lqgalore_san", "-Wl,-rpath," + OBJ, "-o", exe]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return exe


if __name__ == "__main__":
    print(build(verbose=True))
