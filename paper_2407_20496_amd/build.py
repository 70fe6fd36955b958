"""Build libhinm.so (gfx950) in-tree with hipcc.  Used by __graft_entry__.build() and by hand:

    python -m paper_2407_20496_amd.build
    python -m paper_2407_20496_amd.build --sanitize    # host code under ASan + UBSan -> _build/libhinm_sanitize.so

The sanitized library is for CPU runs of the argument-validation tests only (tests/test_sanitize.py): the
device code in it is the ordinary one and the GPU is never touched under a sanitizer.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhinm.so")
OBJ_DIR = os.path.join(HERE, "_build")

SOURCES = ["hinm_api.hip", "pack_kernels.hip", "icp_search.hip", "ocp_search.hip", "prepare.hip", "spmm_reference.hip", "spmm_skinny.hip", "spmm_tile.hip", "spmm_vectors.hip",
           "spmm_tile_prepared.hip", "spmm_skinny_prepared.hip", "spmm_rows16_prepared.hip", "spmm_panel_prepared.hip",
           "calib_kernels.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-Wall", "-Wno-unused-function",
]


# every -fsanitize= option directly behind an -Xarch_host: the device pass must not see them
SANITIZE_LIB = os.path.join(OBJ_DIR, "libhinm_sanitize.so")
SANITIZE_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                  "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
                  "-Xarch_host", "-shared-libsan", "-g"]


def sanitizer_runtime() -> str:
    """Path of the shared ASan runtime of the compiler that built the sanitized library (to be preloaded into the
    interpreter that loads it)."""
    res = subprocess.run([HIPCC, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = res.stdout.strip()
    if res.returncode != 0 or not os.path.isabs(path):
        # hipcc may not forward -print-file-name: ask the clang it drives
        clang = os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "lib", "llvm", "bin", "clang++")
        res = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
        path = res.stdout.strip()
    return os.path.realpath(path)


def _compile(src: str, sanitize: bool = False) -> str:
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".san.o" if sanitize else ".o"))
    cmd = [HIPCC, *FLAGS, *(SANITIZE_FLAGS if sanitize else []), "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True, sanitize: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda src: _compile(src, sanitize), SOURCES))
    lib = SANITIZE_LIB if sanitize else LIB
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    if sanitize:
        cmd += ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan", "-fno-gpu-sanitize"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    if verbose:
        print(f"built {lib}")
    return lib


if __name__ == "__main__":
    build(sanitize="--sanitize" in sys.argv[1:])
