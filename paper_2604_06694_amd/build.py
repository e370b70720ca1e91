"""Builds libaudiokv.so (the C-ABI library of include/audiokv.h) for gfx950 with hipcc.

Usage: python -m paper_2604_06694_amd.build [-j N]
The library is placed next to this file; objects go to _build/ beside it.
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
BUILD = os.path.join(PKG_DIR, "_build")
LIB = os.path.join(PKG_DIR, "libaudiokv.so")

ARCH = "gfx950"
COMMON = [
    "hipcc", f"--offload-arch={ARCH}", "-O3", "-std=c++20", "-fPIC",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    # packed-fp32 instruction forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]
# float64 budget arithmetic must round exactly like the plain definition: no contraction
PER_FILE = {"allocate.hip": ["-ffp-contract=off"]}


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str) -> str:
    obj = os.path.join(BUILD, src.replace(".hip", ".o"))
    cmd = COMMON + PER_FILE.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(jobs: int = 8, verbose: bool = True) -> str:
    os.makedirs(BUILD, exist_ok=True)
    srcs = sources()
    with cf.ThreadPoolExecutor(max_workers=max(1, min(jobs, 16))) as ex:
        objs = list(ex.map(_compile, srcs))
    cmd = ["hipcc", f"--offload-arch={ARCH}", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources")
    return LIB


# Sources whose host code carries the library's own logic (argument validation, workspace and launch planning):
# the sanitizer build instruments these and links the other objects as they are.
SANITIZED = ["api.hip", "score.hip"]
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined"]


def build_sanitized(verbose: bool = True) -> str:
    """Host-side AddressSanitizer + UndefinedBehaviorSanitizer build: _build/san/libaudiokv_san.so and, against it,
    _build/san/abi_host_check (tests/abi_host_check.cpp), which drives the host paths of every entry point.
    Device code is compiled as usual (GPU sanitizers are not used). Returns the path of the checker."""
    if not all(os.path.exists(os.path.join(BUILD, f.replace(".hip", ".o"))) for f in sources()):
        build(verbose=False)
    san = os.path.join(BUILD, "san")
    os.makedirs(san, exist_ok=True)
    objs = []
    for src in sources():
        if src in SANITIZED:
            obj = os.path.join(san, src.replace(".hip", ".o"))
            cmd = [c for c in COMMON if c != "-O3"] + ["-O1", "-g"] + SAN_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
            r = subprocess.run(cmd, capture_output=True, text=True)
            if r.returncode != 0:
                raise RuntimeError(f"sanitizer compile failed on {src}:\n{r.stderr}")
        else:
            obj = os.path.join(BUILD, src.replace(".hip", ".o"))
        objs.append(obj)
    lib = os.path.join(san, "libaudiokv_san.so")
    r = subprocess.run(["hipcc", f"--offload-arch={ARCH}", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                        "-o", lib] + objs, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"sanitizer link failed:\n{r.stderr}")
    exe = os.path.join(san, "abi_host_check")
    r = subprocess.run(["hipcc", "-x", "c++", "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined",
                        "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"),
                        os.path.join(ROOT, "tests", "abi_host_check.cpp"), "-o", exe, "-L", san, "-laudiokv_san",
                        f"-Wl,-rpath,{san}"], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"checker build failed:\n{r.stderr}")
    if verbose:
        print(f"built {lib} and {exe}")
    return exe


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("-j", type=int, default=8)
    ap.add_argument("--sanitize", action="store_true", help="also build the host-sanitizer library and its checker")
    args = ap.parse_args()
    build(args.j)
    if args.sanitize:
        build_sanitized()
