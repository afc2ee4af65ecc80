"""Build libltea.so (all HIP kernels + the C ABI) for gfx950, in-tree.

    python -m paper_2510_20787_amd.build

hipcc cross-compiles without a GPU.  Objects go to paper_2510_20787_amd/_build/ (git-ignored); the shared
library lands next to this file, where the binding looks for it.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libltea.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str) -> str:
    obj = os.path.join(BUILD, os.path.basename(src)[:-4] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(BUILD, exist_ok=True)
    srcs = sources()
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources")
    return LIB


def build_host_check(verbose: bool = True) -> str:
    """The C ABI's host logic (csrc/api.hip) under AddressSanitizer and UndefinedBehaviorSanitizer, linked with the
    ordinary objects of the other sources (built first if they are not there) and with tests/host_check/abi_host_check.cpp into an
    executable.  Host code only: device code is compiled as always.  Returns the path of the executable."""
    os.makedirs(BUILD, exist_ok=True)
    root = os.path.dirname(HERE)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    api_o = os.path.join(BUILD, "api_hostsan.o")
    drv_o = os.path.join(BUILD, "abi_host_check.o")
    exe = os.path.join(BUILD, "abi_host_check")
    noise = "is not a recognized feature for this target"
    steps = [
        [HIPCC, *FLAGS, *san, "-c", os.path.join(CSRC, "api.hip"), "-o", api_o],
        [HIPCC, "-x", "hip", *FLAGS, *san, "-I", os.path.join(root, "include"), "-c",
         os.path.join(root, "tests", "host_check", "abi_host_check.cpp"), "-o", drv_o],
    ]
    others = [os.path.join(BUILD, os.path.basename(s_)[:-4] + ".o") for s_ in sources() if not s_.endswith("/api.hip")]
    if any(not os.path.exists(o) for o in others):
        build(verbose=False)
    steps.append([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", exe,
                  api_o, drv_o, *others])
    for cmd in steps:
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("host-check build failed:\n" + " ".join(cmd) + "\n" +
                               "\n".join(l for l in r.stderr.splitlines() if noise not in l))
    if verbose:
        print(f"built {exe}")
    return exe


if __name__ == "__main__":
    build()
    if "--host-check" in sys.argv:
        build_host_check()
