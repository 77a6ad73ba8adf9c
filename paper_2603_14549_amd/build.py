"""Builds libasap.so (the C-ABI library of hand-written gfx950 kernels) in-tree with hipcc.

    python -m paper_2603_14549_amd.build

Objects go to _build/ at the repository root (not committed); the library lands next to the
package as paper_2603_14549_amd/lib/libasap.so, where the binding looks for it.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB_DIR = os.path.join(PKG, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libasap.so")
SOURCES = ["asap_api.hip", "asap_score.hip", "asap_select.hip", "asap_sim.hip", "asap_paper.hip", "asap_merge.hip",
           "asap_compact.hip", "asap_attention.hip", "asap_front.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         # packed-fp32 VALU forms stay off on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src: str, obj_dir: str) -> str:
    obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(verbose: bool = True) -> str:
    obj_dir = os.path.join(ROOT, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    os.makedirs(LIB_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, obj_dir), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    if verbose:
        print(f"built {LIB_PATH}")
    return LIB_PATH


if __name__ == "__main__":
    build_library()


def build_sanitized_host(out_dir: str) -> str:
    """The same sources with AddressSanitizer and UndefinedBehaviorSanitizer on the HOST half only (argument
    checks, workspace sizing, launch-shape choices, the Eq. 7-8 utilities); the device code is compiled as
    always.  For the CPU-only test that sweeps the host entry points; nothing GPU-side is sanitised or run."""
    os.makedirs(out_dir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    flags = [f if f != "-O3" else "-O1" for f in FLAGS] + san

    def one(src: str) -> str:
        obj = os.path.join(out_dir, src.replace(".hip", ".o"))
        res = subprocess.run([HIPCC, *flags, "-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc (sanitised host) failed on {src}:\n{res.stderr}")
        return obj
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(one, SOURCES))
    lib = os.path.join(out_dir, "libasap_san.so")
    res = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined",
                          "-fno-gpu-sanitize", "-o", lib, *objs], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link (sanitised host) failed:\n" + res.stderr)
    return lib
