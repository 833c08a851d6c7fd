"""Build liblaser.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2602_11562_amd.build

Cross-compiles without a GPU. The shared library is written next to this file so it
travels with the source tree; nothing is installed.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblaser.so")
OBJDIR = os.path.join(HERE, "_build")

SOURCES = ["laser_api.hip", "sta_generic.hip", "sta_mfma.hip", "sta_stream.hip", "gsta_generic.hip",
           "gsta_tiled.hip", "fused_forward.hip", "multires.hip", "segment_ffn.hip", "ffn_gsta.hip", "project.hip", "sta_backward.hip", "gsta_backward.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _compile(src: str, extra=()) -> str:
    obj = os.path.join(OBJDIR, ("tuning_" if extra else "") + src.replace(".hip", ".o"))
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(jobs: int = 6, tuning: bool = False, out: str = LIB) -> str:
    """Compile every HIP source and link liblaser.so. Always rebuilds. `tuning` builds the variant whose launch
    shapes can be overridden through environment variables (parameter sweeps only; never the shipped library)."""
    os.makedirs(OBJDIR, exist_ok=True)
    extra = ("-DLASER_TUNING",) if tuning else ()
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda src: _compile(src, extra), SOURCES))
    tmp = out + ".tmp"
    r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, out)
    return out


def build_host_check(out: str) -> str:
    """Build tests/abi_host_check.cpp into an executable whose host code of laser_api.hip (argument validation,
    kernel selection, size arithmetic) is instrumented with AddressSanitizer and UndefinedBehaviorSanitizer; the
    kernel launchers are the objects of the last build_library() (device code is never sanitized, and nothing
    here reaches a launch). No GPU needed to build or run it."""
    os.makedirs(OBJDIR, exist_ok=True)
    objs = [os.path.join(OBJDIR, src.replace(".hip", ".o")) for src in SOURCES if src != "laser_api.hip"]
    if not all(os.path.exists(o) for o in objs):
        build_library()
    san = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
    api_obj = os.path.join(OBJDIR, "san_laser_api.o")
    arch_host = [x for f in san for x in ("-Xarch_host", f)]
    steps = [
        [_hipcc(), *[f for f in HIPCC_FLAGS if f != "-O3"], "-O1", "-g", *arch_host, "-c",
         os.path.join(CSRC, "laser_api.hip"), "-o", api_obj],
        ["/opt/rocm/lib/llvm/bin/clang++", "-O1", "-g", *san, "-I" + os.path.join(ROOT, "include"), "-c",
         os.path.join(ROOT, "tests", "abi_host_check.cpp"), "-o", os.path.join(OBJDIR, "abi_host_check.o")],
        [_hipcc(), "--offload-arch=gfx950", "-fno-gpu-sanitize", *san, os.path.join(OBJDIR, "abi_host_check.o"),
         api_obj, *objs, "-o", out],
    ]
    for cmd in steps:
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("host check build failed:\n" + " ".join(cmd) + "\n" + r.stderr[-4000:])
    return out


if __name__ == "__main__":
    if len(sys.argv) > 2 and sys.argv[1] == "--tuning":      # python -m paper_2602_11562_amd.build --tuning OUT.so
        print(build_library(tuning=True, out=os.path.abspath(sys.argv[2])))
    else:
        print(build_library())
