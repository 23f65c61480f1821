"""Builds libchunkkv.so (gfx950) in-tree with hipcc.  Run: python -m paper_2502_00299_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libchunkkv.so")
SOURCES = ["api.hip", "compact.hip", "decode.hip", "quality.hip", "topk.hip", "score_misc.hip", "score_bf16.hip", "score_f32.hip", "score_f16.hip",
           "score_single_bf16.hip", "score_single_f16.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed-fp32 instructions are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # no kernel relies on NaN propagation: lets max() compile to one instruction
         "-fno-honor-nans",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


def build_host_sanitizer_check(out_dir: str) -> str:
    """Builds tests/host_sanitizer_main.cpp against the library's sources with AddressSanitizer and
    UndefinedBehaviorSanitizer on the HOST pass only (device code is compiled as usual and never runs in that
    program): api.hip, which holds every argument check and workspace plan, is recompiled with the sanitizers;
    the kernels' objects are the ones build() made.  Returns the path of the executable."""
    os.makedirs(out_dir, exist_ok=True)
    if not all(os.path.exists(os.path.join(OBJ, s.replace(".hip", ".o"))) for s in SOURCES):
        build(verbose=False)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    api_o = os.path.join(out_dir, "api_san.o")
    main_o = os.path.join(out_dir, "host_sanitizer_main.o")
    exe = os.path.join(out_dir, "host_sanitizer_check")
    clangxx = os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "lib", "llvm", "bin", "clang++")
    if not os.path.exists(clangxx):
        clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    steps = [
        [HIPCC, *FLAGS, *san, "-c", os.path.join(CSRC, "api.hip"), "-o", api_o],
        [clangxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-fno-omit-frame-pointer", "-I", os.path.join(ROOT, "include"), "-c",
         os.path.join(ROOT, "tests", "host_sanitizer_main.cpp"), "-o", main_o],
        [clangxx, "-fsanitize=address,undefined", "-o", exe, main_o, api_o,
         *[os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES if s != "api.hip"],
         "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"],
    ]
    for cmd in steps:
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("host sanitizer build failed:\n" + " ".join(cmd) + "\n" + r.stderr[-4000:])
    return exe


if __name__ == "__main__":
    build()
