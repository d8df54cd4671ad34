"""Builds libflashcache.so (gfx950) in-tree with hipcc.  Used by __graft_entry__.build()."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libflashcache.so")
# (source, object name, extra flags): fft.hip is compiled once per lane radix of the transform kernel
UNITS = [
    ("fft.hip", "fft_r4.o", ["-DFC_FFT_R=4"]),
    ("fft.hip", "fft_r8.o", ["-DFC_FFT_R=8"]),
    ("fft.hip", "fft_r16.o", ["-DFC_FFT_R=16"]),
    ("fft.hip", "fft_r2.o", ["-DFC_FFT_R=2"]),
    ("fft.hip", "fft_r1.o", ["-DFC_FFT_R=1"]),
    ("dense.hip", "dense.o", []),
    ("decode.hip", "decode.o", []),
    ("select_gather.hip", "select_gather.o", []),
    ("allocate.hip", "allocate.o", []),
    ("api.hip", "api.o", []),
    ("profile.hip", "profile.o", []),
]

# Packed-fp32 instruction selection is switched off for all device code: some packed forms have
# given wrong results on this hardware, and the compiler would otherwise form them by itself.
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
    "-Wno-unused-command-line-argument",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False, defines=(), output: str = LIB_PATH, extra_flags=()) -> str:
    """Compiles every translation unit and links the shared library; returns its path.

    `defines` / `output` make an experiment build beside the product one (its own object
    directory), e.g. defines=("FC_FFT_KNOBS",) for the build whose transform geometry can be
    overridden from the environment, or ("FC_FFT_NOPAIR",) for the generic block fold."""
    hipcc = hipcc_path()
    tag = "".join("_" + d.lower() for d in defines)
    if extra_flags:
        tag += "_x" + format(abs(hash(tuple(extra_flags))) % (1 << 32), "08x")
    obj_dir = os.path.join(PKG_DIR, "_build" + tag)
    os.makedirs(obj_dir, exist_ok=True)
    dflags = ["-D" + d for d in defines] + list(extra_flags)

    def compile_one(unit) -> str:
        src, obj_name, extra = unit
        obj = os.path.join(obj_dir, obj_name)
        cmd = [hipcc, *HIPCC_FLAGS, *dflags, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{res.stdout}\n{res.stderr}")
        if verbose and res.stderr.strip():
            sys.stderr.write(res.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, UNITS))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", output, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}\n{res.stderr}")
    return output


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description="build libflashcache.so, or an experiment build of it")
    ap.add_argument("--define", action="append", default=[], help="extra -D macro (repeatable)")
    ap.add_argument("--output", default=LIB_PATH, help="path of the shared library to write")
    ap.add_argument("--flag", action="append", default=[],
                    help="extra hipcc argument for every unit (repeatable; write --flag=-mllvm --flag=-some-option)")
    a = ap.parse_args()
    if (a.define or a.flag) and os.path.abspath(a.output) == LIB_PATH:
        ap.error("an experiment build needs its own --output (the product library takes no extra flags)")
    print(build(verbose=True, defines=tuple(a.define), output=os.path.abspath(a.output), extra_flags=tuple(a.flag)))
