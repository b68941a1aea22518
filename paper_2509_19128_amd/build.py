"""Compile the HIP sources in csrc/ into libpl.so for gfx950 (in-tree, next to this file)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libpl.so")
OBJ = os.path.join(HERE, "_build")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
          # packed fp32 arithmetic is kept out of every kernel
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# the sampler's float32 decision must not be re-associated or fused
PER_FILE = {"kernels_sample.hip": ["-ffp-contract=off"]}
SOURCES = ["pl_engine.hip", "kernels_attn.hip", "kernels_gemm.hip", "kernels_misc.hip", "kernels_sample.hip",
           "kernels_is.hip", "kernels_f32.hip"]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + err)
    if err.strip():
        sys.stderr.write(err + "\n")


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    objs = []
    jobs = []
    for src in SOURCES:
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        objs.append(obj)
        jobs.append([HIPCC, *COMMON, *PER_FILE.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj])
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        list(ex.map(_run, jobs))
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *objs])
    if verbose:
        print("built", OUT)
    return OUT


class SanitizerUnavailable(RuntimeError):
    pass


def build_sanitized_driver(driver_c: str, out_dir: str) -> str:
    """Link a C driver program against the library's objects with the HOST code of pl_engine.hip (all the
    host logic) compiled under AddressSanitizer + UndefinedBehaviorSanitizer; device code is untouched.
    Returns the path of the executable.  The kernel objects come from the ordinary build."""
    if not all(os.path.exists(os.path.join(OBJ, s.replace(".hip", ".o"))) for s in SOURCES):
        build()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-g"]
    eng = os.path.join(out_dir, "pl_engine_san.o")
    drv = os.path.join(out_dir, "driver.o")
    exe = os.path.join(out_dir, "sanitize_driver")
    try:
        _run([HIPCC, *COMMON, *san, "-c", os.path.join(CSRC, "pl_engine.hip"), "-o", eng])
        _run([HIPCC, "-x", "c", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
              "-c", driver_c, "-o", drv])
        others = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES if s != "pl_engine.hip"]
        _run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
              "-o", exe, drv, eng, *others])
    except RuntimeError as ex:
        if "sanitize" in str(ex) and ("unsupported" in str(ex) or "cannot find" in str(ex) or "not found" in str(ex)):
            raise SanitizerUnavailable(str(ex)[-500:])
        raise
    return exe


if __name__ == "__main__":
    build(verbose=True)
