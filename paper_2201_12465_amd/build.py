"""Builds the two shared libraries for gfx950 with hipcc.

libflmi355.so       the product: HIP kernels + host runtime + the C ABI of include/fl_layer.h, and
                    nothing else (no test entry points, no kernel-selection overrides).
libflmi355_test.so  the same objects, with the host files that differ compiled under
                    -DFL_TEST_EXPORTS, plus the entry points of include/fl_test.h (single kernels,
                    allocator over a fake store, tape with stub operators, probes).

`python -m paper_2201_12465_amd.build` compiles every source in csrc/ and links both next to this
file.  hipcc cross-compiles, so no GPU is needed.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libflmi355.so")
TEST_LIB = os.path.join(HERE, "libflmi355_test.so")
# compiled once, linked into both libraries
SHARED = ["gemm.hip", "gemm_pipe.hip", "gemm_f32_small.hip", "attention.hip", "attention_mfma.hip", "attention_bwd_fused.hip",
          "attention_mfma_f32.hip", "layernorm.hip", "reduce.hip", "optimizer.hip", "dropout.hip", "transpose.hip",
          "static_scratch.hip", "allocator.cpp"]
# compiled twice: without and with -DFL_TEST_EXPORTS
VARIANT = ["layer.cpp", "select.cpp"]
TEST_ONLY = ["test_exports.cpp"]
# packed-fp32 instructions are switched off for all device code
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def _compile(job) -> str:
    src, test = job
    obj = os.path.join(OBJ, src + (".test.o" if test else ".o"))
    cmd = [_hipcc(), *COMMON, "-c", os.path.join(CSRC, src), "-o", obj]
    if test:
        cmd.insert(1, "-DFL_TEST_EXPORTS")
    if src.endswith(".hip"):
        cmd[1:1] = DEVICE_FLAGS
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"compiling {src} failed:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    jobs = [(s, False) for s in SHARED + VARIANT] + [(s, True) for s in VARIANT + TEST_ONLY]
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = dict(zip(jobs, ex.map(_compile, jobs)))
    # only the C ABI is visible from outside: everything else stays local to its library
    vers = os.path.join(OBJ, "exports.map")
    with open(vers, "w") as f:
        f.write("{ global: fl_*; local: *; };\n")
    for lib, members in ((LIB, [(s, False) for s in SHARED + VARIANT]),
                         (TEST_LIB, [(s, False) for s in SHARED] + [(s, True) for s in VARIANT + TEST_ONLY])):
        cmd = [_hipcc(), "-shared", "-fPIC", *DEVICE_FLAGS[:1], f"-Wl,--version-script={vers}", "-o", lib,
               *[objs[m] for m in members]]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"linking {os.path.basename(lib)} failed:\n" + r.stderr)
        if verbose:
            print("built", lib)
    return LIB


if __name__ == "__main__":
    build()
