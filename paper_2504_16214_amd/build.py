"""Builds libmoe_w4a16.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2504_16214_amd.build                 # the library
    python -m paper_2504_16214_amd.build --host-ubsan    # plus a copy with a sanitized host layer

Objects go to paper_2504_16214_amd/_build/, the library next to this file.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoe_w4a16.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++20",
         # packed-FP32 VALU forms are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _units():
    units = []
    for dt in (0, 1):
        for kw in (1, 2, 4):
            units.append(("gemm_inst.hip", f"gemm_inst_dt{dt}_kw{kw}.o", [f"-DMOE_DT={dt}", f"-DMOE_KW={kw}"]))
    for dt in (0, 1):      # operand-order (prepacked) weight variants, group 128 only
        units.append(("gemm_inst.hip", f"gemm_inst_pre_dt{dt}.o", [f"-DMOE_DT={dt}", "-DMOE_KW=4", "-DMOE_PRE=1"]))
    for dt in (0, 1):      # eight-wave workgroups (128-token tiles), group 128 only
        units.append(("gemm_inst.hip", f"gemm_inst_wide_dt{dt}.o", [f"-DMOE_DT={dt}", "-DMOE_KW=4", "-DMOE_WIDE=1"]))
    for src in ("align.hip", "elementwise.hip", "router.hip", "fp8_gemm.hip", "fp8_quant.hip", "api.hip"):
        units.append((src, src.replace(".hip", ".o"), []))
    return units


def _compile(unit):
    src, obj, defs = unit
    cmd = [HIPCC, *FLAGS, *defs, "-c", os.path.join(CSRC, src), "-o", os.path.join(BUILD, obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src} {defs}:\n{err}")
    return err


def build(jobs: int | None = None, verbose: bool = True) -> str:
    os.makedirs(BUILD, exist_ok=True)
    units = _units()
    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        for unit, warn in zip(units, pool.map(_compile, units)):
            if verbose and warn.strip():
                print(f"[{unit[1]}] {warn}", file=sys.stderr)
    objs = [os.path.join(BUILD, u[1]) for u in units]
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


def build_host_ubsan(verbose: bool = True) -> str:
    """A second library, libmoe_w4a16_hostubsan.so, whose HOST code of the C ABI layer (api.hip:
    argument checks, tile and workspace arithmetic, launches) is compiled with the undefined-
    behaviour sanitizer in trapping mode (no runtime library: undefined behaviour executes a trap
    instruction); device code and the other objects are those of build().  Point the binding at it
    with MOE_W4A16_LIBRARY=<path> and run the tests: a trap ends the process with SIGILL."""
    lib = build(verbose=False)
    obj = os.path.join(BUILD, "api_hostubsan.o")
    cmd = [HIPCC, *[f for f in FLAGS if f != "-O3"], "-O1", "-g",
           "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fsanitize-trap=all",
           "-c", os.path.join(CSRC, "api.hip"), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for the sanitized api.hip:\n{r.stderr}")
    objs = [obj if u[1] == "api.o" else os.path.join(BUILD, u[1]) for u in _units()]
    out = os.path.join(HERE, "libmoe_w4a16_hostubsan.so")
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    if verbose:
        print(f"built {lib} and {out}")
    return out


if __name__ == "__main__":
    if "--host-ubsan" in sys.argv[1:]:
        build_host_ubsan()
    else:
        build()
