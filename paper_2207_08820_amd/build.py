"""Build the HIP library in-tree: hipcc cross-compiles for gfx950, no GPU needed.

    python -m paper_2207_08820_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdlrt_hip.so")
# measurement probes of bench.py (VALU peak, copy bandwidth, launch floor): a library of its own, so that the
# product library exports nothing but include/dlrt.h
PROBE_LIB = os.path.join(HERE, "libdlrt_probe.so")
# (source, object name, extra defines); the contraction kernels are built once per activation bit width
UNITS = [("api.hip", "api.o", []), ("pack.hip", "pack.o", []), ("epilogue.hip", "epilogue.o", []),
         ("contract_dispatch.hip", "contract_dispatch.o", []), ("unpacked_mfma.hip", "unpacked_mfma.o", []),
         ("unpacked_dot8.hip", "unpacked_dot8.o", [])] + \
        [("contract_rows.hip", f"contract_rows_a{b}.o", [f"-DDLRT_ABITS={b}"]) for b in (1, 2, 3, 4)] + \
        [("contract.hip", f"contract_a{b}.o", [f"-DDLRT_ABITS={b}"]) for b in (1, 2, 3, 4)] + \
        [("contract_wave.hip", f"contract_wave_a{b}.o", [f"-DDLRT_ABITS={b}"]) for b in (1, 2, 3, 4)] + \
        [("contract_panels.hip", f"contract_panels_a{b}.o", [f"-DDLRT_ABITS={b}"]) for b in (1, 2, 3, 4)]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# packed-fp32 instruction selection is switched off for every device compile
# --offload-compress: the device code of the several hundred kernel instantiations is stored compressed in the
# library (the HIP runtime unpacks it on load): a quarter of the size to ship
FLAGS = ["--offload-arch=gfx950", "--offload-compress", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(unit, extra) -> str:
    name, objname, defines = unit
    obj = os.path.join(OBJ, objname)
    proc = subprocess.run([HIPCC, *FLAGS, *defines, *extra, "-c", os.path.join(CSRC, name), "-o", obj],
                          stderr=subprocess.PIPE, text=True)
    # the host pass warns that it does not know the device-only target feature: harmless, dropped
    noise = "is not a recognized feature for this target"
    err = "\n".join(line for line in proc.stderr.splitlines() if noise not in line)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed on {name} {defines}:\n{err}")
    if err.strip() and os.environ.get("DLRT_BUILD_VERBOSE"):
        print(err, file=sys.stderr)
    return obj


def build_library(extra_flags=()) -> str:
    os.makedirs(OBJ, exist_ok=True)
    # the probe library carries the block kernel once more, with per-block clock sampling compiled in
    probe_units = [("probe.hip", "probe.o", [])] + \
                  [("contract.hip", f"probe_contract_a{b}.o", [f"-DDLRT_ABITS={b}", "-DDLRT_CLOCK_PROBE"]) for b in (1, 2, 3, 4)]
    units = UNITS + probe_units
    with ThreadPoolExecutor(max_workers=min(len(units), os.cpu_count() or 4, 16)) as pool:
        objs = list(pool.map(lambda u: _compile(u, list(extra_flags)), units))
    link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.run([*link, "-o", LIB, *objs[:len(UNITS)]], check=True)
    subprocess.run([*link, "-o", PROBE_LIB, *objs[len(UNITS):]], check=True)
    return LIB


if __name__ == "__main__":
    print(build_library(sys.argv[1:]))
