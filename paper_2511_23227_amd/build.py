"""Compile the HIP sources into paper_2511_23227_amd/libpcpp.so for gfx950 (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpcpp.so")
PROBE_LIB = os.path.join(HERE, "libpcpp_probe.so")     # the benchmark's peak-rate probe, outside the library's interface

# file -> extra flags.  The search kernels must not contract a*b+c into an FMA: the inclusion test
# is a fixed binary64 operation sequence shared with the CPU oracle by convention.
SOURCES = {
    "pcpp_api.hip": [],
    "scan.hip": [],
    "build_triplets.hip": ["-ffp-contract=off"],
    "spatial_order.hip": [],
    "mvmr_generic.hip": [],
    "mvmr_weight.hip": [],
    "mvmr_rows.hip": [],
    # MFMA results in ordinary vector registers unless register pressure moves them (see the file header)
    "mvmr_rows_wide.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
    "mvmr_rows_pc.hip": [],
    "tune.hip": [],
}

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-Wall", "-Wno-unused-function",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(name: str, extra) -> str:
    src = os.path.join(CSRC, name)
    obj = os.path.join(OBJ, name + ".o")
    cmd = ["hipcc", "-c", src, "-o", obj] + COMMON + list(extra)
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops' is not a recognized feature"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {name}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda kv: _compile(*kv), SOURCES.items()))
    tmp = LIB + ".tmp"
    subprocess.run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs, check=True)
    os.replace(tmp, LIB)
    probe = _compile("peak_probe.hip", [])
    tmp = PROBE_LIB + ".tmp"
    subprocess.run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp, probe], check=True)
    os.replace(tmp, PROBE_LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
