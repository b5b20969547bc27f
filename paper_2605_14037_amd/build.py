"""Builds libspkv.so (HIP, gfx950) in-tree with hipcc."""

from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspkv.so")
SOURCES = ["spkv_api.hip", "spkv_write.hip", "spkv_decode.hip", "spkv_prefill.hip",
           "spkv_predictor.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-inline-asm", "-Rpass-analysis=kernel-resource-usage",
]

# Waves per SIMD the decode kernels are expected to reach (registers decide it, and the
# register count depends on how the compiler schedules loads against MFMAs): the library
# adapts its work-item count to whatever the runtime reports, but a drop costs bandwidth.
EXPECTED_OCCUPANCY = {"spkv_decode_splitILi128E": 3}      # every mode and merge width at head_dim 128


def _check_occupancy(remarks: str) -> list:
    import re
    warnings = []
    blocks = re.split(r"remark: Function Name: ", remarks)
    for blk in blocks[1:]:
        name = blk.split()[0]
        m = re.search(r"Occupancy \[waves/SIMD\]: (\d+)", blk)
        for key, want in EXPECTED_OCCUPANCY.items():
            if key in name and m and int(m.group(1)) < want:
                warnings.append(f"{name}: occupancy {m.group(1)} waves/SIMD, expected {want}")
    return warnings


def build(verbose: bool = False) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    cmd = [hipcc] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    lines = [l for l in res.stderr.splitlines() if noise not in l]
    err = "\n".join(l for l in lines if "remark:" not in l and "-Rpass-analysis" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    for w in _check_occupancy(res.stderr):
        print("WARNING:", w, flush=True)
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
