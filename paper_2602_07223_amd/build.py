"""Builds libvegas.so (the C-ABI HIP library) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libvegas.so")

SOURCES = ["vegas_api.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # leading scalar kernel arguments arrive in scalar registers with the wave (gfx940 and later)
    "-mllvm", "-amdgpu-kernarg-preload-count=14",
    "-Wall", "-Wno-unused-function",
]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


TIMELINE_LIB_PATH = os.path.join(HERE, "libvegas_timeline.so")


def build_library(verbose: bool = True, extra_flags=(), timeline: bool = False) -> str:
    """Compile every HIP source into paper_2602_07223_amd/libvegas.so; returns its path.
    timeline=True builds the profiling variant instead (libvegas_timeline.so: the same code with -DVEGAS_TIMELINE,
    whose streaming kernels note per-wave phase times; bench.py --timeline loads it)."""
    out = TIMELINE_LIB_PATH if timeline else LIB_PATH
    if timeline:
        extra_flags = (*extra_flags, "-DVEGAS_TIMELINE")
    cmd = [hipcc_path(), *FLAGS, *extra_flags, "-o", out] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return out


def kernel_resource_usage() -> dict:
    """Compiles the device code once more (nothing is written) with the compiler's resource report switched on and
    returns {demangled kernel name: {"vgprs", "agprs", "sgprs", "scratch_bytes_per_lane", "lds_bytes", "occupancy"}}.
    Used by the CPU tests to hold the streaming kernels to zero scratch (no register spills)."""
    import re
    build_flags = [f for f in FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hipcc_path(), *build_flags, "-c", "--cuda-device-only", "-Rpass-analysis=kernel-resource-usage",
           "-o", os.devnull] + [os.path.join(CSRC, s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    names, out, cur = [], {}, None
    keys = {"VGPRs": "vgprs", "AGPRs": "agprs", "TotalSGPRs": "sgprs", "ScratchSize [bytes/lane]": "scratch_bytes_per_lane",
            "LDS Size [bytes/block]": "lds_bytes", "Occupancy [waves/SIMD]": "occupancy"}
    for line in res.stderr.splitlines():
        m = re.search(r"remark: +(.*?)(?: \[-Rpass-analysis.*)?$", line)
        if not m:
            continue
        text = m.group(1).strip()
        if text.startswith("Function Name:"):
            cur = text.split(":", 1)[1].strip()
            names.append(cur)
            out[cur] = {}
            continue
        for k, short in keys.items():
            if cur is not None and text.startswith(k + ":"):
                out[cur][short] = int(text.split(":", 1)[1].strip())
    filt = shutil.which("llvm-cxxfilt") or "/opt/rocm/llvm/bin/llvm-cxxfilt"
    if names and os.path.exists(filt):
        dem = subprocess.run([filt], input="\n".join(names), capture_output=True, text=True).stdout.splitlines()
        if len(dem) == len(names):
            out = {d: out[n] for d, n in zip(dem, names)}
    return out


if __name__ == "__main__":
    print(build_library(timeline="--timeline" in sys.argv[1:]))
