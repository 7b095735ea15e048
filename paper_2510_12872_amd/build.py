"""Build libkvcomm.so (the C-ABI library of include/kvcomm.h) for gfx950 with hipcc, and the stand-alone
HBM streaming probe that bench.py --hbm-calibration runs.

hipcc cross-compiles without a GPU, so this runs anywhere the ROCm toolchain is installed.
The library is written next to this file; tests, the smoke check and the benchmark load
that file and never compile anything themselves.
"""
import os
import shutil
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libkvcomm.so")
PROBE_SRC = os.path.join(_HERE, "tools", "hbm_stream_probe.hip")
PROBE = os.path.join(_HERE, "tools", "hbm_stream_probe")
SOURCES = ["align_kv.hip", "anchor_weights.hip", "anchor_update.hip", "delta_q8.hip", "suffix_attn.hip", "status.hip"]

# -packed-fp32-ops: keep the compiler from forming packed fp32 instructions.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def hipcc_path():
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the HIP library cannot be built")


def build(verbose=False, extra_flags=()):
    """Compile every HIP source into libkvcomm.so.  Always recompiles."""
    cmd = [hipcc_path()] + HIPCC_FLAGS + list(extra_flags) + ["-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    probe = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument", "-o", PROBE, PROBE_SRC]
    if verbose:
        print(" ".join(probe))
    subprocess.run(probe, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
