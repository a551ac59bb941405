"""Builds libadseq.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "adseq.hip")
LIB = os.path.join(HERE, "libadseq.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",          # the LIF update spells its one fma out; nothing else may fuse
    "-munsafe-fp-atomics",        # hardware fp32 atomic add for the batched gradient accumulation
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
]


LIB_PHASE = os.path.join(HERE, "libadseq_phase.so")


def build_library(verbose: bool = False, phase_clocks: bool = False) -> str:
    """phase_clocks: a second library, libadseq_phase.so, whose window expansion and resident step
    kernels clock their phases (bench.py --phase-clocks reads them); the product library has none."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if phase_clocks:
        cmd = [hipcc] + HIPCC_FLAGS + ["-DADSEQ_PHASE_CLOCK", "-o", LIB_PHASE, SRC]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return LIB_PHASE
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def build_copy_reference() -> str:
    """The plain copy program that the HBM traffic counters are calibrated with."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(HERE, "copy_ref")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", "-o", out, os.path.join(HERE, "csrc", "copy_ref.hip")])
    return out


def build_chip_rates() -> str:
    """The program that measures the launch, atomic, store and gather rates the design rests on."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(HERE, "chip_rates")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", "-o", out, os.path.join(HERE, "csrc", "chip_rates.hip")])
    return out


if __name__ == "__main__":
    import sys
    if "--phase-clocks" in sys.argv[1:]:
        print(build_library(verbose=True, phase_clocks=True))
        sys.exit(0)
    print(build_library(verbose=True))
    print(build_copy_reference())
    print(build_chip_rates())
