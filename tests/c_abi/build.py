"""Builds tests/c_abi/round: a HIP host program that drives the C ABI without Python and
checks one round against the oracle (test infrastructure; both libraries are found through
rpath, so they must have been built first)."""
import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))


def build(verbose: bool = False) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    exe = os.path.join(HERE, "round")
    cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-ffp-contract=off",
           "-I", os.path.join(ROOT, "include"), os.path.join(HERE, "round.cpp"), "-o", exe,
           "-L", os.path.join(ROOT, "paper_2508_15706_amd"), "-lsparseloco",
           "-L", os.path.join(ROOT, "oracle"), "-lsparseloco_oracle",
           "-Wl,-rpath,$ORIGIN/../../paper_2508_15706_amd", "-Wl,-rpath,$ORIGIN/../../oracle"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return exe


if __name__ == "__main__":
    print(build(verbose=True))
