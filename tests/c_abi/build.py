"""Builds the torch-free C ABI check (c_abi_check.cpp) against the in-tree librapid.so and the oracle."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "c_abi_check")


def build(verbose: bool = False) -> str:
    pkg, orc = os.path.join(ROOT, "paper_2502_20330_amd"), os.path.join(ROOT, "oracle")
    cmd = ["hipcc", "-O2", "-std=c++17", "--offload-arch=gfx950", "-I", os.path.join(ROOT, "include"),
           os.path.join(HERE, "c_abi_check.cpp"), "-o", EXE,
           "-L", pkg, "-lrapid", "-L", orc, "-lrapid_oracle",
           "-Wl,-rpath," + pkg, "-Wl,-rpath," + orc,
           "-Wl,-rpath,$ORIGIN/../../paper_2502_20330_amd", "-Wl,-rpath,$ORIGIN/../../oracle"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"building c_abi_check failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print("built", EXE)
    return EXE


if __name__ == "__main__":
    build(verbose=True)
