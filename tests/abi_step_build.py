"""Compile tests/abi_step.c (a plain-C consumer of the C ABI, checked against the C oracle)
into tests/abi_step.bin.  Needs libeep.so and liboracle.so to exist; no GPU needed to build."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "abi_step.c")
BIN = os.path.join(HERE, "abi_step.bin")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build() -> str:
    lib_dir, oracle_dir = os.path.join(ROOT, "paper_2605_10670_amd"), os.path.join(ROOT, "oracle")
    # libraries are named, not given by path, and found at run time relative to the binary,
    # so that the tree can be moved
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROCM, "include"), SRC, "-o", BIN,
           "-L", lib_dir, "-l:libeep.so", "-L", oracle_dir, "-l:liboracle.so",
           "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../paper_2605_10670_amd", "-Wl,-rpath,$ORIGIN/../oracle",
           "-Wl,-rpath," + os.path.join(ROCM, "lib")]
    subprocess.run(cmd, check=True)
    return BIN


if __name__ == "__main__":
    print(build())
