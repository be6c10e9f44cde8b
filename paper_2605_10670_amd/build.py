"""Compile the HIP sources under csrc/ into paper_2605_10670_amd/libeep.so for gfx950."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libeep.so")
SOURCES = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")) +
                 glob.glob(os.path.join(HERE, "csrc", "*.cpp")))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
]


def build() -> str:
    cmd = [HIPCC] + FLAGS + ["-o", LIB] + SOURCES
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
