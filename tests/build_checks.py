"""Compile tests/csrc/device_checks.hip (exhaustive device-side checks of the kernels' arithmetic shortcuts) into
tests/libbof4_device_checks.so.  Test infrastructure only."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libbof4_device_checks.so")
SRC = os.path.join(HERE, "csrc", "device_checks.hip")


def build() -> str:
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC", "-Wno-unused-function",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "paper_2505_06653_amd", "csrc"), "-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
