"""Builds tests/c_abi/check: a plain C11 program (gcc, no HIP compiler, no Python) that drives the
library through include/pre3.h; run by tests/test_gpu_c_abi.py."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
BINARY = os.path.join(HERE, "check")


def build() -> str:
    lib_dir = os.path.join(ROOT, "paper_2506_03887_amd")
    cmd = ["gcc", "-O1", "-std=c11", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-o", BINARY,
           os.path.join(HERE, "check.c"), "-L" + lib_dir, "-lpre3", "-L/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_2506_03887_amd", "-Wl,-rpath,/opt/rocm/lib"]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("gcc failed:\n" + proc.stderr)
    return BINARY


if __name__ == "__main__":
    print(build())
