"""Builds tests/abi_gpu/abi_forward (plain C, gcc) against libradial.so and the HIP runtime."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "abi_forward")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build(extra_flags=()) -> str:
    libdir = os.path.join(ROOT, "paper_2506_19852_amd")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__", *extra_flags,
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROCM, "include"),
           os.path.join(HERE, "abi_forward.c"), "-o", EXE,
           "-L", libdir, "-lradial", f"-Wl,-rpath,{libdir}", "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
           f"-Wl,-rpath,{os.path.join(ROCM, 'lib')}", "-lm"]
    subprocess.check_call(cmd)
    return EXE


if __name__ == "__main__":
    print(build())
