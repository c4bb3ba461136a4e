"""Builds the C program that drives the C ABI (tests/abi_example/abi_example.c) with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SRC = os.path.join(HERE, "abi_example.c")
EXE = os.path.join(HERE, "abi_example")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def is_stale() -> bool:
    lib = os.path.join(ROOT, "paper_2504_17096_amd", "libsailor.so")
    deps = [SRC, os.path.join(ROOT, "include", "sailor.h")]
    if not os.path.exists(EXE):
        return True
    t = os.path.getmtime(EXE)
    return any(os.path.getmtime(f) > t for f in deps) or not os.path.exists(lib)


def build(force: bool = True) -> str:
    if force or is_stale():
        subprocess.check_call([
            "gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__",
            "-I" + os.path.join(ROCM, "include"), "-I" + os.path.join(ROOT, "include"), SRC, "-o", EXE,
            "-L" + os.path.join(ROOT, "paper_2504_17096_amd"), "-lsailor",
            "-L" + os.path.join(ROCM, "lib"), "-lamdhip64", "-lm",
            "-Wl,-rpath,$ORIGIN/../../paper_2504_17096_amd", "-Wl,-rpath," + os.path.join(ROCM, "lib")])
    return EXE


if __name__ == "__main__":
    print(build())
