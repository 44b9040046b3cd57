"""Builds the plain-C caller of the C ABI (test infrastructure)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SOURCE = os.path.join(HERE, "abi_client.c")
BINARY = os.path.join(HERE, "abi_client.bin")


def build(force: bool = False) -> str:
    """gcc -std=c99 against include/specsteer.h, libspecsteer.so and the HIP runtime."""
    if force or not os.path.exists(BINARY) or os.path.getmtime(BINARY) < os.path.getmtime(SOURCE):
        libdir = os.path.join(ROOT, "paper_2603_16219_amd")
        cmd = ["gcc", "-std=c99", "-Wall", "-O1", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
               "-I" + os.path.join(ROOT, "include"), SOURCE, "-o", BINARY, "-L" + libdir, "-lspecsteer",
               "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-Wl,-rpath," + libdir]
        subprocess.run(cmd, check=True, capture_output=True)
    return BINARY
