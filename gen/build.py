"""Build the generator libraries: host (gcc) and device (hipcc, gfx950)."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
HOST_SRC = os.path.join(_HERE, "csrc", "jotgen_host.c")
DEV_SRC = os.path.join(_HERE, "csrc", "jotgen_device.hip")
HOST_LIB = os.path.join(_HERE, "_lib", "libjotgen_host.so")
DEV_LIB = os.path.join(_HERE, "_lib", "libjotgen_device.so")


def _stale(lib, src):
    return not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src)


def build_host(force=False) -> str:
    if force or _stale(HOST_LIB, HOST_SRC):
        os.makedirs(os.path.dirname(HOST_LIB), exist_ok=True)
        subprocess.check_call(["gcc", "-O3", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC",
                               "-shared", "-Wall", "-Wextra", "-o", HOST_LIB, HOST_SRC])
    return HOST_LIB


def build_device(force=False) -> str:
    if force or _stale(DEV_LIB, DEV_SRC):
        os.makedirs(os.path.dirname(DEV_LIB), exist_ok=True)
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O3", "-ffp-contract=off",
                               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                               "-fPIC", "-shared", "-o", DEV_LIB, DEV_SRC])
    return DEV_LIB
