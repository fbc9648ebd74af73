"""Build libjot.so (the C-ABI library) for gfx950 with hipcc.  Cross-compiles without a GPU."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "_lib", "libjot.so")
PROBE_LIB = os.path.join(_HERE, "_lib", "libjot_probe.so")
PROBE_SRC = os.path.join(CSRC, "jot_probe.hip")
SOURCES = ["jot_api.hip"]
HEADERS = ["jot_device.h", "jot_vocab_reduce.h", "jot_decide.h", "jot_compact.h", "jot_schedule.h", "jot_sample.h", "jot_row_step.h",
           os.path.join("..", "..", "include", "jot.h")]

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall"]


def _stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force: bool = False, extra_flags=()) -> str:
    if force or _stale():
        os.makedirs(os.path.dirname(LIB), exist_ok=True)
        cmd = ["hipcc", *HIPCC_FLAGS, *extra_flags, "-o", LIB] + [os.path.join(CSRC, f) for f in SOURCES]
        subprocess.check_call(cmd)
    return LIB


def build_probe(force: bool = False) -> str:
    """Measurement kernels (plain copy / plain read), used by bench.py only."""
    if force or not os.path.exists(PROBE_LIB) or os.path.getmtime(PROBE_LIB) < os.path.getmtime(PROBE_SRC):
        os.makedirs(os.path.dirname(PROBE_LIB), exist_ok=True)
        subprocess.check_call(["hipcc", *HIPCC_FLAGS, "-o", PROBE_LIB, PROBE_SRC])
    return PROBE_LIB


if __name__ == "__main__":
    print(build(force=True))
    print(build_probe(force=True))
