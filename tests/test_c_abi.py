"""Host-only checks of the C ABI: the library loads without a GPU, exports every function the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2602_11133_amd as J
from paper_2602_11133_amd import build as jbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def built():
    if not os.path.exists(J.library_path()):
        jbuild.build()


def good():
    return J.JotParams(B=2, L=64, V=1000, dtype=J.JOT_F32, conf_mode=J.JOT_CONF_RATIO, tau_max=90.0,
                       tau_min=1.0, gamma=0.5, D=8, eps=1e-12, gen_start=16, block_size=0)


def test_every_declared_function_is_exported():
    text = open(os.path.join(ROOT, "include", "jot.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(jot_[a-z0-9_]+)\s*\(", text))
    assert {"jot_init_state", "jot_step", "jot_active_count", "jot_workspace_bytes"} <= declared
    lib = ctypes.CDLL(J.library_path())
    for name in declared:
        assert hasattr(lib, name), name
    # the binding offers the same names
    for name in declared:
        assert hasattr(J, name), name


def test_workspace_size_is_positive_and_aligned():
    n = J.jot_workspace_bytes(good())
    assert n > 0 and n % 256 == 0


@pytest.mark.parametrize("field,value,code", [
    ("V", 1, -1), ("B", 0, -1), ("L", 0, -1), ("dtype", 2, -3), ("conf_mode", 3, -1),
    ("D", -1, -1), ("D", 33, -1), ("gamma", 0.0, -1), ("gamma", 1.5, -1), ("gamma", float("nan"), -1),
    ("tau_min", 100.0, -1), ("tau_max", float("inf"), -1), ("eps", -1e-3, -1),
    ("gen_start", -1, -1), ("gen_start", 65, -1), ("block_size", -2, -1),
])
def test_invalid_parameters_are_rejected(field, value, code):
    p = good()
    setattr(p, field, value)
    with pytest.raises(J.JotError) as e:
        J.jot_workspace_bytes(p)
    assert e.value.code == code


def test_init_rejects_bad_pointers_before_any_device_work():
    p = good()
    n = J.jot_workspace_bytes(p)
    with pytest.raises(J.JotError) as e:
        J.jot_init_state(p, 0, n, 4096, 4096)
    assert e.value.code == -2                       # null workspace
    with pytest.raises(J.JotError) as e:
        J.jot_init_state(p, 4096 + 8, n, 4096, 4096)
    assert e.value.code == -5                       # misaligned workspace
    with pytest.raises(J.JotError) as e:
        J.jot_init_state(p, 4096, n - 1, 4096, 4096)
    assert e.value.code == -4                       # too small
    with pytest.raises(J.JotError) as e:
        J.jot_init_state(p, 4096, n, 0, 4096)
    assert e.value.code == -2


def test_null_state_is_an_error_not_a_crash():
    lib = J.load_library()
    assert lib.jot_step(None, None, 0, 0, None) == -2
    assert lib.jot_active_count(None) == -2
    assert lib.jot_tokens(None) is None
    lib.jot_release(None)
    assert J.jot_strerror(-4) == "workspace too small"
    assert J.jot_strerror(0) == "success"


def test_static_entry_point_rejects_bad_arguments_before_any_device_work():
    p = good()
    sb, sl = p.L * p.V, p.V

    def call(pp=p, logits=4096, stride_b=sb, stride_l=sl, tok=4096, msk=4096, act=4096, cnt=4096):
        return J.load_library().jot_step_static(ctypes.byref(pp) if pp is not None else None, logits, stride_b,
                                                stride_l, tok, msk, act, cnt, None)

    assert call(pp=None) == -2
    assert call(tok=None) == -2 and call(msk=None) == -2 and call(act=None) == -2 and call(cnt=None) == -2
    assert call(logits=None) == -2
    assert call(tok=4098) == -5 and call(act=4098) == -5 and call(cnt=4100) == -5 and call(logits=4104) == -5
    assert call(stride_l=p.V - 1) == -1 and call(stride_b=1) == -1
    bad = good()
    bad.V = 1
    assert call(pp=bad) == -1
    big = good()
    big.B, big.L = 64, 1280
    assert J.jot_workspace_bytes(big) > J.JOT_STATIC_MAX_WORKSPACE
    assert call(pp=big, stride_b=big.L * big.V) == -10
    assert "scratch" in J.jot_strerror(-10)


def test_poll_and_wait_calls_reject_a_null_state():
    lib = J.load_library()
    assert lib.jot_active_count_poll(None, None) == -2
    assert lib.jot_wait_on_stream(None, None) == -2
    assert lib.jot_step_index(None) == -2
    assert lib.jot_anomaly_count(None) == -2


def test_package_has_no_cpu_fallback():
    # the binding computes nothing: it must not import the oracle or numpy math paths for the method
    src = open(os.path.join(ROOT, "paper_2602_11133_amd", "binding.py")).read()
    assert "oracle" not in src


def test_header_is_valid_c_and_cpp(tmp_path):
    import subprocess
    src = tmp_path / "use_jot.c"
    src.write_text('#include "jot.h"\nint main(void) { jot_params p; p.B = 1; (void)p; return jot_workspace_bytes(0) < 0 ? 0 : 1; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc, str(src)])
    subprocess.check_call(["g++", "-std=c++11", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)])
