"""ctypes binding of include/jot.h.  Same names as the C entry points; arguments are plain
integers (device addresses, e.g. torch.Tensor.data_ptr()) and Python numbers.  Nothing is
computed here."""
from __future__ import annotations

import ctypes
import os

import numpy as np

__all__ = [
    "JOT_F32", "JOT_BF16", "JOT_CONF_RATIO", "JOT_CONF_MAXPROB", "JOT_CONF_PROBGAP",
    "JotParams", "JotError", "load_library", "library_path",
    "jot_workspace_bytes", "jot_init_state", "jot_step", "jot_step_scheduled", "jot_step_sampled", "jot_step_ex", "jot_step_static", "JOT_STATIC_MAX_WORKSPACE", "JotStepOptions", "jot_last_flags", "jot_last_kl", "jot_last_gap", "jot_last_final_token", "jot_active_count", "jot_active_count_poll", "jot_wait_on_stream", "jot_step_index",
    "jot_anomaly_count", "jot_tokens", "jot_masked", "jot_commit_step", "jot_active_list",
    "jot_commit_log", "jot_examined_list", "jot_last_token", "jot_last_conf", "jot_last_p1",
    "jot_last_p2", "jot_last_tau", "jot_profile_enable", "jot_profile_read", "jot_release",
    "jot_strerror", "device_to_host",
]

JOT_F32, JOT_BF16 = 0, 1
JOT_CONF_RATIO, JOT_CONF_MAXPROB, JOT_CONF_PROBGAP = 0, 1, 2
JOT_STATIC_MAX_WORKSPACE = 4 << 20

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "_lib", "libjot.so")


class JotParams(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("L", ctypes.c_int32), ("V", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("conf_mode", ctypes.c_int32),
        ("tau_max", ctypes.c_float), ("tau_min", ctypes.c_float), ("gamma", ctypes.c_float),
        ("D", ctypes.c_int32), ("eps", ctypes.c_float),
        ("gen_start", ctypes.c_int32), ("block_size", ctypes.c_int32),
    ]


class JotStepOptions(ctypes.Structure):
    _fields_ = [
        ("n_transfer_dev", ctypes.c_void_p), ("transfer_frac", ctypes.c_float),
        ("uniforms_dev", ctypes.c_void_p), ("enable_global_gap", ctypes.c_int32),
        ("global_gap", ctypes.c_float),
        ("enable_kl", ctypes.c_int32), ("prev_logits_dev", ctypes.c_void_p),
        ("kl_threshold", ctypes.c_float), ("kl_min_prob", ctypes.c_float),
        ("logits_compact", ctypes.c_int32),
    ]


class JotError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {jot_strerror(code)} ({code})")


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libjot.so.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with "
                          "`python -m paper_2602_11133_amd.build` (hipcc, gfx950)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    pp = ctypes.POINTER(JotParams)
    sig = {
        "jot_workspace_bytes": (i64, [pp]),
        "jot_init_state": (ctypes.c_int, [ctypes.POINTER(vp), pp, vp, i64, vp, vp, vp]),
        "jot_step": (ctypes.c_int, [vp, vp, i64, i64, vp]),
        "jot_step_scheduled": (ctypes.c_int, [vp, vp, i64, i64, vp, ctypes.c_float, vp]),
        "jot_step_sampled": (ctypes.c_int, [vp, vp, i64, i64, vp, ctypes.c_float, vp, vp]),
        "jot_step_ex": (ctypes.c_int, [vp, vp, i64, i64, ctypes.POINTER(JotStepOptions), vp]),
        "jot_step_static": (ctypes.c_int, [pp, vp, i64, i64, vp, vp, vp, vp, vp]),
        "jot_last_flags": (vp, [vp]), "jot_last_kl": (vp, [vp]), "jot_last_gap": (vp, [vp]), "jot_last_final_token": (vp, [vp]),
        "jot_active_count": (i64, [vp]),
        "jot_active_count_poll": (i64, [vp, ctypes.POINTER(i32)]),
        "jot_wait_on_stream": (ctypes.c_int, [vp, vp]),
        "jot_step_index": (i32, [vp]),
        "jot_anomaly_count": (i64, [vp]),
        "jot_tokens": (vp, [vp]), "jot_masked": (vp, [vp]), "jot_commit_step": (vp, [vp]),
        "jot_active_list": (vp, [vp]),
        "jot_commit_log": (vp, [vp, ctypes.POINTER(i64)]),
        "jot_examined_list": (vp, [vp, ctypes.POINTER(i64)]),
        "jot_last_token": (vp, [vp]), "jot_last_conf": (vp, [vp]), "jot_last_p1": (vp, [vp]),
        "jot_last_p2": (vp, [vp]), "jot_last_tau": (vp, [vp]),
        "jot_profile_enable": (ctypes.c_int, [vp, ctypes.c_int]),
        "jot_profile_read": (ctypes.c_int, [vp, i32, ctypes.POINTER(ctypes.c_float)]),
        "jot_release": (None, [vp]),
        "jot_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _check(rc: int, where: str) -> int:
    if rc < 0:
        raise JotError(int(rc), where)
    return int(rc)


def jot_strerror(code: int) -> str:
    return load_library().jot_strerror(int(code)).decode()


def jot_workspace_bytes(p: JotParams) -> int:
    return _check(load_library().jot_workspace_bytes(ctypes.byref(p)), "jot_workspace_bytes")


def jot_init_state(p: JotParams, workspace_dev: int, workspace_bytes: int, tokens_dev: int,
                   masked_dev: int, stream: int = 0) -> int:
    """Returns the state handle (an integer)."""
    out = ctypes.c_void_p()
    _check(load_library().jot_init_state(ctypes.byref(out), ctypes.byref(p), workspace_dev,
                                         workspace_bytes, tokens_dev, masked_dev, stream),
           "jot_init_state")
    return out.value


def jot_step(s: int, logits_dev: int, stride_b: int, stride_l: int, stream: int = 0) -> None:
    _check(load_library().jot_step(s, logits_dev, stride_b, stride_l, stream), "jot_step")


def jot_step_scheduled(s: int, logits_dev: int, stride_b: int, stride_l: int, n_transfer_dev: int,
                       transfer_frac: float, stream: int = 0) -> None:
    _check(load_library().jot_step_scheduled(s, logits_dev, stride_b, stride_l, n_transfer_dev or None,
                                             float(transfer_frac), stream), "jot_step_scheduled")


def jot_step_sampled(s: int, logits_dev: int, stride_b: int, stride_l: int, n_transfer_dev: int,
                     transfer_frac: float, uniforms_dev: int, stream: int = 0) -> None:
    _check(load_library().jot_step_sampled(s, logits_dev, stride_b, stride_l, n_transfer_dev or None,
                                           float(transfer_frac), uniforms_dev or None, stream),
           "jot_step_sampled")


def jot_step_ex(s: int, logits_dev: int, stride_b: int, stride_l: int, opt: "JotStepOptions | None",
                stream: int = 0) -> None:
    _check(load_library().jot_step_ex(s, logits_dev, stride_b, stride_l,
                                      ctypes.byref(opt) if opt is not None else None, stream), "jot_step_ex")


def jot_step_static(p: JotParams, logits_dev: int, stride_b: int, stride_l: int, tokens_dev: int,
                    masked_dev: int, active_out_dev: int, n_active_out_dev: int, stream: int = 0) -> None:
    _check(load_library().jot_step_static(ctypes.byref(p), logits_dev, stride_b, stride_l, tokens_dev, masked_dev,
                                          active_out_dev, n_active_out_dev, stream), "jot_step_static")


def jot_active_count(s: int) -> int:
    return _check(load_library().jot_active_count(s), "jot_active_count")


def jot_active_count_poll(s: int):
    """(count stored by the last completed step, number of completed steps); never waits."""
    done = ctypes.c_int32()
    n = _check(load_library().jot_active_count_poll(s, ctypes.byref(done)), "jot_active_count_poll")
    return n, done.value


def jot_wait_on_stream(s: int, stream: int) -> None:
    _check(load_library().jot_wait_on_stream(s, stream), "jot_wait_on_stream")


def jot_step_index(s: int) -> int:
    return _check(load_library().jot_step_index(s), "jot_step_index")


def jot_anomaly_count(s: int) -> int:
    return _check(load_library().jot_anomaly_count(s), "jot_anomaly_count")


def _ptr(name: str, s: int) -> int:
    p = getattr(load_library(), name)(s)
    if not p:
        raise JotError(-2, name)
    return p


def jot_tokens(s: int) -> int: return _ptr("jot_tokens", s)
def jot_masked(s: int) -> int: return _ptr("jot_masked", s)
def jot_commit_step(s: int) -> int: return _ptr("jot_commit_step", s)
def jot_active_list(s: int) -> int: return _ptr("jot_active_list", s)
def jot_last_token(s: int) -> int: return _ptr("jot_last_token", s)
def jot_last_conf(s: int) -> int: return _ptr("jot_last_conf", s)
def jot_last_p1(s: int) -> int: return _ptr("jot_last_p1", s)
def jot_last_p2(s: int) -> int: return _ptr("jot_last_p2", s)
def jot_last_tau(s: int) -> int: return _ptr("jot_last_tau", s)
def jot_last_flags(s: int) -> int: return _ptr("jot_last_flags", s)
def jot_last_kl(s: int) -> int: return _ptr("jot_last_kl", s)
def jot_last_gap(s: int) -> int: return _ptr("jot_last_gap", s)
def jot_last_final_token(s: int) -> int: return _ptr("jot_last_final_token", s)


def jot_commit_log(s: int):
    """(device address, number of triples)"""
    n = ctypes.c_int64()
    p = load_library().jot_commit_log(s, ctypes.byref(n))
    if not p:
        raise JotError(-6, "jot_commit_log")
    return p, n.value


def jot_examined_list(s: int):
    """(device address, number of entries)"""
    n = ctypes.c_int64()
    p = load_library().jot_examined_list(s, ctypes.byref(n))
    if not p:
        raise JotError(-6, "jot_examined_list")
    return p, n.value


def jot_profile_enable(s: int, on: bool) -> None:
    _check(load_library().jot_profile_enable(s, int(bool(on))), "jot_profile_enable")


def jot_profile_read(s: int, step: int) -> float:
    """Milliseconds the vocabulary-reduction kernel of step `step` took."""
    ms = ctypes.c_float()
    _check(load_library().jot_profile_read(s, int(step), ctypes.byref(ms)), "jot_profile_read")
    return ms.value


def jot_release(s: int) -> None:
    load_library().jot_release(s)


# ---- plumbing: synchronous device -> host copy of a raw device range into a numpy array -------
_hip = None


def device_to_host(dev_ptr: int, count: int, dtype) -> np.ndarray:
    """hipMemcpy of `count` elements of `dtype` starting at device address dev_ptr."""
    global _hip
    out = np.empty(int(count), dtype)
    if count == 0:
        return out
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
        _hip.hipMemcpy.restype = ctypes.c_int
    rc = _hip.hipMemcpy(out.ctypes.data, dev_ptr, out.nbytes, 2)   # 2 = hipMemcpyDeviceToHost
    if rc != 0:
        raise RuntimeError(f"hipMemcpy failed with {rc}")
    return out
