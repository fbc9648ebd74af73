"""ctypes binding of the host generator."""
import ctypes

import numpy as np

from . import build as _build
from .configs import BF16, F32, JotConfig
from .tables import build_table

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build_host())
        lib.jotgen_rows_host.restype = None
        lib.jotgen_rows_host.argtypes = [
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int32, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint32,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int]
        lib.jotgen_philox4x32.restype = None
        lib.jotgen_philox4x32.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def philox4x32(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, np.uint32)
    k = np.asarray(key, np.uint32)
    out = np.zeros(4, np.uint32)
    _load().jotgen_philox4x32(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


NOISE_STREAM = 0


class HostGenerator:
    """Logit rows of a configuration on the host.  rows(step, pos, T, R) -> [len(pos), V] array
    (float32, or uint16 bf16 bit patterns); the array is a view of an internal buffer that the
    next call reuses."""

    def __init__(self, cfg: JotConfig, target: np.ndarray, rival: np.ndarray, threads: int = 1):
        self.cfg = cfg
        self.table = build_table(cfg.noise, cfg.noise_scale)
        self.target = np.ascontiguousarray(target, np.int32)
        self.rival = np.ascontiguousarray(rival, np.int32)
        self.threads = threads
        self._buf = None

    def rows(self, step: int, pos: np.ndarray, T: np.ndarray, R: np.ndarray) -> np.ndarray:
        cfg = self.cfg
        pos = np.ascontiguousarray(pos, np.int64)
        T = np.ascontiguousarray(T, np.float32)
        R = np.ascontiguousarray(R, np.float32)
        assert T.size == R.size == self.target.size == cfg.B * cfg.L
        # one reusable buffer: the returned array is a view that the next call overwrites
        need = pos.size * cfg.V
        if self._buf is None or self._buf.size < need:
            self._buf = np.zeros(max(need, 1), np.float32 if cfg.dtype == F32 else np.uint16)
        out = self._buf[:need].reshape(pos.size, cfg.V)
        if pos.size:
            _load().jotgen_rows_host(
                out.ctypes.data, cfg.dtype, pos.size, cfg.V, cfg.V, pos.ctypes.data,
                step, cfg.seed, NOISE_STREAM, self.table.ctypes.data, self.target.ctypes.data,
                T.ctypes.data, self.rival.ctypes.data, R.ctypes.data, self.threads)
        return out
