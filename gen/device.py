"""ctypes binding of the device generator.  torch is used for device memory only."""
import ctypes

import numpy as np
import torch

from . import build as _build
from .configs import F32, JotConfig
from .host import NOISE_STREAM
from .tables import build_table

_lib = None


def _load():
    global _lib
    if _lib is None:
        import os
        if not os.path.exists(_build.DEV_LIB):
            _build.build_device()
        lib = ctypes.CDLL(_build.DEV_LIB)
        vp, i64, i32, u32, u64 = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32,
                                  ctypes.c_uint64)
        lib.jotgen_rows_device.restype = ctypes.c_int
        lib.jotgen_rows_device.argtypes = [vp, ctypes.c_int, i64, i64, i32, i32, vp, vp, i64, u32, u64,
                                           u32, vp, vp, vp, vp, vp, vp]
        lib.jotgen_fill_device.restype = ctypes.c_int
        lib.jotgen_fill_device.argtypes = [vp, i64, u32, vp]
        _lib = lib
    return _lib


class DeviceGenerator:
    """Writes logit rows of a configuration straight into a [B, L, V] device tensor."""

    def __init__(self, cfg: JotConfig, target: np.ndarray, rival: np.ndarray, device="cuda:0"):
        self.cfg = cfg
        self.device = torch.device(device)
        self.table = torch.from_numpy(build_table(cfg.noise, cfg.noise_scale)).to(self.device)
        self.target = torch.from_numpy(np.ascontiguousarray(target, np.int32)).to(self.device)
        self.rival = torch.from_numpy(np.ascontiguousarray(rival, np.int32)).to(self.device)
        self.T = torch.zeros(cfg.B * cfg.L, dtype=torch.float32, device=self.device)
        self.R = torch.zeros(cfg.B * cfg.L, dtype=torch.float32, device=self.device)

    def alloc_logits(self, poison: bool = True) -> torch.Tensor:
        cfg = self.cfg
        dt = torch.float32 if cfg.dtype == F32 else torch.bfloat16
        t = torch.empty((cfg.B, cfg.L, cfg.V), dtype=dt, device=self.device)
        if poison:
            self.poison(t)
        return t

    def poison(self, t: torch.Tensor) -> None:
        """Fill with NaN bit patterns: rows that are never generated must never be read."""
        n_words = t.numel() * t.element_size() // 4
        word = 0x7FC07FC0 if t.element_size() == 2 else 0x7FC00000
        rc = _load().jotgen_fill_device(t.data_ptr(), n_words, word, torch.cuda.current_stream().cuda_stream)
        assert rc == 0, rc

    def set_planted(self, T: np.ndarray, R: np.ndarray) -> None:
        self.T.copy_(torch.from_numpy(np.ascontiguousarray(T, np.float32)))
        self.R.copy_(torch.from_numpy(np.ascontiguousarray(R, np.float32)))

    def fill(self, logits: torch.Tensor, step: int, pos_dev_ptr: int, n_rows: int, n_rows_dev_ptr: int = 0):
        """Generate rows for the positions listed (int32, device) at pos_dev_ptr."""
        cfg = self.cfg
        assert logits.is_contiguous() and tuple(logits.shape) == (cfg.B, cfg.L, cfg.V)
        rc = _load().jotgen_rows_device(
            logits.data_ptr(), cfg.dtype, cfg.L * cfg.V, cfg.V, cfg.L, cfg.V, pos_dev_ptr,
            n_rows_dev_ptr or None, n_rows, step, cfg.seed, NOISE_STREAM, self.table.data_ptr(),
            self.target.data_ptr(), self.T.data_ptr(), self.rival.data_ptr(), self.R.data_ptr(),
            torch.cuda.current_stream().cuda_stream)
        assert rc == 0, rc
