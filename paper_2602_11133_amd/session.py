"""A decoding state on the GPU as a Python object: allocates the workspace as a torch tensor,
marshals arguments into the C entry points and copies results back to numpy arrays.  Nothing is
computed here; torch supplies device memory and the stream only."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as J


class JotSession:
    """One decoding state on the GPU (jot_init_state ... jot_release)."""

    def __init__(self, params: J.JotParams, tokens: np.ndarray, masked: np.ndarray, device="cuda:0"):
        self.p = params
        self.dev = torch.device(device)
        self.n = params.B * params.L
        self.ws_bytes = J.jot_workspace_bytes(params)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.dev)
        assert self.ws.data_ptr() % 256 == 0
        tok = torch.from_numpy(np.ascontiguousarray(tokens, np.int32)).to(self.dev)
        msk = torch.from_numpy(np.ascontiguousarray(masked, np.uint8)).to(self.dev)
        self.stream = torch.cuda.current_stream().cuda_stream
        self.h = J.jot_init_state(params, self.ws.data_ptr(), self.ws_bytes, tok.data_ptr(),
                                  msk.data_ptr(), self.stream)

    def close(self):
        if self.h:
            torch.cuda.synchronize()
            J.jot_release(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step(self, logits: torch.Tensor, stride_b=None, stride_l=None, n_transfer=None, transfer_frac=0.0,
             uniforms=None, global_gap=None, kl=None, prev_logits=None, compact=False):
        """kl = (kl_threshold, kl_min_prob) turns the KL stability rule on; prev_logits is then the
        tensor the previous step was given (same layout).  compact: `logits` is [n_examined, stride]
        with one row per entry of the examined list."""
        if compact:
            sb, sl = 0, (logits.stride(0) if stride_l is None else stride_l)
        else:
            sb = logits.stride(0) if stride_b is None else stride_b
            sl = logits.stride(1) if stride_l is None else stride_l
        if global_gap is not None or kl is not None or compact:     # the general entry point
            opt = J.JotStepOptions()
            if n_transfer is not None:
                self._nt = torch.from_numpy(np.ascontiguousarray(n_transfer, np.int32)).to(self.dev)
                opt.n_transfer_dev = self._nt.data_ptr()
            opt.transfer_frac = transfer_frac
            if uniforms is not None:
                self._u = torch.from_numpy(np.ascontiguousarray(uniforms, np.float32)).to(self.dev)
                opt.uniforms_dev = self._u.data_ptr()
            if global_gap is not None:
                opt.enable_global_gap = 1
                opt.global_gap = global_gap
            opt.logits_compact = 1 if compact else 0
            if kl is not None:
                assert prev_logits.stride() == logits.stride() and prev_logits.dtype == logits.dtype
                opt.enable_kl = 1
                opt.prev_logits_dev = prev_logits.data_ptr()
                opt.kl_threshold, opt.kl_min_prob = kl
            J.jot_step_ex(self.h, logits.data_ptr(), sb, sl, opt, self.stream)
            return
        if uniforms is not None:
            self._u = torch.from_numpy(np.ascontiguousarray(uniforms, np.float32)).to(self.dev)
            nt = 0
            if n_transfer is not None:
                self._nt = torch.from_numpy(np.ascontiguousarray(n_transfer, np.int32)).to(self.dev)
                nt = self._nt.data_ptr()
            J.jot_step_sampled(self.h, logits.data_ptr(), sb, sl, nt, transfer_frac, self._u.data_ptr(), self.stream)
            return
        if n_transfer is None and transfer_frac == 0.0:
            J.jot_step(self.h, logits.data_ptr(), sb, sl, self.stream)
            return
        nt = 0
        if n_transfer is not None:
            self._nt = torch.from_numpy(np.ascontiguousarray(n_transfer, np.int32)).to(self.dev)
            nt = self._nt.data_ptr()
        J.jot_step_scheduled(self.h, logits.data_ptr(), sb, sl, nt, transfer_frac, self.stream)

    # ---- read-back
    def active_count(self) -> int:
        return J.jot_active_count(self.h)

    def active_list(self) -> np.ndarray:
        n = self.active_count()
        return J.device_to_host(J.jot_active_list(self.h), n, np.int32)

    def tokens(self) -> np.ndarray:
        self.active_count()
        return J.device_to_host(J.jot_tokens(self.h), self.n, np.int32).reshape(self.p.B, self.p.L)

    def masked(self) -> np.ndarray:
        self.active_count()
        return J.device_to_host(J.jot_masked(self.h), self.n, np.uint8).reshape(self.p.B, self.p.L).astype(bool)

    def commit_step(self) -> np.ndarray:
        self.active_count()
        return J.device_to_host(J.jot_commit_step(self.h), self.n, np.int32).reshape(self.p.B, self.p.L)

    def commit_log(self) -> np.ndarray:
        ptr, n = J.jot_commit_log(self.h)
        return J.device_to_host(ptr, 3 * n, np.int32).reshape(n, 3)

    def last(self) -> dict:
        ptr, n = J.jot_examined_list(self.h)
        out = {"active": J.device_to_host(ptr, n, np.int32)}
        out["token"] = J.device_to_host(J.jot_last_token(self.h), n, np.int32)
        for name in ("conf", "p1", "p2", "tau"):
            out[name] = J.device_to_host(getattr(J, "jot_last_" + name)(self.h), n, np.float32)
        out["flags"] = J.device_to_host(J.jot_last_flags(self.h), n, np.uint8)
        out["final"] = J.device_to_host(J.jot_last_final_token(self.h), n, np.int32)
        out["kl"] = J.device_to_host(J.jot_last_kl(self.h), n, np.float32)
        out["gap"] = J.device_to_host(J.jot_last_gap(self.h), n, np.float32)
        return out
