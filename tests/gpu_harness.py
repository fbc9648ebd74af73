"""GPU side of the parity tests: drives the C-ABI library through the Python binding and
reads its results back.  torch supplies device memory and the stream, nothing else."""
from __future__ import annotations

import numpy as np
import torch

import paper_2602_11133_amd as J
from gen.configs import F32


def params_of(cfg) -> J.JotParams:
    return J.JotParams(B=cfg.B, L=cfg.L, V=cfg.V, dtype=cfg.dtype, conf_mode=cfg.conf_mode,
                       tau_max=cfg.tau_max, tau_min=cfg.tau_min, gamma=cfg.gamma, D=cfg.D,
                       eps=cfg.eps, gen_start=cfg.gen_start, block_size=cfg.block_size)


class GpuJot:
    """One decoding state on the GPU."""

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


def gather_compact(logits: torch.Tensor, active_dev_ptr: int, n: int, pad_elems: int = 0) -> torch.Tensor:
    """[n, V + pad] tensor holding the rows of the examined positions in list order -- what a decoder
    that applies its output projection to the examined positions only would produce (test plumbing:
    the full tensor is gathered by the list the library exposes).  Padding is NaN."""
    B, L, V = logits.shape
    if n:
        idx = torch.from_numpy(J.device_to_host(active_dev_ptr, n, np.int32).astype(np.int64)).to(logits.device)
    else:
        idx = torch.zeros(0, dtype=torch.int64, device=logits.device)
    out = torch.full((max(n, 1), V + pad_elems), float("nan"), dtype=logits.dtype, device=logits.device)
    if n:
        out[:n, :V] = logits.view(B * L, V).index_select(0, idx)
    return out


def upload_rows(logits: torch.Tensor, positions: np.ndarray, rows: np.ndarray, dtype: int) -> None:
    """Write host rows ([n, V] float32 or bf16 bit patterns) into logits[b, i, :] for the given
    flattened positions."""
    B, L, V = logits.shape
    flat = logits.view(B * L, V)
    idx = torch.from_numpy(np.ascontiguousarray(positions, np.int64)).to(logits.device)
    if dtype == F32:
        src = torch.from_numpy(np.ascontiguousarray(rows, np.float32)).to(logits.device)
    else:
        src = torch.from_numpy(np.ascontiguousarray(rows, np.uint16).view(np.int16)).to(logits.device).view(torch.bfloat16)
    flat.index_copy_(0, idx, src)


def rel_err(got: np.ndarray, want: np.ndarray) -> np.ndarray:
    with np.errstate(divide="ignore", invalid="ignore"):
        e = np.abs(got.astype(np.float64) - want) / np.abs(want)
    e[(got == want)] = 0.0
    return e


KL_TOL = 1e-5         # absolute, on divergences of order 1 and below; relative above


def compare_step(gpu_last: dict, rec, act_full: np.ndarray, tol: float, select=None):
    """Element-by-element comparison of one step.  `select` optionally restricts the GPU's
    examined list to the entries the oracle followed (boolean mask over the GPU list)."""
    g = {k: (v[select] if select is not None else v) for k, v in gpu_last.items()}
    np.testing.assert_array_equal(g["active"], act_full.astype(np.int32))           # bit exact
    np.testing.assert_array_equal(g["token"], rec.token)                             # bit exact
    ok = rec.status == 0
    assert np.all(np.isnan(g["conf"][~ok]))
    assert rel_err(g["p1"][ok], rec.p1[ok]).max(initial=0) <= tol
    # relative to the confidence itself, except that the gap p1 - p2 (which cancels when the two
    # are close) is measured on the scale of p1, the larger of the numbers it is formed from
    conf_err = np.abs(g["conf"][ok].astype(np.float64) - rec.conf[ok]) / np.maximum(np.abs(rec.conf[ok]), rec.p1[ok])
    assert conf_err.max(initial=0) <= tol
    # tau is compared on the scale of the thresholds (tau_min may be 0, where a relative bound is void)
    tau_scale = max(1.0, float(np.abs(rec.tau).max(initial=0)))
    assert np.abs(g["tau"].astype(np.float64) - rec.tau).max(initial=0) <= 1e-5 * tau_scale
    big = ok & (rec.p2 > 1e-30)           # p2 below that is subnormal in binary32
    assert rel_err(g["p2"][big], rec.p2[big]).max(initial=0) <= max(tol, 2e-5)
    with np.errstate(invalid="ignore"):
        exit_gpu = ok & (g["conf"] >= g["tau"])
    want_exit = rec.exit if rec.exit is not None else rec.commit
    np.testing.assert_array_equal(exit_gpu, want_exit)
    np.testing.assert_array_equal((g["flags"] & 1).astype(bool), want_exit)
    want_sched = rec.sched if rec.sched is not None else np.zeros_like(rec.commit)
    np.testing.assert_array_equal((g["flags"] & 2).astype(bool), want_sched)
    want_rowwide = rec.rowwide if rec.rowwide is not None else np.zeros_like(rec.commit)
    np.testing.assert_array_equal((g["flags"] & 4).astype(bool), want_rowwide)
    if rec.gap is not None:                # both operands are input values: one binary32 rounding
        fin = ok & np.isfinite(rec.gap)
        assert np.all(np.abs(g["gap"][fin].astype(np.float64) - rec.gap[fin]) <= 1e-6 * np.maximum(1.0, rec.gap[fin]))
        assert np.all(g["gap"][ok & np.isposinf(rec.gap)] == np.inf)
    want_stable = rec.stable if rec.stable is not None else np.zeros_like(rec.commit)
    np.testing.assert_array_equal((g["flags"] & 8).astype(bool), want_stable)
    if rec.kl is not None and np.isfinite(rec.kl).any():
        fin = np.isfinite(rec.kl)
        assert not np.isfinite(g["kl"][~fin]).any()              # no history / no softmax / infinite
        err = np.abs(g["kl"][fin].astype(np.float64) - rec.kl[fin])
        assert (err <= KL_TOL * np.maximum(1.0, np.abs(rec.kl[fin]))).all(), float(err.max())
    want_final = rec.final_token if rec.final_token is not None else rec.token
    np.testing.assert_array_equal(g["final"][rec.commit], want_final[rec.commit])   # bit exact
