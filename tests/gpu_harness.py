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


from paper_2602_11133_amd.session import JotSession as GpuJot  # noqa: E402,F401


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
