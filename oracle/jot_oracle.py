"""CPU oracle for the JoT token-finalization pass.

TEST INFRASTRUCTURE ONLY: a plain, slow, double-precision evaluation of the
paper's definitions, used to check the GPU library.  It imports nothing from
the GPU package and the GPU package imports nothing from here.

Followed passages of the paper (Section 4.1 and Algorithm 1):

* confidence metric, Eq. 2:      r^i = p1^i / (p2^i + eps), from softmax(l^i)
* spatial weight, Eq. 3:         w^i = sum_{j not masked, 1 <= |i-j| <= D} gamma^|i-j|
* softening factor, Eq. 4:       phi^i = min(1, w^i / w_max),  w_max = 2 sum_{d=1..D} gamma^d
* adaptive threshold, Eq. 5:     tau^i = tau_max - (tau_max - tau_min) phi^i
* early-exit decision, Eq. 6:    finalize i  iff  r^i >= tau^i, token = argmax_v pi^i_v
* Algorithm 1:                   the masked set M_n is fixed at the top of step n; every
                                 decision of the step uses that snapshot.
* "Implementation details":      eps = 1e-12; prompt tokens count as resolved context and
                                 the spatial sum runs over the whole canvas; with
                                 semi-autoregressive decoding only the current block is
                                 examined; finalization is uncapped.

Readings taken where the paper is silent:
the argmax takes the smallest index among equal logits; p2 is the second entry
of the sorted multiset (a duplicated maximum gives p2 = p1); positions outside
the canvas contribute nothing to Eq. 3; d = 0 is excluded (i itself is masked);
D = 0 means no spatial modulation (phi = 0); a row with NaN / +inf logits, or
only -inf logits, has no softmax and is never finalized.

Transfer schedule (Section 3.2 "Iterative Sampling"; Section 4.2 "Interaction with transfer
schedules" and "Implementation details"): each step the decoder's own schedule reveals a number
k of the masked positions, those with the highest confidence max_v pi_v; the early-exit mask is
OR-ed on top of it and is uncapped.  Here: per batch row b, among the positions examined this
step, U_b = the k_b positions with the largest p1 (equal p1: lower index first), and the step
finalizes J_b | U_b where J_b is the set passing Eq. 6.  k_b = min(valid_b, n_transfer[b] +
floor(transfer_frac * examined_b)): an absolute count per row (a precomputed per-step table, as
in block-wise decoders) plus a fraction of what is still examined (as in decoders that reveal
num_masked * (1 - s/t) per step).  Rows without a softmax are never selected.

Row-wide early commit (the global rule Section 2 attributes to Prophet: once the top-2
confidence gap exceeds a threshold, every remaining masked position is finalized at once; the
thresholds quoted for it in Section 6.1, 7.5 / 5 / 2.5, are on the logit scale).  Here: per batch
row, g_b = mean over the row's examined positions that have a softmax of the top-2 LOGIT gap
m1 - m2; if g_b >= global_gap (a threshold the caller passes for this step, so a staged
threshold is the caller's schedule) every such position of the row is finalized this step.

Stability rule (the per-token rule Section 2 attributes to KLASS: the KL divergence between the
distributions of consecutive steps identifies predictions that have stopped moving; Section 6.1
quotes its two thresholds, tau_KL and tau_conf).  Here: an examined position is stable at step n
if it was examined, with a softmax, at step n - 1 too, D(pi_n || pi_{n-1}) <= kl_threshold and
p1 >= kl_min_prob; stable positions are finalized, OR-ed with the other rules.  pi_{n-1} comes from
the previous step's logits, which the caller keeps and passes.

Besides the paper's ratio r, two other confidence signals computed from the same
(p1, p2) are selectable, because the workloads this is tested on quote
thresholds on the probability scale: p1 itself, and the gap p1 - p2.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "jot_oracle.c")
_LIB = os.path.join(_HERE, "_lib", "libjot_oracle.so")

F32, BF16 = 0, 1
CONF_RATIO, CONF_MAXPROB, CONF_PROBGAP = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile jot_oracle.c with gcc (-O2, no fast-math, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_LIB), exist_ok=True)
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.jot_oracle_row_stats.argtypes = [
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int]
        lib.jot_oracle_row_stats.restype = None
        lib.jot_oracle_softmax_row.argtypes = [
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int32, ctypes.c_void_p]
        lib.jot_oracle_softmax_row.restype = ctypes.c_int
        lib.jot_oracle_sample_row.argtypes = [
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int32, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p]
        lib.jot_oracle_sample_row.restype = ctypes.c_int32
        lib.jot_oracle_kl_row.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int32]
        lib.jot_oracle_kl_row.restype = ctypes.c_double
        lib.jot_oracle_kl_rows.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
                                           ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.jot_oracle_kl_rows.restype = None
        _lib = lib
    return _lib


def _check_rows(rows: np.ndarray, dtype: int) -> np.ndarray:
    want = np.float32 if dtype == F32 else np.uint16
    if rows.dtype != want:
        raise TypeError(f"rows must be {want} for dtype {dtype}, got {rows.dtype}")
    if rows.ndim != 2:
        raise ValueError("rows must be [n_rows, V]")
    return np.ascontiguousarray(rows)


def row_stats(rows: np.ndarray, dtype: int, threads: int = 1):
    """(a, m1, m2, S, status) per row; see jot_oracle.c.  bf16 rows are uint16 bit patterns."""
    rows = _check_rows(rows, dtype)
    n, V = rows.shape
    a = np.zeros(n, np.int32)
    m1 = np.zeros(n, np.float64)
    m2 = np.zeros(n, np.float64)
    S = np.zeros(n, np.float64)
    st = np.zeros(n, np.int32)
    if n:
        _load().jot_oracle_row_stats(
            rows.ctypes.data, dtype, n, V, V, a.ctypes.data, m1.ctypes.data, m2.ctypes.data,
            S.ctypes.data, st.ctypes.data, int(threads))
    return a, m1, m2, S, st


def softmax_row(row: np.ndarray, dtype: int) -> np.ndarray:
    """Whole probability vector of one row in double (tests only)."""
    row = _check_rows(row.reshape(1, -1), dtype)
    pi = np.zeros(row.shape[1], np.float64)
    _load().jot_oracle_softmax_row(row.ctypes.data, dtype, row.shape[1], pi.ctypes.data)
    return pi


def sample_row(row: np.ndarray, dtype: int, u: float):
    """Inverse-CDF sample of one row for the uniform number u: (token, cdf_below, cdf_above);
    token = first index whose cumulative probability exceeds u.  -1 if the row has no softmax."""
    row = _check_rows(row.reshape(1, -1), dtype)
    lo, hi = ctypes.c_double(), ctypes.c_double()
    v = _load().jot_oracle_sample_row(row.ctypes.data, dtype, row.shape[1], float(u),
                                      ctypes.byref(lo), ctypes.byref(hi))
    return int(v), lo.value, hi.value


def kl_row(row_now: np.ndarray, row_prev: np.ndarray, dtype: int) -> float:
    """D(pi_now || pi_prev) of two logit rows in double (NaN if either has no softmax)."""
    a = _check_rows(row_now.reshape(1, -1), dtype)
    b = _check_rows(row_prev.reshape(1, -1), dtype)
    return float(_load().jot_oracle_kl_row(a.ctypes.data, b.ctypes.data, dtype, a.shape[1]))


def kl_rows(rows_now: np.ndarray, rows_prev: np.ndarray, dtype: int, select: np.ndarray, threads: int = 1) -> np.ndarray:
    """kl_row for the rows where `select` is true (NaN elsewhere), rows spread over threads."""
    a = _check_rows(rows_now, dtype)
    b = _check_rows(rows_prev, dtype)
    assert a.shape == b.shape
    sel = np.ascontiguousarray(select, np.uint8)
    out = np.full(a.shape[0], np.nan)
    if a.shape[0]:
        _load().jot_oracle_kl_rows(a.ctypes.data, b.ctypes.data, dtype, a.shape[0], a.shape[1], sel.ctypes.data,
                                   out.ctypes.data, int(threads))
    return out


@dataclass
class OracleParams:
    B: int
    L: int                      # canvas length, prompt included
    V: int
    dtype: int = F32
    conf_mode: int = CONF_RATIO
    tau_max: float = 90.0
    tau_min: float = 1.0
    gamma: float = 0.5
    D: int = 8
    eps: float = 1e-12
    gen_start: int = 0          # first generation position; blocks are counted from here
    block_size: int = 0         # 0: every masked position is examined; >0: current block only


def w_max(gamma: float, D: int) -> float:
    """Eq. 4: the largest value Eq. 3 can take, 2 * sum_{d=1..D} gamma^d."""
    return 2.0 * sum(gamma ** d for d in range(1, D + 1))


def spatial_weight(resolved: np.ndarray, gamma: float, D: int) -> np.ndarray:
    """Eq. 3 for every position of every row.  resolved: [B, L] bool (True = not masked).

    Zero padding outside the canvas; the d = 0 term is not part of the sum.
    """
    B, L = resolved.shape
    res = resolved.astype(np.float64)
    w = np.zeros((B, L), np.float64)
    for d in range(1, D + 1):
        g = gamma ** d
        if d < L:
            w[:, d:] += g * res[:, :-d]      # neighbour i - d
            w[:, :-d] += g * res[:, d:]      # neighbour i + d
    return w


def threshold(resolved: np.ndarray, p: OracleParams):
    """Eq. 4 and Eq. 5: (tau^i, phi^i) for every position, from the step-start mask."""
    if p.D == 0:
        phi = np.zeros(resolved.shape, np.float64)
    else:
        phi = np.minimum(1.0, spatial_weight(resolved, p.gamma, p.D) / w_max(p.gamma, p.D))
    return p.tau_max - (p.tau_max - p.tau_min) * phi, phi


def confidence(p1: np.ndarray, p2: np.ndarray, mode: int, eps: float) -> np.ndarray:
    if mode == CONF_RATIO:
        return p1 / (p2 + eps)                # Eq. 2
    if mode == CONF_MAXPROB:
        return p1
    if mode == CONF_PROBGAP:
        return p1 - p2
    raise ValueError("unknown confidence mode")


def eligible(masked: np.ndarray, p: OracleParams) -> np.ndarray:
    """Positions examined this step.  Full mode: every masked position.  Block mode: the
    masked positions of each row's current block, i.e. the block (counted in units of
    block_size from gen_start) that holds the row's lowest masked position."""
    if p.block_size <= 0:
        return masked.copy()
    B, L = masked.shape
    out = np.zeros_like(masked)
    idx = np.arange(L)
    blk = np.floor_divide(idx - p.gen_start, p.block_size)
    for b in range(B):
        where = np.flatnonzero(masked[b])
        if where.size:
            out[b] = masked[b] & (blk == blk[where[0]])
    return out


@dataclass
class StepRecord:
    """Everything one step produced, for element-wise comparison."""
    step: int
    active: np.ndarray          # [A] flattened positions b*L+i examined, ascending
    token: np.ndarray           # [A] argmax token
    p1: np.ndarray              # [A]
    p2: np.ndarray              # [A]
    conf: np.ndarray            # [A]
    tau: np.ndarray             # [A] tau^i
    phi: np.ndarray             # [A]
    commit: np.ndarray          # [A] bool: finalized this step (early exit OR schedule)
    status: np.ndarray          # [A] 1 = row without a softmax (never committed)
    exit: np.ndarray = None     # [A] bool: passed Eq. 6
    sched: np.ndarray = None    # [A] bool: picked by the transfer schedule
    k_row: np.ndarray = None    # [B] number of positions the schedule picked per batch row
    final_token: np.ndarray = None  # [A] token written if finalized: argmax, or the sample
    stable: np.ndarray = None       # [A] bool: finalized by the KL stability rule
    kl: np.ndarray = None           # [A] D(pi_n || pi_{n-1}); nan where there is no previous distribution
    rowwide: np.ndarray = None      # [A] bool: finalized by the row-wide gap rule
    gap_row: np.ndarray = None      # [B] mean top-2 logit gap of the row's examined positions (nan: none)
    cdf_margin: np.ndarray = None   # [A] with sampling: distance of u from the nearer edge of the
                                    #     chosen token's CDF interval (inf where nothing is sampled)
    gap: np.ndarray = None          # [A] top-2 logit gap l_(1) - l_(2) (+inf: one finite logit; nan: no softmax)


@dataclass
class OracleState:
    params: OracleParams
    tokens: np.ndarray          # [B, L] int32
    masked: np.ndarray          # [B, L] bool
    step_index: int = 0
    commit_log: list = field(default_factory=list)   # (step, b*L+i, token)
    anomalies: int = 0
    threads: int = 1
    last_ok_step: np.ndarray = None   # [B, L] last step at which the position was examined with a softmax

    @classmethod
    def init(cls, params: OracleParams, tokens: np.ndarray, masked: np.ndarray, threads: int = 1):
        p = params
        if tokens.shape != (p.B, p.L) or masked.shape != (p.B, p.L):
            raise ValueError("tokens/masked must be [B, L]")
        if p.V < 2 or p.D < 0 or not (0.0 < p.gamma <= 1.0) or p.tau_min > p.tau_max:
            raise ValueError("invalid parameters")
        return cls(p, tokens.astype(np.int32).copy(), masked.astype(bool).copy(), threads=threads,
                   last_ok_step=np.full((p.B, p.L), -1, np.int64))

    def active_list(self) -> np.ndarray:
        """Ascending flattened indices b*L+i of the positions the next step examines."""
        return np.flatnonzero(eligible(self.masked, self.params).reshape(-1)).astype(np.int64)

    def active_count(self) -> int:
        return int(self.active_list().size)

    def evaluate(self, rows: np.ndarray, n_transfer=None, transfer_frac: float = 0.0,
                 sample_u=None, global_gap=None, prev_rows=None, kl_threshold=None,
                 kl_min_prob: float = 0.0) -> StepRecord:
        """Decisions of the next step for the given logit rows (rows[k] belongs to
        active_list()[k]) WITHOUT changing the state.  n_transfer ([B] ints) and transfer_frac
        describe the transfer schedule of this step; by default it reveals nothing.
        sample_u: optional [B, L] uniform numbers in [0, 1); when given, a finalized position
        takes a token sampled from pi (inverse CDF at sample_u[b, i]) instead of the argmax.
        global_gap: optional threshold of the row-wide early-commit rule for this step.
        prev_rows / kl_threshold / kl_min_prob: the stability rule; prev_rows[k] is the previous
        step's logit row of active_list()[k]."""
        p = self.params
        act = self.active_list()
        if rows.shape[0] != act.size:
            raise ValueError("one logit row per active position expected")
        M = self.masked.copy()                                  # M_n, fixed for the step
        a, m1, m2, S, st = row_stats(rows, p.dtype, self.threads)
        ok = st == 0
        with np.errstate(all="ignore"):
            p1 = np.where(ok, 1.0 / S, np.nan)
            p2 = np.where(ok, np.exp(m2 - m1) / S, np.nan)
            conf = confidence(p1, p2, p.conf_mode, p.eps)
        tau_all, phi_all = threshold(~M, p)
        tau = tau_all.reshape(-1)[act]
        phi = phi_all.reshape(-1)[act]
        with np.errstate(invalid="ignore"):
            exit_ = ok & (conf >= tau)                          # Eq. 6
        sched, k_row = self._schedule(act, p1, ok, n_transfer, transfer_frac)
        rowwide, gap_row = self._rowwide(act, m1, m2, ok, global_gap)
        stable, kl = self._stable(act, rows, prev_rows, p1, ok, kl_threshold, kl_min_prob)
        commit = exit_ | sched | rowwide | stable               # logical OR, uncapped
        final = a.copy()
        margin = np.full(act.size, np.inf)
        if sample_u is not None:
            uflat = np.asarray(sample_u, np.float64).reshape(-1)
            for k in np.flatnonzero(commit):
                u = uflat[act[k]]
                v, lo, hi = sample_row(rows[k], p.dtype, u)
                final[k] = v
                margin[k] = min(u - lo, hi - u)
        with np.errstate(invalid="ignore"):
            gap = np.where(ok, m1 - m2, np.nan)
        return StepRecord(self.step_index + 1, act, a, p1, p2, conf, tau, phi, commit, st,
                          exit_, sched, k_row, final, stable, kl, rowwide, gap_row, margin, gap)

    def _stable(self, act, rows, prev_rows, p1, ok, kl_threshold, kl_min_prob):
        """KL stability rule; needs the position to have been examined, with a softmax, in the
        step before."""
        stable = np.zeros(act.size, bool)
        kl = np.full(act.size, np.nan)
        if kl_threshold is None:
            return stable, kl
        had_prev = self.last_ok_step.reshape(-1)[act] == self.step_index
        kl = kl_rows(rows, prev_rows, self.params.dtype, ok & had_prev, self.threads)
        with np.errstate(invalid="ignore"):
            stable = ok & had_prev & (kl <= kl_threshold) & (p1 >= kl_min_prob)
        return stable, kl

    def _rowwide(self, act, m1, m2, ok, global_gap):
        """Row-wide early commit: mean top-2 logit gap of a row's examined positions >= threshold
        finalizes all of them."""
        p = self.params
        rowwide = np.zeros(act.size, bool)
        gap_row = np.full(p.B, np.nan)
        if global_gap is None:
            return rowwide, gap_row
        row_of = act // p.L
        for b in range(p.B):
            mine = np.flatnonzero((row_of == b) & ok)
            if mine.size:
                gap_row[b] = float(np.mean(m1[mine] - m2[mine]))
                if gap_row[b] >= global_gap:
                    rowwide[mine] = True
        return rowwide, gap_row

    def _schedule(self, act, p1, ok, n_transfer, transfer_frac):
        """Per batch row: the k positions with the largest p1 among the examined ones."""
        p = self.params
        sched = np.zeros(act.size, bool)
        k_row = np.zeros(p.B, np.int64)
        if n_transfer is None and transfer_frac == 0.0:
            return sched, k_row
        n_transfer = np.zeros(p.B, np.int64) if n_transfer is None else np.asarray(n_transfer, np.int64)
        row_of = act // p.L
        for b in range(p.B):
            mine = np.flatnonzero(row_of == b)                  # ascending position
            valid = mine[ok[mine]]
            k = int(n_transfer[b]) + int(np.floor(float(transfer_frac) * mine.size))
            k = max(0, min(k, valid.size))
            k_row[b] = k
            if k:
                order = sorted(valid.tolist(), key=lambda j: (-p1[j], j))   # largest p1, then lowest index
                sched[order[:k]] = True
        return sched, k_row

    def apply(self, rec: StepRecord) -> None:
        """Commit the step: all finalizations take effect together."""
        p = self.params
        self.step_index = rec.step
        flat_tok = self.tokens.reshape(-1)
        flat_msk = self.masked.reshape(-1)
        for k in np.flatnonzero(rec.commit):                    # ascending b*L+i
            pos = int(rec.active[k])
            assert flat_msk[pos]
            tok = rec.token[k] if rec.final_token is None else rec.final_token[k]
            flat_tok[pos] = tok
            flat_msk[pos] = False
            self.commit_log.append((rec.step, pos, int(tok)))
        self.anomalies += int(rec.status.sum())
        self.last_ok_step.reshape(-1)[rec.active[rec.status == 0]] = rec.step

    def step(self, rows: np.ndarray, n_transfer=None, transfer_frac: float = 0.0, sample_u=None,
             global_gap=None, prev_rows=None, kl_threshold=None, kl_min_prob: float = 0.0) -> StepRecord:
        rec = self.evaluate(rows, n_transfer, transfer_frac, sample_u, global_gap, prev_rows, kl_threshold,
                            kl_min_prob)
        self.apply(rec)
        return rec

    def step_full(self, logits: np.ndarray, n_transfer=None, transfer_frac: float = 0.0,
                  sample_u=None, global_gap=None) -> StepRecord:
        """Convenience for small cases: logits is the whole [B, L, V] array."""
        p = self.params
        act = self.active_list()
        rows = logits.reshape(p.B * p.L, p.V)[act]
        return self.step(rows, n_transfer, transfer_frac, sample_u, global_gap)
