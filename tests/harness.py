"""Lock-step driver shared by the CPU and GPU tests: runs the oracle over a synthetic
trajectory, keeps every confidence clear of its threshold by adjusting the *input*
(never the oracle), and hands each step's inputs and expected outputs to the caller.
"""
from __future__ import annotations

import numpy as np

from gen.configs import JotConfig
from gen.host import HostGenerator
from gen.trajectory import Trajectory
from oracle import jot_oracle as O

GUARD = 1e-4          # |conf - tau| >= GUARD * max(1, |tau|) for every examined position
GUARD_U = 1e-6        # sampling: the uniform number stays this far (in probability) from both
                      # edges of the chosen token's CDF interval
GUARD_KL = 2e-5       # stability rule: |KL - tau_KL| >= GUARD_KL * max(1, tau_KL), |p1 - tau_conf| >= GUARD
MAX_BUMPS = 200


def oracle_params(cfg: JotConfig) -> O.OracleParams:
    return O.OracleParams(B=cfg.B, L=cfg.L, V=cfg.V, dtype=cfg.dtype, conf_mode=cfg.conf_mode,
                          tau_max=cfg.tau_max, tau_min=cfg.tau_min, gamma=cfg.gamma, D=cfg.D,
                          eps=cfg.eps, gen_start=cfg.gen_start, block_size=cfg.block_size)


def too_close(rec: O.StepRecord, L: int = 0, kl=None) -> np.ndarray:
    """Examined entries whose decision is not well posed: a confidence within the guard band of
    its threshold, or -- with a transfer schedule -- the last position the schedule takes in a
    row when the best position it leaves behind has nearly the same p1."""
    ok = rec.status == 0
    with np.errstate(invalid="ignore"):
        near = ok & (np.abs(rec.conf - rec.tau) < GUARD * np.maximum(1.0, np.abs(rec.tau)))
    if kl is not None:
        tau_kl, tau_conf = kl
        with np.errstate(invalid="ignore"):
            has = ok & np.isfinite(rec.kl)
            near |= has & (np.abs(rec.kl - tau_kl) < GUARD_KL * max(1.0, tau_kl))
            if tau_conf > 0.0:
                near |= has & (rec.kl <= tau_kl) & (np.abs(rec.p1 - tau_conf) < GUARD)
    if rec.sched is not None and rec.sched.any():
        row_of = rec.active // L
        for b in np.unique(row_of[rec.sched]):
            mine = np.flatnonzero((row_of == b) & ok)
            taken, left = mine[rec.sched[mine]], mine[~rec.sched[mine]]
            if taken.size and left.size:
                lo = taken[np.argmin(rec.p1[taken])]
                if rec.p1[lo] - rec.p1[left].max() < GUARD * rec.p1[lo]:
                    near[lo] = True
    return np.flatnonzero(near)


class LockstepRun:
    def __init__(self, cfg: JotConfig, threads: int = 1, batch_rows=None, share=None):
        """batch_rows: optional list of batch rows b to follow (rows are independent decodes);
        the oracle then runs on that sub-batch only, positions are reported in the full
        canvas numbering.  share: another LockstepRun of the same configuration whose trajectory
        (and hence input adjustments) and row generators this one uses too -- for following a
        large batch as several sub-batches, one after the other, within each step."""
        self.cfg = cfg
        self.traj = share.traj if share else Trajectory(cfg)
        self.gen = share.gen if share else HostGenerator(cfg, self.traj.target, self.traj.rival, threads)
        tokens, masked = self.traj.initial_canvas()
        self.batch_rows = list(range(cfg.B)) if batch_rows is None else list(batch_rows)
        sub = cfg.replace(B=len(self.batch_rows))
        self.state = O.OracleState.init(oracle_params(sub), tokens[self.batch_rows],
                                        masked[self.batch_rows], threads=threads)
        self.n_bumps = 0
        self.gen_prev = share.gen_prev if share else HostGenerator(cfg, self.traj.target, self.traj.rival, threads)
        self.prev_tables = None          # final planted tables of the step before

    def to_full(self, sub_pos: np.ndarray) -> np.ndarray:
        L = self.cfg.L
        rows = np.asarray(self.batch_rows, np.int64)
        return rows[sub_pos // L] * L + sub_pos % L

    def active_full(self) -> np.ndarray:
        return self.to_full(self.state.active_list())

    def draw_uniforms(self, step: int) -> np.ndarray:
        """[B, L] float32 uniform numbers in [0, 1) for sampling-based finalization at this step."""
        rng = np.random.default_rng([self.cfg.seed, 0x756E6966, step])
        return rng.random((self.cfg.B, self.cfg.L), dtype=np.float32)

    def next_step(self, n_transfer=None, transfer_frac: float = 0.0, sample_u=None, global_gap=None, kl=None):
        """Advance the oracle one step.  Returns (rec, T, R, rows) where rec.active is in
        sub-batch numbering, T/R are the final planted tables of this step (full canvas) and
        rows are the logit rows the oracle saw (a view valid until the next call).
        n_transfer ([B] of the FULL batch) / transfer_frac: the step's transfer schedule.
        sample_u ([B, L] float32 of the FULL batch, modified in place where a number has to be
        redrawn to stay clear of a CDF edge): sampling-based finalization.
        kl = (kl_threshold, kl_min_prob): the KL stability rule against the previous step's rows."""
        if n_transfer is not None:
            n_transfer = np.asarray(n_transfer)[self.batch_rows]
        st, tr = self.state, self.traj
        n = st.step_index + 1
        act_full = self.active_full()
        T, R = tr.planted(n)
        rows = self.gen.rows(n, act_full, T, R)
        u_sub = None if sample_u is None else sample_u[self.batch_rows]
        redraw = np.random.default_rng([self.cfg.seed, 0x72656472, n])
        kl_kw = {}
        if kl is not None:
            if self.prev_tables is None:
                prev_rows = rows                  # first step: no position has a history, never read
            else:
                prev_rows = self.gen_prev.rows(n - 1, act_full, *self.prev_tables)
            kl_kw = dict(prev_rows=prev_rows, kl_threshold=kl[0], kl_min_prob=kl[1])
        rec = st.evaluate(rows, n_transfer, transfer_frac, u_sub, global_gap, **kl_kw)
        for _ in range(MAX_BUMPS):
            bad = too_close(rec, self.cfg.L, kl)
            amount = {}                           # entry -> how much to raise its target logit (default 0.25)
            if global_gap is not None:            # a row's mean gap too close to the row-wide threshold:
                scale = max(1.0, abs(global_gap))
                near = np.flatnonzero(np.abs(rec.gap_row - global_gap) < GUARD * scale)
                row_of = rec.active // self.cfg.L
                for b in near:                    # move the mean by raising one target logit of that row
                    mine = np.flatnonzero((row_of == b) & (rec.status == 0))
                    amount[int(mine[0])] = 4.0 * GUARD * scale * mine.size
                    bad = np.union1d(bad, mine[:1])
            if sample_u is not None:
                edge = np.flatnonzero(rec.commit & (rec.cdf_margin < GUARD_U))
                if edge.size:                   # a new uniform number for that position (an input)
                    for k in edge:
                        bb, ii = divmod(int(act_full[k]), self.cfg.L)
                        sample_u[bb, ii] = redraw.random(dtype=np.float32)
                    u_sub = sample_u[self.batch_rows]
                    if bad.size == 0:
                        rec = st.evaluate(rows, n_transfer, transfer_frac, u_sub, global_gap, **kl_kw)
                        continue
            if bad.size == 0:
                break
            for k in bad:
                tr.bump(n, int(act_full[k]), amount.get(int(k), 0.25))
            self.n_bumps += int(bad.size)
            T, R = tr.planted(n)
            fixer = HostGenerator(self.cfg, tr.target, tr.rival, 1)
            rows[bad] = fixer.rows(n, act_full[bad], T, R)
            rec = st.evaluate(rows, n_transfer, transfer_frac, u_sub, global_gap, **kl_kw)
        else:
            raise RuntimeError("could not clear the guard band")
        st.apply(rec)
        self.prev_tables = (T, R)
        return rec, T, R, rows
