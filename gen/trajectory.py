"""Planted-token trajectories: which token each generation position converges to, and how its
logit rises over the denoising steps.  Everything here is computed on the host in double and
handed to the generators as float32 tables; nothing here looks at a softmax or a threshold.
"""
from __future__ import annotations

import numpy as np
from scipy import special

from .configs import JotConfig


class Trajectory:
    def __init__(self, cfg: JotConfig):
        self.cfg = cfg
        B, L, V, gs = cfg.B, cfg.L, cfg.V, cfg.gen_start
        rng = np.random.default_rng([cfg.seed, 0x7472616A])
        n = B * L
        gen = np.zeros((B, L), bool)
        gen[:, gs:] = True
        self.gen = gen.reshape(-1)
        self.prompt_tokens = rng.integers(0, V, (B, L)).astype(np.int32)
        self.target = np.where(self.gen, rng.integers(0, V, n), -1).astype(np.int32)
        self.rival = np.full(n, -1, np.int32)
        self.boost = rng.uniform(0.0, 8.0, n)                    # 'single' trajectories
        self.conv = self._convergence_steps(rng).reshape(-1)     # step around which the target rises
        self.release = np.zeros(n, np.int64)
        if cfg.rival_frac > 0:
            has = self.gen & (rng.random(n) < cfg.rival_frac)
            other = (self.target + 1 + rng.integers(0, V - 1, n)) % V      # any token but the target
            self.rival = np.where(has, other, -1).astype(np.int32)
            lo = max(1, (3 * cfg.steps) // 4)
            self.release = rng.integers(lo, cfg.steps + 1, n)
        self.base = cfg.planted_base()
        self.overrides: dict[tuple[int, int], float] = {}

    def _convergence_steps(self, rng) -> np.ndarray:
        cfg = self.cfg
        B, L, gs, T = cfg.B, cfg.L, cfg.gen_start, cfg.steps
        if cfg.conv == "uniform":
            return rng.integers(1, T + 1, (B, L))
        if cfg.conv == "mixture":                                # 70 % early, 30 % late
            split = max(1, T // 4)
            early = rng.integers(1, split + 1, (B, L))
            late = rng.integers(split, T + 1, (B, L))
            return np.where(rng.random((B, L)) < 0.7, early, late)
        if cfg.conv == "block_ar":
            # block k converges inside the step window (k*w, (k+1)*w], w = steps / blocks; inside a
            # block neighbouring positions are correlated: z_j = 0.8 z_{j-1} + 0.6 e_j (rho = 0.8)
            bs = cfg.block_size
            nblk = -(-(L - gs) // bs)
            w = max(1, T // nblk)
            c = np.ones((B, L), np.int64)
            e = rng.standard_normal((B, L))
            for b in range(B):
                z = 0.0
                for i in range(gs, L):
                    j = (i - gs) % bs
                    z = e[b, i] if j == 0 else 0.8 * z + 0.6 * e[b, i]
                    k = (i - gs) // bs
                    c[b, i] = k * w + int(np.ceil(w * special.ndtr(z)))
            return np.clip(c, 1, T)
        raise ValueError(cfg.conv)

    # ------------------------------------------------------------------ inputs
    def initial_canvas(self):
        """tokens [B, L] int32 (prompt tokens; masked slots hold an arbitrary id) and masked [B, L]."""
        cfg = self.cfg
        masked = self.gen.reshape(cfg.B, cfg.L).copy()
        tokens = np.where(masked, cfg.V - 1, self.prompt_tokens).astype(np.int32)
        return tokens, masked

    def planted(self, step: int):
        """float32 tables (T, R) over the flattened canvas for this step: the amounts added to the
        noise at the target and at the rival token."""
        cfg = self.cfg
        if cfg.traj == "single":
            t = self.base - 4.0 + self.boost
        else:
            x = (step - self.conv) / cfg.width
            t = self.base + cfg.amp * (2.0 * special.expit(x) - 1.0)
        r = t - 0.05 - np.maximum(0, step - self.release)       # ties until release, then decays 1/step
        t = np.where(self.gen, t, 0.0)
        for (s, pos), dv in self.overrides.items():
            if s == step:
                t[pos] += dv
        r = np.where(self.rival >= 0, r, 0.0)
        return t.astype(np.float32), r.astype(np.float32)

    def bump(self, step: int, pos: int, delta: float = 0.25) -> None:
        """Raise the target logit of one position at one step (used to keep a confidence away
        from its threshold); part of the input from then on."""
        self.overrides[(step, pos)] = self.overrides.get((step, pos), 0.0) + delta
