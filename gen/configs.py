"""The five synthetic workloads, as data.

Shapes follow 7B/8B masked-diffusion denoisers (vocabulary 126 464 and 152 064, generation
lengths 256-1024, 256/512 steps, semi-autoregressive block 32).  They stand in for the
benchmark runs the paper measures on; no benchmark item is reproduced anywhere.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass

F32, BF16 = 0, 1
CONF_RATIO, CONF_MAXPROB, CONF_PROBGAP = 0, 1, 2


@dataclass(frozen=True)
class JotConfig:
    name: str
    B: int
    L: int                  # canvas length, prompt included
    gen_start: int          # prompt length
    V: int
    dtype: int
    steps: int              # configured number of denoising steps
    block_size: int = 0
    noise: str = "normal"   # 'normal' | 'student3'
    noise_scale: float = 1.0
    conf_mode: int = CONF_MAXPROB
    tau_max: float = 0.9
    tau_min: float = 0.0
    gamma: float = 0.5
    D: int = 8
    eps: float = 1e-12
    seed: int = 0x6A6F7431
    # trajectory of the planted target logit
    traj: str = "sigmoid"   # 'single' | 'sigmoid'
    conv: str = "uniform"   # 'uniform' | 'mixture' | 'block_ar'
    amp: float = 8.0        # sigmoid amplitude A
    width: float = 2.0      # sigmoid width s (steps)
    rival_frac: float = 0.0 # share of positions with a near-tying second planted token
    base: str = "partition" # 'partition' | 'noise_max' | 'literal': level the planted logit is measured from

    def replace(self, **kw) -> "JotConfig":
        return dataclasses.replace(self, **kw)

    @property
    def n_gen(self) -> int:
        return self.L - self.gen_start

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2

    def planted_base(self) -> float:
        """'partition': ln(V) + sigma^2/2, the log partition function of the Gaussian noise, so a
        planted logit base + x has probability about sigmoid(x).  'noise_max': the 1 - 1/V
        quantile of the noise, i.e. the typical largest noise logit of a row (used with the
        ratio signal, where the target must clear the runner-up by ln(tau)).  'literal': 4, so that
        the single-step trajectory base - 4 + U[0, 8] is the bare offset U[0, 8] on top of the
        noise (degenerate on purpose: nothing reaches a probability threshold, everything clears
        a ratio threshold below 1)."""
        if self.base == "literal":
            return 4.0
        if self.base == "partition":
            return math.log(self.V) + 0.5 * self.noise_scale ** 2
        from scipy import stats
        q = stats.norm.ppf if self.noise == "normal" else (lambda u: stats.t.ppf(u, 3))
        return float(self.noise_scale * q(1.0 - 1.0 / self.V))


CONFIGS = {
    # single step, 32 prompt + 64 masked
    1: JotConfig("cfg1_single_step", B=1, L=96, gen_start=32, V=32000, dtype=F32, steps=1,
                 traj="single", seed=0x6A6F7431),
    # Dream-shaped full decode loop
    2: JotConfig("cfg2_full_loop", B=1, L=320, gen_start=64, V=126464, dtype=BF16, steps=256,
                 conv="uniform", seed=0x6A6F7432),
    # batch of 8, early/late mixture; tau_max swept over {0.7, 0.8, 0.9}
    3: JotConfig("cfg3_batch_sweep", B=8, L=384, gen_start=128, V=152064, dtype=BF16, steps=64,
                 conv="mixture", seed=0x6A6F7433),
    # LLaDA-shaped block-wise decode
    4: JotConfig("cfg4_blockwise", B=32, L=640, gen_start=128, V=126464, dtype=BF16, steps=512,
                 block_size=32, conv="block_ar", seed=0x6A6F7434),
    # largest: fp32, heavy-tailed noise, near-tying rivals, the paper's ratio signal and defaults
    5: JotConfig("cfg5_large_fp32", B=64, L=1280, gen_start=256, V=152064, dtype=F32, steps=256,
                 noise="student3", noise_scale=0.02, conf_mode=CONF_RATIO, tau_max=90.0, tau_min=1.0,
                 conv="uniform", rival_frac=0.05, base="noise_max", seed=0x6A6F7435),
}
