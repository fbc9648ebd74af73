#!/usr/bin/env python3
"""Writes tests/golden/config1_expected.json: what the CPU oracle computes for the single-step
workload (B=1, 32 prompt + 64 masked positions, V=32000, fp32) under the three confidence
signals.  Calls only the generator and the oracle; never the GPU library.  Re-run it only when
the input recipe or the oracle is changed on purpose, and say why in the commit message."""
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

from gen.configs import CONF_MAXPROB, CONF_PROBGAP, CONF_RATIO, CONFIGS  # noqa: E402
from harness import LockstepRun  # noqa: E402


def main():
    out = {"_about": "oracle results for workload 1, step 1; written by write_config1_expected.py"}
    for name, mode, tau_max, tau_min in (("maxprob", CONF_MAXPROB, 0.9, 0.0), ("ratio", CONF_RATIO, 90.0, 1.0),
                                         ("probgap", CONF_PROBGAP, 0.9, 0.0)):
        cfg = CONFIGS[1].replace(conf_mode=mode, tau_max=tau_max, tau_min=tau_min)
        run = LockstepRun(cfg, threads=1)
        rec, T, R, rows = run.next_step()
        out[name] = {
            "active": rec.active.tolist(), "token": rec.token.tolist(),
            "p1": [float.hex(float(x)) for x in rec.p1], "conf": [float.hex(float(x)) for x in rec.conf],
            "tau": [float.hex(float(x)) for x in rec.tau], "commit": rec.commit.astype(int).tolist(),
            "bumps": run.n_bumps,
        }
    with open(os.path.join(HERE, "config1_expected.json"), "w") as f:
        json.dump(out, f, indent=0)


if __name__ == "__main__":
    main()
