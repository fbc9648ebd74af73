"""The oracle on the synthetic workloads (CPU only): the full-size single-step configuration,
and size-reduced versions of the four decode loops, checked through properties that hold at
any size."""
import numpy as np
import pytest

from gen.configs import CONF_MAXPROB, CONF_PROBGAP, CONF_RATIO, CONFIGS
from harness import GUARD, LockstepRun
from oracle import jot_oracle as O


@pytest.mark.parametrize("mode,tau_max,tau_min", [(CONF_MAXPROB, 0.9, 0.0), (CONF_RATIO, 90.0, 1.0),
                                                   (CONF_PROBGAP, 0.9, 0.0)])
def test_config1_single_step(mode, tau_max, tau_min):
    cfg = CONFIGS[1].replace(conf_mode=mode, tau_max=tau_max, tau_min=tau_min)
    run = LockstepRun(cfg, threads=4)
    rec, T, R, rows = run.next_step()
    assert rec.active.size == 64 and rec.status.sum() == 0
    assert np.all(np.abs(rec.conf - rec.tau) >= GUARD * np.maximum(1, rec.tau))
    # planted offsets span p_target from about 0.02 to 0.98: a healthy share passes, not all
    # (the ratio signal only needs the target ln(90) above the runner-up, which most offsets give)
    assert 5 <= rec.commit.sum() <= (60 if mode == CONF_RATIO else 45)
    # committed tokens are the planted targets (boosted well above the noise)
    np.testing.assert_array_equal(rec.token[rec.commit], run.traj.target[run.to_full(rec.active)][rec.commit])
    # first generation position sits next to the prompt: phi = 1/2
    assert rec.phi[0] == 0.5 and rec.phi[20] == 0.0


def test_config1_with_the_bare_offset_finalizes_none_or_all():
    # planted logit = U[0, 8] on top of unit noise at V = 32000: p_target ~ e^8 / (e^8 + V e^0.5) ~ 0.05 at most,
    # a little more where the target's own noise draw is high
    cfg = CONFIGS[1].replace(base="literal")
    rec, *_ = LockstepRun(cfg, threads=4).next_step()
    assert rec.commit.sum() == 0 and rec.p1.max() < 0.25
    rec, *_ = LockstepRun(cfg.replace(conf_mode=CONF_RATIO, tau_max=0.9, tau_min=0.9), threads=4).next_step()
    assert rec.commit.all() and np.all(rec.conf >= 1.0)


SMALL = {
    2: dict(V=4096, L=64 + 48, steps=40),
    3: dict(V=4096, B=3, L=128 + 40, steps=32),
    4: dict(V=2048, B=2, L=128 + 96, steps=96),
    5: dict(V=4096, B=2, L=256 + 64, steps=48),
}


@pytest.mark.parametrize("cid", [2, 3, 4, 5])
def test_reduced_decode_loops(cid):
    cfg = CONFIGS[cid].replace(**SMALL[cid])
    run = LockstepRun(cfg, threads=4)
    st = run.state
    n_masked0 = int(st.masked.sum())
    counts = []
    for n in range(1, cfg.steps + 9):
        if st.active_count() == 0:
            break
        before = st.masked.copy()
        rec, T, R, rows = run.next_step()
        counts.append(rec.active.size)
        assert np.all(np.abs(rec.conf - rec.tau) >= GUARD * np.maximum(1, np.abs(rec.tau)))
        if cfg.block_size:
            blk = (rec.active % cfg.L - cfg.gen_start) // cfg.block_size
            for b in range(cfg.B):
                assert len(set(blk[rec.active // cfg.L == b])) <= 1
            assert rec.active.size <= cfg.B * cfg.block_size
        assert not np.any(st.masked & ~before)
    # trajectories converge: every position is finalized a few steps after the configured horizon
    assert st.active_count() == 0 and not st.masked.any()
    assert len(st.commit_log) == n_masked0
    if not cfg.block_size:
        assert all(a >= b for a, b in zip(counts, counts[1:]))      # active set only shrinks
    # most positions end on their planted target
    tgt = run.traj.target.reshape(cfg.B, cfg.L)
    agree = np.mean(st.tokens[:, cfg.gen_start:] == tgt[:, cfg.gen_start:])
    assert agree > (0.5 if cid == 5 else 0.9), agree


def test_sub_batch_equals_full_batch_rows():
    cfg = CONFIGS[3].replace(V=1024, B=4, L=128 + 24, steps=20)
    full = LockstepRun(cfg)
    sub = LockstepRun(cfg, batch_rows=[2])
    for n in range(1, 12):
        if full.state.active_count() == 0:
            break
        full.next_step()
        if sub.state.active_count():
            sub.next_step()
    if full.n_bumps == 0 and sub.n_bumps == 0:      # overrides are inputs; equal only when none were needed
        np.testing.assert_array_equal(full.state.tokens[2], sub.state.tokens[0])
        np.testing.assert_array_equal(full.state.masked[2], sub.state.masked[0])


def test_config1_matches_the_stored_oracle_results(golden_dir):
    """Guards the input recipe and the oracle against accidental drift: the stored file was
    written by tests/golden/write_config1_expected.py (generator + oracle only)."""
    import json
    import os
    stored = json.load(open(os.path.join(golden_dir, "config1_expected.json")))
    for name, mode, tau_max, tau_min in (("maxprob", CONF_MAXPROB, 0.9, 0.0), ("ratio", CONF_RATIO, 90.0, 1.0),
                                         ("probgap", CONF_PROBGAP, 0.9, 0.0)):
        cfg = CONFIGS[1].replace(conf_mode=mode, tau_max=tau_max, tau_min=tau_min)
        rec, _, _, _ = LockstepRun(cfg, threads=2).next_step()
        want = stored[name]
        assert rec.active.tolist() == want["active"] and rec.token.tolist() == want["token"]
        assert rec.commit.astype(int).tolist() == want["commit"]
        for key in ("p1", "conf", "tau"):
            got = getattr(rec, key)
            ref = np.array([float.fromhex(h) for h in want[key]])
            np.testing.assert_allclose(got, ref, rtol=1e-13, atol=0)
