"""Pins for the row-wide early-commit rule in the oracle (the global rule Section 2 describes:
when the top-2 gap clears a threshold, all remaining masked positions are finalized together)."""
import math

import numpy as np
import pytest

from oracle import jot_oracle as O


def make(B=2, L=12, V=9, gs=3, seed=0, **kw):
    rng = np.random.default_rng(seed)
    p = O.OracleParams(B=B, L=L, V=V, gen_start=gs, conf_mode=O.CONF_RATIO, tau_max=1e9, tau_min=1e9, D=2, **kw)
    masked = np.zeros((B, L), bool)
    masked[:, gs:] = True
    logits = (rng.standard_normal((B, L, V)) * 2).astype(np.float32)
    return p, np.zeros((B, L), np.int32), masked, logits


def brute_gap(logits_row_positions):
    gaps = []
    for l in logits_row_positions:
        top = sorted((float(x) for x in l), reverse=True)
        gaps.append(top[0] - top[1])
    return sum(gaps) / len(gaps)


def test_mean_gap_and_all_or_nothing_per_row():
    p, tokens, masked, logits = make()
    logits[1, :, 4] += 30.0                       # row 1 is very decided, row 0 is not
    st = O.OracleState.init(p, tokens, masked)
    rec = st.step_full(logits, global_gap=8.0)
    for b in range(p.B):
        want = brute_gap([logits[b, i] for i in range(p.gen_start, p.L)])
        assert abs(rec.gap_row[b] - want) < 1e-12
    assert rec.gap_row[0] < 8.0 <= rec.gap_row[1]
    row_of = rec.active // p.L
    assert not rec.commit[row_of == 0].any() and rec.commit[row_of == 1].all()
    assert np.array_equal(rec.commit, rec.rowwide)
    assert st.masked[0, p.gen_start:].all() and not st.masked[1].any()
    np.testing.assert_array_equal(st.tokens[1, p.gen_start:], np.argmax(logits[1, p.gen_start:], -1))


def test_threshold_is_inclusive_and_off_by_default():
    p, tokens, masked, logits = make(B=1)
    st = O.OracleState.init(p, tokens, masked)
    g = st.evaluate(logits.reshape(-1, p.V)[st.active_list()], global_gap=1e9).gap_row[0]
    assert st.evaluate(logits.reshape(-1, p.V)[st.active_list()], global_gap=g).commit.all()
    assert not st.evaluate(logits.reshape(-1, p.V)[st.active_list()], global_gap=math.nextafter(g, 1e9)).commit.any()
    rec = st.evaluate(logits.reshape(-1, p.V)[st.active_list()])
    assert not rec.rowwide.any() and np.isnan(rec.gap_row).all()


def test_rows_without_softmax_neither_count_nor_commit_and_rule_is_ored():
    p, tokens, masked, logits = make(B=1)
    logits[0, :, 2] += 25.0
    logits[0, 5, 0] = np.nan
    p2 = O.OracleParams(**{**p.__dict__, "tau_max": 3.0, "tau_min": 1.0})
    st = O.OracleState.init(p2, tokens, masked)
    rec = st.step_full(logits, global_gap=5.0, n_transfer=[1])
    ok = rec.status == 0
    assert rec.rowwide[ok].all() and not rec.rowwide[~ok].any() and st.masked[0, 5]
    assert np.array_equal(rec.commit, rec.exit | rec.sched | rec.rowwide)
    want = brute_gap([logits[0, i] for i in range(p.gen_start, p.L) if i != 5])
    assert abs(rec.gap_row[0] - want) < 1e-12


def test_block_mode_applies_the_rule_to_the_current_block_only():
    p, tokens, masked, logits = make(B=1, L=3 + 12, block_size=4)
    logits[0, :, 1] += 40.0
    st = O.OracleState.init(p, tokens, masked)
    steps = 0
    while st.active_count():
        assert steps < 10
        rec = st.step_full(logits, global_gap=6.0)
        assert rec.active.size == 4 and rec.commit.all()
        steps += 1
    assert steps == 3
