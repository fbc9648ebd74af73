"""Pins for the KL stability signal of the oracle (the per-token rule Section 2 describes: the KL
divergence between consecutive-step distributions marks predictions that stopped moving)."""
import math

import numpy as np
import pytest
from scipy.special import rel_entr, softmax
from scipy.stats import entropy

from oracle import jot_oracle as O


def test_kl_matches_scipy_and_basic_properties():
    rng = np.random.default_rng(0)
    for V in (2, 9, 500):
        x = (np.round(rng.standard_normal(V) * 2 * 1024) / 1024).astype(np.float32)   # shifts below stay exact
        y = (x + np.round(rng.standard_normal(V) * 0.3 * 1024) / 1024).astype(np.float32)
        p, q = softmax(x.astype(np.float64)), softmax(y.astype(np.float64))
        kl = O.kl_row(x, y, O.F32)
        assert abs(kl - entropy(p, q)) < 1e-13 and abs(kl - rel_entr(p, q).sum()) < 1e-13   # library routines
        assert kl > 0 and O.kl_row(x, x, O.F32) == 0.0
        assert abs(O.kl_row(x + 7, y - 3, O.F32) - kl) < 1e-12                               # shift invariance
        assert abs(O.kl_row(y, x, O.F32) - entropy(q, p)) < 1e-13 and O.kl_row(y, x, O.F32) != kl  # direction


def test_two_token_closed_form_and_infinities():
    a, b = 0.8, 0.3                                   # pi = (a, 1-a), rho = (b, 1-b)
    x = np.array([math.log(a), math.log(1 - a)], np.float32)
    y = np.array([math.log(b), math.log(1 - b)], np.float32)
    p = softmax(x.astype(np.float64))
    q = softmax(y.astype(np.float64))
    want = p[0] * math.log(p[0] / q[0]) + p[1] * math.log(p[1] / q[1])
    assert abs(O.kl_row(x, y, O.F32) - want) < 1e-14
    ninf = np.float32(-np.inf)
    assert O.kl_row(np.array([0, 0], np.float32), np.array([0, ninf], np.float32), O.F32) == math.inf
    assert O.kl_row(np.array([0, ninf], np.float32), np.array([0, 0], np.float32), O.F32) == pytest.approx(math.log(2))
    assert math.isnan(O.kl_row(np.array([0, np.nan], np.float32), np.array([0, 0], np.float32), O.F32))


def make_state(seed, B=2, L=14, V=20, gs=4, **kw):
    rng = np.random.default_rng(seed)
    p = O.OracleParams(B=B, L=L, V=V, gen_start=gs, conf_mode=O.CONF_RATIO, tau_max=1e9, tau_min=1e9, D=2, **kw)
    masked = np.zeros((B, L), bool)
    masked[:, gs:] = True
    return p, O.OracleState.init(p, np.zeros((B, L), np.int32), masked), rng


def test_rule_needs_history_small_kl_and_enough_confidence():
    p, st, rng = make_state(1)
    base = (rng.standard_normal((p.B, p.L, p.V))).astype(np.float32)
    base[:, :, 3] += 9.0                              # every row confident in token 3 ...
    base[1, 7, 3] -= 8.5                              # ... except this one, in both steps
    l1 = base.copy()
    l2 = base + (rng.standard_normal(base.shape) * 0.01).astype(np.float32)     # barely moved
    l2[0, 6] = rng.standard_normal(p.V).astype(np.float32) * 3                  # this one moved a lot
    flat = lambda lg: lg.reshape(p.B * p.L, p.V)
    act = st.active_list()
    rec1 = st.step(flat(l1)[act], prev_rows=flat(l1)[act], kl_threshold=0.01, kl_min_prob=0.9)
    assert not rec1.stable.any() and np.isnan(rec1.kl).all()                      # no previous step yet
    act = st.active_list()
    rec2 = st.step(flat(l2)[act], prev_rows=flat(l1)[act], kl_threshold=0.01, kl_min_prob=0.9)
    moved = int(np.flatnonzero(act == 0 * p.L + 6)[0])
    unsure = int(np.flatnonzero(act == 1 * p.L + 7)[0])
    assert not rec2.stable[moved] and rec2.kl[moved] > 0.01
    assert not rec2.stable[unsure] and rec2.p1[unsure] < 0.9 and rec2.kl[unsure] <= 0.01
    others = np.ones(act.size, bool)
    others[[moved, unsure]] = False
    assert rec2.stable[others].all() and np.all(rec2.kl[others] <= 0.01) and np.all(rec2.kl[others] >= 0)
    for k in np.flatnonzero(others)[:5]:
        bb, ii = divmod(int(act[k]), p.L)
        assert abs(rec2.kl[k] - entropy(softmax(l2[bb, ii].astype(np.float64)), softmax(l1[bb, ii].astype(np.float64)))) < 1e-13
    assert np.array_equal(rec2.commit, rec2.stable)
    assert st.masked[0, 6] and st.masked[1, 7] and st.masked.sum() == 2


def test_rule_is_ored_with_the_others_and_off_by_default():
    p, st, rng = make_state(2)
    lg = rng.standard_normal((p.B, p.L, p.V)).astype(np.float32)
    lg[:, :, 1] += 12.0
    act = st.active_list()
    rows = lg.reshape(-1, p.V)[act]
    st.step(rows)
    act = st.active_list()
    rec = st.evaluate(rows, n_transfer=[1, 0], prev_rows=rows, kl_threshold=1e-6, kl_min_prob=0.5)
    assert rec.stable.all() and np.all(rec.kl == 0.0)
    assert np.array_equal(rec.commit, rec.exit | rec.sched | rec.rowwide | rec.stable)
    assert st.evaluate(rows, prev_rows=rows, kl_threshold=0.0).stable.all()              # the comparison is inclusive
    rec0 = st.evaluate(rows)
    assert not rec0.stable.any() and np.isnan(rec0.kl).all()


def test_new_block_has_no_history():
    p, st, rng = make_state(3, B=1, L=4 + 8, gs=4, block_size=4)
    lg = rng.standard_normal((1, p.L, p.V)).astype(np.float32)
    lg[:, :, 2] += 15.0
    flat = lg.reshape(-1, p.V)
    rec = st.step(flat[st.active_list()], prev_rows=flat[st.active_list()], kl_threshold=0.1)
    assert not rec.commit.any()
    rec = st.step(flat[st.active_list()], prev_rows=flat[st.active_list()], kl_threshold=0.1)
    assert rec.commit.all() and rec.active.tolist() == [4, 5, 6, 7]               # first block, now with history
    rec = st.step(flat[st.active_list()], prev_rows=flat[st.active_list()], kl_threshold=0.1)
    assert rec.active.tolist() == [8, 9, 10, 11] and not rec.commit.any()         # new block: no history yet


def test_history_means_the_step_just_before():
    p, st, rng = make_state(4, B=1, L=8, gs=4)
    lg = rng.standard_normal((1, p.L, p.V)).astype(np.float32)
    lg[:, :, 2] += 15.0
    flat = lg.reshape(-1, p.V)
    act = st.active_list()
    st.step(flat[act])
    broken = flat[act].copy()
    broken[1, 0] = np.nan                                                          # position 5 has no softmax this step
    st.step(broken)
    rec = st.step(flat[act], prev_rows=flat[act], kl_threshold=0.1)
    assert rec.stable.tolist() == [True, False, True, True]                        # 5 was fine two steps ago: not enough
