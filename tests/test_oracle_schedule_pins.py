"""Pins for the transfer-schedule part of the oracle (Section 3.2; Section 4.2 "Interaction with
transfer schedules", "Implementation details": logical OR, uncapped)."""
import itertools
import math

import numpy as np
import pytest

from oracle import jot_oracle as O


def brute_force(logits, masked, mode, tau_max, tau_min, gamma, D, eps, gen_start, block, k, frac):
    """One step for ONE row straight from the text, Python loops only.  Returns the set finalized."""
    L = len(masked)
    if block > 0 and any(masked):
        first = min(i for i in range(L) if masked[i])
        examined = [i for i in range(L) if masked[i] and (i - gen_start) // block == (first - gen_start) // block]
    else:
        examined = [i for i in range(L) if masked[i]]
    wmax = 2 * sum(gamma ** d for d in range(1, D + 1))
    exits, conf_s = set(), {}
    for i in examined:
        l = [float(x) for x in logits[i]]
        z = sum(math.exp(x) for x in l)
        pi = sorted((math.exp(x) / z for x in l), reverse=True)
        p1, p2 = pi[0], pi[1]
        conf = {0: p1 / (p2 + eps), 1: p1, 2: p1 - p2}[mode]
        w = sum(gamma ** abs(i - j) for j in range(L) if j != i and abs(i - j) <= D and not masked[j])
        tau = tau_max - (tau_max - tau_min) * (min(1.0, w / wmax) if D else 0.0)
        if conf >= tau:
            exits.add(i)
        conf_s[i] = p1
    kk = min(len(examined), k + int(math.floor(frac * len(examined))))
    ranked = sorted(examined, key=lambda i: (-conf_s[i], i))
    return exits | set(ranked[:kk]), exits, set(ranked[:kk])


@pytest.mark.parametrize("L,V,mode,tau_max,tau_min,block,k,frac", [
    (7, 8, O.CONF_RATIO, 9.0, 0.8, 0, 1, 0.0),
    (7, 8, O.CONF_MAXPROB, 0.7, 0.0, 0, 2, 0.0),
    (6, 5, O.CONF_RATIO, 50.0, 0.8, 0, 0, 0.5),
    (8, 6, O.CONF_PROBGAP, 0.6, 0.05, 3, 1, 0.34),
    (6, 4, O.CONF_RATIO, 1e9, 1e9, 2, 1, 0.0),
])
def test_every_mask_matches_brute_force_with_schedule(L, V, mode, tau_max, tau_min, block, k, frac):
    rng = np.random.default_rng(L * 31 + V)
    # distinct irrational-ish logits: no two positions share p1, so the ranking is unambiguous
    logits = (rng.integers(-6, 7, (L, V)) / 2 + rng.random((L, V)) * 1e-3).astype(np.float32)
    gamma, D, eps, gs = 0.5, 2, 1e-12, 1
    p = O.OracleParams(B=1, L=L, V=V, conf_mode=mode, tau_max=tau_max, tau_min=tau_min, gamma=gamma,
                       D=D, eps=eps, gen_start=gs, block_size=block)
    for bits in itertools.product([False, True], repeat=L):
        st = O.OracleState.init(p, np.zeros((1, L), np.int32), np.array(bits)[None])
        rec = st.step_full(logits[None], n_transfer=[k], transfer_frac=frac)
        both, exits, sched = brute_force(logits, list(bits), mode, tau_max, tau_min, gamma, D, eps, gs, block, k, frac)
        assert set(rec.active[rec.commit].tolist()) == both
        assert set(rec.active[rec.exit].tolist()) == exits
        assert set(rec.active[rec.sched].tolist()) == sched
        assert np.array_equal(rec.commit, rec.exit | rec.sched)               # logical OR
        assert rec.k_row[0] == len(sched)
        for i in both:
            assert st.tokens[0, i] == int(np.argmax(logits[i])) and not st.masked[0, i]


def case(seed, B=3, L=30, V=40, gs=6, **kw):
    rng = np.random.default_rng(seed)
    p = O.OracleParams(B=B, L=L, V=V, gen_start=gs, **kw)
    masked = np.zeros((B, L), bool)
    masked[:, gs:] = True
    tokens = np.zeros((B, L), np.int32)
    logits = (rng.standard_normal((B, L, V)) * 2).astype(np.float32)
    return p, tokens, masked, logits, rng


def test_no_schedule_is_the_default_and_k_zero_changes_nothing():
    p, tokens, masked, logits, _ = case(1, conf_mode=O.CONF_RATIO, tau_max=4.0, tau_min=1.0)
    a = O.OracleState.init(p, tokens, masked)
    b = O.OracleState.init(p, tokens, masked)
    ra = a.step_full(logits)
    rb = b.step_full(logits, n_transfer=[0, 0, 0], transfer_frac=0.0)
    assert np.array_equal(ra.commit, rb.commit) and not rb.sched.any()
    assert np.array_equal(ra.commit, ra.exit)


def test_unreachable_threshold_degrades_to_plain_top_k_decoding():
    # Section 4.2 states that a step in which nothing clears its threshold is a step of the ordinary
    # decoder: with tau out of reach every step reveals exactly k per row, most confident first.
    p, tokens, masked, logits, rng = case(2, conf_mode=O.CONF_MAXPROB, tau_max=2.0, tau_min=1.5)
    st = O.OracleState.init(p, tokens, masked)
    n = int(masked[0].sum())
    k = [1, 5, 24]
    steps = 0
    while st.active_count():
        assert steps < 100, "decoding does not terminate"
        before = st.masked.copy()
        rec = st.step_full(logits, n_transfer=k)
        steps += 1
        assert not rec.exit.any()
        for b in range(p.B):
            mine = rec.active // p.L == b
            want_k = min(k[b], int(before[b].sum()))
            assert rec.sched[mine].sum() == want_k == rec.k_row[b]
            if want_k:
                # every selected position is at least as confident as every unselected one
                assert rec.p1[mine][rec.sched[mine]].min() >= rec.p1[mine][~rec.sched[mine]].max(initial=-1)
    assert steps == math.ceil(n / 1)            # the slowest row sets the number of steps
    assert len(st.commit_log) == p.B * n


def test_fraction_one_reveals_everything_and_fraction_is_floored():
    p, tokens, masked, logits, _ = case(3, conf_mode=O.CONF_MAXPROB, tau_max=2.0, tau_min=1.5)
    st = O.OracleState.init(p, tokens, masked)
    rec = st.step_full(logits, transfer_frac=0.26)
    assert rec.k_row.tolist() == [6, 6, 6]      # floor(0.26 * 24)
    rec = st.step_full(logits, transfer_frac=1.0)
    assert st.active_count() == 0 and rec.sched.all()


def test_equal_confidence_is_ranked_by_position_and_rows_without_softmax_are_skipped():
    B, L, V = 1, 10, 6
    p = O.OracleParams(B=B, L=L, V=V, conf_mode=O.CONF_MAXPROB, tau_max=2.0, tau_min=1.5, D=0)
    logits = np.zeros((B, L, V), np.float32)
    logits[0, :, 2] = 3.0                        # identical rows: identical p1
    logits[0, 4, 1] = np.nan                     # no softmax
    logits[0, 7, :] = -np.inf
    st = O.OracleState.init(p, np.zeros((B, L), np.int32), np.ones((B, L), bool))
    rec = st.step_full(logits, n_transfer=[3])
    assert rec.active[rec.sched].tolist() == [0, 1, 2]
    rec = st.step_full(logits, n_transfer=[100])
    assert rec.k_row[0] == 5 and st.masked[0].tolist() == [False] * 4 + [True] + [False] * 2 + [True] + [False] * 2


def test_schedule_stays_inside_the_current_block_and_guarantees_termination():
    p, tokens, masked, logits, rng = case(5, B=2, L=6 + 16, gs=6, conf_mode=O.CONF_RATIO, tau_max=1e9,
                                          tau_min=1e9, block_size=4)
    st = O.OracleState.init(p, tokens, masked)
    steps = 0
    while st.active_count():
        assert steps < 100, "decoding does not terminate"
        rec = st.step_full(logits, n_transfer=[1, 2])
        steps += 1
        blk = (rec.active % p.L - p.gen_start) // p.block_size
        for b in range(p.B):
            assert len(set(blk[rec.active // p.L == b])) <= 1
    assert steps == 16                           # row 0: one position per step, 16 positions
    # early exit only adds to the schedule: with a reachable threshold it finishes no later
    p2 = O.OracleParams(**{**p.__dict__, "tau_max": 3.0, "tau_min": 1.0})
    st2 = O.OracleState.init(p2, tokens, masked)
    steps2 = 0
    while st2.active_count():
        assert steps2 < 100, "decoding does not terminate"
        st2.step_full(logits, n_transfer=[1, 2])
        steps2 += 1
    assert steps2 <= steps
