"""Pins for the CPU oracle: it is checked against things other than itself.

* numbers the paper prints (tests/golden/paper_printed_values.json),
* closed forms and special cases of Eq. 2-5,
* library routines used as a third opinion (scipy softmax / logsumexp, numpy sort),
* brute force over every mask for tiny canvases, written here from the equations
  with plain Python loops and math.exp,
* invariants of Algorithm 1's loop.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from gen.bf16 import bf16_bits_to_f32, f32_to_bf16_bits
from oracle import jot_oracle as O


@pytest.fixture(scope="module")
def printed(golden_dir):
    with open(os.path.join(golden_dir, "paper_printed_values.json")) as f:
        return json.load(f)


def rows_of(x, dtype):
    x = np.asarray(x, np.float32)
    if x.ndim == 1:
        x = x[None]
    return x if dtype == O.F32 else f32_to_bf16_bits(x)


# --------------------------------------------------------------------------- softmax / S / p1

@pytest.mark.parametrize("V", [2, 3, 16, 257, 4099])
def test_probabilities_sum_to_one_and_match_scipy(V):
    rng = np.random.default_rng(V)
    row = (rng.standard_normal(V) * 3).astype(np.float32)
    pi = O.softmax_row(row, O.F32)
    assert abs(pi.sum() - 1.0) < 1e-12
    np.testing.assert_allclose(pi, softmax(row.astype(np.float64)), rtol=1e-12, atol=0)
    a, m1, m2, S, st = O.row_stats(row[None], O.F32)
    assert st[0] == 0
    # S = exp(logsumexp(l) - m1): library log-sum-exp as the independent routine
    assert abs(S[0] - math.exp(logsumexp(row.astype(np.float64)) - float(row.max()))) < 1e-11 * S[0]
    # p1, p2 are the two largest entries of the full probability vector
    top = np.sort(pi)[::-1]
    assert abs(1.0 / S[0] - top[0]) < 1e-14
    assert abs(math.exp(m2[0] - m1[0]) / S[0] - top[1]) < 1e-14
    assert a[0] == int(np.argmax(row))


def test_uniform_row():
    for V in (2, 7, 1000):
        a, m1, m2, S, st = O.row_stats(np.full((1, V), 0.25, np.float32), O.F32)
        assert a[0] == 0 and m1[0] == m2[0] == 0.25
        assert abs(S[0] - V) < 1e-12 * V
        eps = 1e-12
        r = O.confidence(1 / S, np.exp(m2 - m1) / S, O.CONF_RATIO, eps)[0]
        assert abs(r - 1.0 / (1.0 + eps * V)) < 1e-15


def test_shift_invariance_and_minus_inf_is_deletion():
    rng = np.random.default_rng(1)
    row = rng.integers(-40, 40, 64).astype(np.float32) / 4     # exactly shiftable
    base = O.row_stats(row[None], O.F32)
    shifted = O.row_stats((row + 100.0)[None], O.F32)
    assert base[0][0] == shifted[0][0]
    assert base[3][0] == shifted[3][0]                           # S identical bit for bit
    assert base[2][0] - base[1][0] == shifted[2][0] - shifted[1][0]
    # inserting -inf entries changes nothing except the indices
    ins = np.insert(row, [0, 10, 64], -np.inf).astype(np.float32)
    withinf = O.row_stats(ins[None], O.F32)
    assert withinf[4][0] == 0
    assert withinf[3][0] == base[3][0] and withinf[1][0] == base[1][0] and withinf[2][0] == base[2][0]
    kept = np.flatnonzero(np.isfinite(ins))
    assert kept[base[0][0]] == withinf[0][0]


def test_rows_without_softmax_are_flagged():
    bad = np.zeros((4, 8), np.float32)
    bad[0, 3] = np.nan
    bad[1, 5] = np.inf
    bad[2, :] = -np.inf
    a, m1, m2, S, st = O.row_stats(bad, O.F32)
    assert list(st) == [1, 1, 1, 0]
    assert np.isnan(S[:3]).all() and S[3] == 8.0


def test_bf16_is_widened_exactly():
    rng = np.random.default_rng(2)
    x = (rng.standard_normal((5, 300)) * 4).astype(np.float32)
    h = f32_to_bf16_bits(x)
    wide = bf16_bits_to_f32(h)
    r16 = O.row_stats(h, O.BF16)
    r32 = O.row_stats(wide, O.F32)
    for u, v in zip(r16, r32):
        np.testing.assert_array_equal(u, v)


# --------------------------------------------------------------------------- top-2 / ratio / argmax

def test_ratio_closed_form_and_printed_logit_gaps(printed):
    eps = printed["eps"]["value"]
    assert eps == 1e-12
    for pair in printed["logit_gap_for_tau"]["pairs"]:
        tau = pair["tau"]
        gap = math.log(tau)
        assert round(gap, pair["digits"]) == pair["gap_printed"]
        # a row whose top-2 logits differ by ln(tau) has ratio tau (up to eps and fp32 rounding of the gap)
        V = 50
        row = np.full(V, -30.0, np.float32)
        row[17] = np.float32(gap)
        row[4] = 0.0
        a, m1, m2, S, st = O.row_stats(row[None], O.F32)
        assert a[0] == 17
        p1, p2 = 1 / S, np.exp(m2 - m1) / S
        r = O.confidence(p1, p2, O.CONF_RATIO, eps)[0]
        g32 = float(np.float32(gap))
        assert abs(r - 1.0 / (math.exp(-g32) + eps * S[0])) < 1e-9 * r     # closed form
        assert abs(r - tau) < 1e-5 * tau
        # the other two signals from the same (p1, p2)
        assert O.confidence(p1, p2, O.CONF_MAXPROB, eps)[0] == p1[0]
        assert O.confidence(p1, p2, O.CONF_PROBGAP, eps)[0] == p1[0] - p2[0]


def test_flip_budget_arithmetic_printed(printed):
    fb = printed["flip_budget"]
    assert round(2 * fb["L"] / (1 + fb["tau"]), fb["digits"]) == fb["printed"]


def test_committed_positions_leave_the_runner_up_a_small_head_to_head_share():
    # Fact used by Section 5's flip bound: a position only commits when r = p1/p2 >= tau, so among
    # the two leading tokens alone the second one then has probability p2/(p1 + p2) <= 1/(1 + tau)
    # (here tau is the position's own tau^i, since the threshold is spatially modulated).  Checked
    # from the full probability vectors on every position a multi-step decode commits.
    rng = np.random.default_rng(11)
    B, L, V, gs = 2, 40, 30, 6
    p = O.OracleParams(B=B, L=L, V=V, conf_mode=O.CONF_RATIO, tau_max=20.0, tau_min=1.5, gamma=0.5, D=4, gen_start=gs)
    masked = np.zeros((B, L), bool)
    masked[:, gs:] = True
    st = O.OracleState.init(p, np.zeros((B, L), np.int32), masked)
    n_committed = 0
    for step in range(12):
        act = st.active_list()
        if act.size == 0:
            break
        rows = (rng.standard_normal((act.size, V)) * (1.0 + 0.5 * step)).astype(np.float32)
        rec = st.step(rows)
        for k in np.flatnonzero(rec.commit):
            pi = np.sort(O.softmax_row(rows[k], O.F32))[::-1]
            share = pi[1] / (pi[0] + pi[1])
            assert share <= 1.0 / (1.0 + rec.tau[k]) + 1e-12
            assert 2.0 * share <= 2.0 / (1.0 + p.tau_min) + 1e-12       # hence the per-position flip bound
            n_committed += 1
        for k in np.flatnonzero(~rec.commit & (rec.status == 0)):       # and the converse up to eps
            pi = np.sort(O.softmax_row(rows[k], O.F32))[::-1]
            assert pi[1] / (pi[0] + pi[1]) > 1.0 / (1.0 + rec.tau[k]) - 1e-9
    assert n_committed > 20


@pytest.mark.parametrize("seed", range(20))
def test_top2_and_argmax_brute_force_small_vocab(seed):
    rng = np.random.default_rng(seed)
    V = int(rng.integers(2, 17))
    row = rng.integers(-3, 4, V).astype(np.float32)              # coarse grid: many ties
    a, m1, m2, S, st = O.row_stats(row[None], O.F32)
    order = sorted(range(V), key=lambda v: (-row[v], v))
    assert a[0] == order[0]
    assert m1[0] == row[order[0]] and m2[0] == row[order[1]]
    probs = sorted((math.exp(float(x) - float(row.max())) for x in row), reverse=True)
    tot = sum(probs)
    assert abs(1 / S[0] - probs[0] / tot) < 1e-15
    assert abs(math.exp(m2[0] - m1[0]) / S[0] - probs[1] / tot) < 1e-15


def test_duplicated_maximum_gives_ratio_one_and_lowest_index():
    row = np.array([0.0, 2.0, -1.0, 2.0, 2.0, 1.0], np.float32)
    a, m1, m2, S, st = O.row_stats(row[None], O.F32)
    assert a[0] == 1 and m1[0] == m2[0] == 2.0
    r = O.confidence(1 / S, np.exp(m2 - m1) / S, O.CONF_RATIO, 0.0)[0]
    assert r == 1.0


def test_vocabulary_permutation():
    rng = np.random.default_rng(5)
    row = rng.integers(-8, 9, 40).astype(np.float32)
    perm = rng.permutation(40)
    base = O.row_stats(row[None], O.F32)
    permd = O.row_stats(row[perm][None], O.F32)
    assert permd[1][0] == base[1][0] and permd[2][0] == base[2][0]
    assert abs(permd[3][0] - base[3][0]) < 1e-12 * base[3][0]
    # lowest-index rule re-applied in the permuted order
    assert permd[0][0] == min(k for k in range(40) if row[perm[k]] == row.max())


# --------------------------------------------------------------------------- Eq. 3-5

def test_w_max_closed_forms(printed):
    exact = {(0.5, 8): 1.9921875, (0.5, 16): 2 * (1 - 2.0 ** -16), (0.5, 4): 1.875}
    for (g, D), val in exact.items():
        assert O.w_max(g, D) == val
    for g in printed["sweep_grid"]["gamma"]:
        for D in printed["sweep_grid"]["D"]:
            closed = 2 * g * (1 - g ** D) / (1 - g)              # geometric series
            assert abs(O.w_max(g, D) - closed) < 1e-13 * closed
    assert O.w_max(1.0, 5) == 10.0


def eq3_brute(resolved_row, i, gamma, D):
    w = 0.0
    for j in range(len(resolved_row)):
        if j != i and abs(i - j) <= D and resolved_row[j]:
            w += gamma ** abs(i - j)
    return w


@pytest.mark.parametrize("gamma,D", [(0.5, 8), (0.3, 4), (0.9, 16), (0.7, 8), (1.0, 3)])
def test_spatial_weight_against_double_loop(gamma, D):
    rng = np.random.default_rng(int(gamma * 100) + D)
    res = rng.random((3, 41)) < 0.5
    w = O.spatial_weight(res, gamma, D)
    for b in range(3):
        for i in range(41):
            assert abs(w[b, i] - eq3_brute(res[b], i, gamma, D)) < 1e-13
    # mirror symmetry: reversing the row reverses the weights
    np.testing.assert_allclose(O.spatial_weight(res[:, ::-1], gamma, D), w[:, ::-1], rtol=0, atol=1e-15)


def test_threshold_special_cases(printed):
    d = printed["defaults"]["dream"]
    p = O.OracleParams(B=1, L=64, V=8, tau_max=d["tau_max"], tau_min=d["tau_min"],
                       gamma=d["gamma"], D=d["D"], gen_start=16)
    masked = np.zeros((1, 64), bool)
    masked[0, 16:] = True                                        # 16 prompt tokens, 48 masked
    tau, phi = O.threshold(~masked, p)
    # first generation position: the whole left half-window is resolved, the right is not
    assert phi[0, 16] == 0.5 and tau[0, 16] == 45.5
    # second: left neighbours at distance 2..8
    assert abs(phi[0, 17] - 0.49609375 / 1.9921875) < 1e-16
    # interior of the masked region (no resolved neighbour within D): strict threshold
    assert np.all(phi[0, 24:56] == 0) and np.all(tau[0, 24:56] == 90.0)
    # last position: canvas end contributes nothing
    assert phi[0, 63] == 0.0
    # a single masked hole surrounded by resolved tokens: phi = 1, tau = tau_min
    hole = np.zeros((1, 64), bool)
    hole[0, 30] = True
    tau, phi = O.threshold(~hole, p)
    assert phi[0, 30] == 1.0 and tau[0, 30] == 1.0
    # hole at the canvas edge can never reach phi = 1 (zero padding)
    edge = np.zeros((1, 64), bool)
    edge[0, 0] = True
    tau, phi = O.threshold(~edge, p)
    assert phi[0, 0] == 0.5
    # D = 0 or tau_min = tau_max: no spatial modulation, tau^i = tau everywhere
    p0 = O.OracleParams(B=1, L=64, V=8, D=0)
    assert np.all(O.threshold(~masked, p0)[0] == 90.0)
    pf = O.OracleParams(B=1, L=64, V=8, tau_min=90.0)
    assert np.all(O.threshold(~masked, pf)[0] == 90.0)


def test_dyadic_weights_are_exact_for_gamma_half():
    rng = np.random.default_rng(11)
    res = rng.random((2, 50)) < 0.6
    w = O.spatial_weight(res, 0.5, 8)
    assert np.all(w * 256 == np.round(w * 256))


# --------------------------------------------------------------------------- brute force over all masks

def brute_force_step(logits, masked, tokens, mode, tau_max, tau_min, gamma, D, eps, gen_start, block):
    """One step straight from Eq. 2-6 with Python loops; returns (tokens, masked, commits)."""
    L = len(masked)
    if block > 0 and any(masked):
        first = min(i for i in range(L) if masked[i])
        blk = (first - gen_start) // block
        examined = [i for i in range(L) if masked[i] and (i - gen_start) // block == blk]
    else:
        examined = [i for i in range(L) if masked[i]]
    wmax = 2 * sum(gamma ** d for d in range(1, D + 1))
    new_tokens, new_masked, commits = list(tokens), list(masked), []
    for i in examined:
        l = [float(x) for x in logits[i]]
        z = sum(math.exp(x) for x in l)
        pi = [math.exp(x) / z for x in l]
        order = sorted(range(len(l)), key=lambda v: (-l[v], v))
        p1, p2 = pi[order[0]], pi[order[1]]
        conf = {0: p1 / (p2 + eps), 1: p1, 2: p1 - p2}[mode]
        w = sum(gamma ** abs(i - j) for j in range(L)
                if j != i and abs(i - j) <= D and not masked[j])
        phi = min(1.0, w / wmax) if D > 0 else 0.0
        tau = tau_max - (tau_max - tau_min) * phi
        if conf >= tau:
            new_tokens[i] = order[0]
            new_masked[i] = False
            commits.append((i, order[0]))
    return new_tokens, new_masked, commits


@pytest.mark.parametrize("L,V,mode,tau_max,tau_min,block", [
    (8, 16, O.CONF_RATIO, 7.0, 0.8, 0),
    (8, 5, O.CONF_MAXPROB, 0.6, 0.0, 0),
    (7, 16, O.CONF_PROBGAP, 0.5, 0.05, 0),
    (8, 9, O.CONF_RATIO, 3.0, 0.8, 3),
    (6, 2, O.CONF_MAXPROB, 0.7, 0.2, 2),
])
def test_every_mask_matches_brute_force(L, V, mode, tau_max, tau_min, block):
    rng = np.random.default_rng(L * 100 + V)
    # small grid in steps of 0.5 (tied maxima give r = 1 - tiny, so tau_min stays off 1 here);
    # the grid is clear of every threshold for these seeds (asserted below)
    logits = (rng.integers(-4, 5, (L, V)) / 2).astype(np.float32)
    gamma, D, eps, gs = 0.5, 2, 1e-12, 1
    p = O.OracleParams(B=1, L=L, V=V, conf_mode=mode, tau_max=tau_max, tau_min=tau_min,
                       gamma=gamma, D=D, eps=eps, gen_start=gs, block_size=block)
    for bits in itertools.product([False, True], repeat=L):
        masked = np.array(bits)[None]
        tokens = np.full((1, L), 99, np.int32)
        st = O.OracleState.init(p, tokens, masked)
        rec = st.step_full(logits[None])
        assert np.all(np.abs(rec.conf - rec.tau) > 1e-9), "test grid sits on a threshold"
        bt, bm, bc = brute_force_step(logits, list(bits), [99] * L, mode, tau_max, tau_min,
                                      gamma, D, eps, gs, block)
        assert st.tokens[0].tolist() == bt
        assert st.masked[0].tolist() == bm
        assert [(pos, tok) for (_, pos, tok) in st.commit_log] == bc


# --------------------------------------------------------------------------- limiting thresholds, no-op steps

def random_case(seed, B=2, L=24, V=32, gen_start=5, **kw):
    rng = np.random.default_rng(seed)
    p = O.OracleParams(B=B, L=L, V=V, gen_start=gen_start, **kw)
    masked = np.zeros((B, L), bool)
    masked[:, gen_start:] = rng.random((B, L - gen_start)) < 0.8
    tokens = rng.integers(0, V, (B, L)).astype(np.int32)
    logits = (rng.standard_normal((B, L, V)) * 3).astype(np.float32)
    return p, tokens, masked, logits


@pytest.mark.parametrize("mode", [O.CONF_RATIO, O.CONF_MAXPROB, O.CONF_PROBGAP])
def test_threshold_zero_finalizes_everything_in_one_step(mode):
    p, tokens, masked, logits = random_case(3, conf_mode=mode, tau_max=0.0, tau_min=0.0)
    st = O.OracleState.init(p, tokens, masked)
    rec = st.step_full(logits)
    assert rec.commit.all() and not st.masked.any() and st.active_count() == 0
    np.testing.assert_array_equal(st.tokens[masked], np.argmax(logits, -1)[masked])
    np.testing.assert_array_equal(st.tokens[~masked], tokens[~masked])


@pytest.mark.parametrize("mode", [O.CONF_MAXPROB, O.CONF_PROBGAP])
def test_threshold_above_one_finalizes_nothing(mode):
    p, tokens, masked, logits = random_case(4, conf_mode=mode, tau_max=1.5, tau_min=1.0 + 1e-9)
    st = O.OracleState.init(p, tokens, masked)
    rec = st.step_full(logits)
    assert not rec.commit.any()
    np.testing.assert_array_equal(st.tokens, tokens)            # no pass: state untouched
    np.testing.assert_array_equal(st.masked, masked)
    assert st.commit_log == [] and st.step_index == 1


def test_ratio_is_at_least_one_minus_tiny():
    # r >= 1/(1 + eps*S): any tau_max <= 1 - 1e-6 finalizes every position in ratio mode
    p, tokens, masked, logits = random_case(6, conf_mode=O.CONF_RATIO, tau_max=1 - 1e-6, tau_min=0.5)
    st = O.OracleState.init(p, tokens, masked)
    assert st.step_full(logits).commit.all()


# --------------------------------------------------------------------------- loop invariants

@pytest.mark.parametrize("block", [0, 4])
@pytest.mark.parametrize("mode,tau_max,tau_min", [(O.CONF_RATIO, 20.0, 1.0), (O.CONF_MAXPROB, 0.8, 0.0)])
def test_loop_invariants(block, mode, tau_max, tau_min):
    B, L, V, gs = 3, 29, 24, 6
    rng = np.random.default_rng(17 + block)
    p = O.OracleParams(B=B, L=L, V=V, conf_mode=mode, tau_max=tau_max, tau_min=tau_min,
                       gamma=0.5, D=3, gen_start=gs, block_size=block)
    masked0 = np.zeros((B, L), bool)
    masked0[:, gs:] = True
    tokens0 = rng.integers(0, V, (B, L)).astype(np.int32)
    st = O.OracleState.init(p, tokens0, masked0)
    target = rng.integers(0, V, (B, L))
    conv = rng.integers(1, 30, (B, L))
    prev_tokens, prev_masked = st.tokens.copy(), st.masked.copy()
    for n in range(1, 60):
        act = st.active_list()
        if act.size == 0:
            break
        # active list = masked and eligible, ascending
        assert np.all(np.diff(act) > 0)
        np.testing.assert_array_equal(act, np.flatnonzero(O.eligible(st.masked, p).reshape(-1)))
        logits = rng.standard_normal((B, L, V)).astype(np.float32)
        boost = 12.0 / (1 + np.exp(-(n - conv) / 2.0))
        np.put_along_axis(logits, target[..., None], (np.take_along_axis(logits, target[..., None], -1)
                                                      + boost[..., None]).astype(np.float32), -1)
        elig_before = O.eligible(st.masked, p)
        rec = st.step_full(logits)
        assert rec.step == n == st.step_index
        frozen = ~prev_masked
        np.testing.assert_array_equal(st.tokens[frozen], prev_tokens[frozen])    # frozen never change
        assert not np.any(st.masked & ~prev_masked)                               # finalized set only grows
        newly = prev_masked & ~st.masked
        assert not np.any(newly & ~elig_before)                                   # never outside the examined set
        np.testing.assert_array_equal(st.tokens[st.masked], prev_tokens[st.masked])
        prev_tokens, prev_masked = st.tokens.copy(), st.masked.copy()
    log = st.commit_log
    assert len({pos for (_, pos, _) in log}) == len(log)                          # each position once
    assert all(log[k][0] < log[k + 1][0] or (log[k][0] == log[k + 1][0] and log[k][1] < log[k + 1][1])
               for k in range(len(log) - 1))
    assert len(log) == int(masked0.sum() - st.masked.sum())
    if block:
        # blocks are finished strictly in order within each row
        for b in range(B):
            steps = {}
            for (s, pos, _) in log:
                if pos // L == b:
                    steps.setdefault((pos % L - gs) // block, []).append(s)
            ks = sorted(steps)
            for k0, k1 in zip(ks, ks[1:]):
                assert max(steps[k0]) < min(steps[k1])


def run_loop(p, tokens, masked, logit_seq):
    st = O.OracleState.init(p, tokens, masked)
    history = []
    for logits in logit_seq:
        if st.active_count() == 0:
            break
        st.step_full(logits)
        history.append(st.masked.copy())
    return history


def test_monotonicity_in_tau_max_and_spatial_only_helps():
    B, L, V, gs = 2, 40, 50, 8
    rng = np.random.default_rng(23)
    masked = np.zeros((B, L), bool)
    masked[:, gs:] = True
    tokens = np.zeros((B, L), np.int32)
    seq = []
    target = rng.integers(0, V, (B, L))
    conv = rng.integers(1, 20, (B, L))
    for n in range(1, 26):
        lg = rng.standard_normal((B, L, V)).astype(np.float32)
        boost = (10.0 / (1 + np.exp(-(n - conv) / 1.5))).astype(np.float32)
        np.put_along_axis(lg, target[..., None], boost[..., None] + 4.0, -1)
        seq.append(lg)
    hist = {}
    for tm in (0.7, 0.8, 0.9):
        p = O.OracleParams(B=B, L=L, V=V, conf_mode=O.CONF_MAXPROB, tau_max=tm, tau_min=0.0,
                           gamma=0.5, D=8, gen_start=gs)
        hist[tm] = run_loop(p, tokens, masked, seq)
    for lo, hi in ((0.7, 0.8), (0.8, 0.9)):
        for n in range(len(hist[hi])):
            m_lo = hist[lo][n] if n < len(hist[lo]) else np.zeros_like(masked)
            assert not np.any(m_lo & ~hist[hi][n])       # lower tau_max: superset finalized at every step
    # spatial modulation only lowers thresholds: with it the finalized set is a superset at every step
    on = O.OracleParams(B=B, L=L, V=V, conf_mode=O.CONF_RATIO, tau_max=90.0, tau_min=1.0, D=8, gen_start=gs)
    off = O.OracleParams(B=B, L=L, V=V, conf_mode=O.CONF_RATIO, tau_max=90.0, tau_min=1.0, D=0, gen_start=gs)
    h_on, h_off = run_loop(on, tokens, masked, seq), run_loop(off, tokens, masked, seq)
    assert len(h_on) <= len(h_off)
    for n in range(len(h_off)):
        m_on = h_on[n] if n < len(h_on) else np.zeros_like(masked)
        assert not np.any(m_on & ~h_off[n])


def test_simultaneous_update_within_a_step():
    # two adjacent masked holes between resolved tokens: each sees the other as masked this step,
    # even though both commit; next step nothing is left.
    L, V = 9, 4
    p = O.OracleParams(B=1, L=L, V=V, conf_mode=O.CONF_RATIO, tau_max=90.0, tau_min=1.0, gamma=0.5, D=1)
    masked = np.zeros((1, L), bool)
    masked[0, 4:6] = True
    logits = np.zeros((1, L, V), np.float32)
    # gap g: r = e^g.  With one resolved neighbour (phi = 1/2) tau = 45.5; with both (phi = 1) tau = 1.
    logits[0, 4, 2] = math.log(50.0)     # passes 45.5
    logits[0, 5, 1] = math.log(40.0)     # would only pass if position 4 already counted as resolved
    st = O.OracleState.init(p, np.zeros((1, L), np.int32), masked)
    rec = st.step_full(logits)
    assert rec.tau.tolist() == [45.5, 45.5]
    assert rec.commit.tolist() == [True, False]
    rec2 = st.step_full(logits)
    assert rec2.tau.tolist() == [1.0] and rec2.commit.tolist() == [True]
    assert st.commit_log == [(1, 4, 2), (2, 5, 1)]


def test_softmax_is_defined_for_rows_of_any_magnitude():
    # Section 4.1 defines pi = softmax(l) for every finite row: only differences from the row maximum
    # enter.  Rows far from zero (where binary32 still resolves the differences) must give the
    # softmax of the shifted row, fill values of any size count as probability 0.
    from scipy.special import softmax
    small = np.array([0.0, 1.0, 2.0, 0.5, -3.0, 2.0], np.float32)
    want = softmax(small.astype(np.float64))
    for shift in (2.0 ** 22, -(2.0 ** 22), 1.0e9, -1.0e9, 2.0 ** 100, -(2.0 ** 100)):
        row = (small.astype(np.float64) * (1.0 if abs(shift) < 2 ** 23 else 0.0) + shift).astype(np.float32)
        exact = row.astype(np.float64) - float(row.max())         # what binary32 kept of the differences
        got = O.softmax_row(row, O.F32)
        np.testing.assert_allclose(got, softmax(exact), rtol=1e-14, atol=0)
        if abs(shift) < 2 ** 23:
            np.testing.assert_allclose(got, want, rtol=1e-14, atol=0)
    rows = np.zeros((4, 6), np.float32)
    rows[0, :] = [-1e30, 1.0, -3e38, 0.0, -1e9, -np.inf]
    rows[1, :] = 4.1e6
    rows[2, :] = -3.0e38
    rows[3, :] = [3.0e38, -3.0e38, 0, 0, 0, 0]
    a, m1, m2, S, st = O.row_stats(rows, O.F32)
    assert st.tolist() == [0, 0, 0, 0]
    assert a.tolist() == [1, 0, 0, 0]
    assert abs(S[0] - (1 + math.exp(-1))) < 1e-15 and S[1] == 6.0 and S[2] == 6.0 and S[3] == 1.0
