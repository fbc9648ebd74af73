"""Pins for sampling-based finalization in the oracle (Section 4.1, "Early-Exit Decision": the
finalized token may be sampled from the predicted distribution instead of the argmax)."""
import math

import numpy as np
import pytest
from scipy import stats
from scipy.special import softmax

from oracle import jot_oracle as O


def test_inverse_cdf_matches_numpy_searchsorted():
    rng = np.random.default_rng(0)
    for V in (2, 5, 64, 1000):
        row = (rng.standard_normal(V) * 2).astype(np.float32)
        cdf = np.cumsum(softmax(row.astype(np.float64)))
        for u in rng.random(200):
            v, lo, hi = O.sample_row(row, O.F32, u)
            want = int(np.searchsorted(cdf, u, side="right"))      # first index with cdf > u
            if min(abs(cdf - u)) > 1e-12:
                assert v == min(want, V - 1)
                assert lo <= u < hi
                assert abs(hi - cdf[v]) < 1e-12 and abs((hi - lo) - softmax(row.astype(np.float64))[v]) < 1e-12


def test_extreme_uniforms_and_zero_probability_tokens():
    row = np.array([-np.inf, 0.0, -np.inf, math.log(3.0), -np.inf], np.float32)   # pi = (0, 1/4, 0, 3/4, 0)
    assert O.sample_row(row, O.F32, 0.0)[0] == 1          # never a token of probability 0
    assert O.sample_row(row, O.F32, 0.2499)[0] == 1
    assert O.sample_row(row, O.F32, 0.2501)[0] == 3
    assert O.sample_row(row, O.F32, 1.0 - 1e-16)[0] == 3
    assert O.sample_row(row, O.F32, 1.0)[0] == 3          # rounding fallback: last token with mass
    assert O.sample_row(np.array([np.nan, 0.0], np.float32), O.F32, 0.3)[0] == -1


def test_samples_follow_the_distribution():
    rng = np.random.default_rng(3)
    row = np.array([0.0, 1.0, -1.0, 2.0, 0.5, -3.0], np.float32)
    pi = softmax(row.astype(np.float64))
    n = 20000
    counts = np.zeros(6)
    for u in rng.random(n):
        counts[O.sample_row(row, O.F32, u)[0]] += 1
    chi = stats.chisquare(counts, pi * n)
    assert chi.pvalue > 1e-3, chi


def test_sampling_changes_tokens_not_decisions():
    rng = np.random.default_rng(5)
    B, L, V, gs = 2, 20, 12, 4
    p = O.OracleParams(B=B, L=L, V=V, conf_mode=O.CONF_RATIO, tau_max=3.0, tau_min=1.0, gamma=0.5, D=2, gen_start=gs)
    masked = np.zeros((B, L), bool)
    masked[:, gs:] = True
    logits = (rng.standard_normal((B, L, V)) * 1.5).astype(np.float32)
    u = rng.random((B, L))
    a = O.OracleState.init(p, np.zeros((B, L), np.int32), masked)
    b = O.OracleState.init(p, np.zeros((B, L), np.int32), masked)
    ra = a.step_full(logits)
    rb = b.step_full(logits, sample_u=u)
    assert np.array_equal(ra.commit, rb.commit) and np.array_equal(ra.token, rb.token)
    np.testing.assert_array_equal(a.masked, b.masked)
    pi = softmax(logits.astype(np.float64), -1)
    changed = 0
    for k in np.flatnonzero(rb.commit):
        pos = rb.active[k]
        bb, ii = divmod(int(pos), L)
        cdf = np.cumsum(pi[bb, ii])
        assert rb.final_token[k] == int(np.searchsorted(cdf, u[bb, ii], side="right"))
        assert b.tokens[bb, ii] == rb.final_token[k]
        assert rb.cdf_margin[k] >= 0
        changed += rb.final_token[k] != rb.token[k]
    assert changed > 0                                    # with these flat rows sampling does differ
    assert [t for (_, _, t) in b.commit_log] == rb.final_token[rb.commit].tolist()
    # u -> chosen so that every sample is the argmax: identical to argmax finalization
    assert np.all(np.isinf(rb.cdf_margin[~rb.commit]))


def test_peaked_distribution_samples_its_argmax():
    row = np.full(50, -40.0, np.float32)
    row[17] = 0.0
    for u in (1e-9, 0.3, 0.999999):      # (u = 0 would pick token 0, whose mass e^-40 is tiny but not zero)
        assert O.sample_row(row, O.F32, u)[0] == 17


def test_convention_at_the_upper_edge():
    # Inverse-CDF sampling takes the first token whose cumulative probability exceeds u; the
    # cumulative probability reaches 1 at the last token with a non-zero probability, so a number
    # that the rounded sum never exceeds (u = 1, not a valid draw from [0, 1)) selects that token,
    # and the largest binary32 number below 1 selects by the ordinary rule.
    V = 64
    row = np.full(V, -2.0, np.float32)
    row[7] = 30.0                      # p = 1 - 63 e^-32 ~ 1 - 8e-13
    row[50:] = -np.inf                 # zero-probability tail
    below_one = float(np.nextafter(np.float32(1.0), np.float32(0.0)))
    assert O.sample_row(row, O.F32, below_one)[0] == 7
    assert O.sample_row(row, O.F32, 1.0)[0] == 49
    assert O.sample_row(row, O.F32, 0.0)[0] == 0
    flat = np.zeros(V, np.float32)
    flat[40:] = -np.inf
    assert O.sample_row(flat, O.F32, below_one)[0] == 39 and O.sample_row(flat, O.F32, 1.0)[0] == 39
    # brute force on the explicit probability vector
    pi = O.softmax_row(row, O.F32)
    cum = np.cumsum(pi)
    assert int(np.argmax(cum > below_one)) == 7 and not (cum > 1.0).any()
    assert np.flatnonzero(pi > 0)[-1] == 49
