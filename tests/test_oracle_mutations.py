"""Do the pins bite?  Each case plants one plausible mistake IN THE ORACLE (on the CPU, in a
copy that is thrown away) and checks that at least one pin of tests/test_oracle_pins.py fails.
"""
import ctypes
import json
import os
import re
import subprocess

import numpy as np
import pytest

import test_oracle_pins as P
import test_oracle_rowwide_pins as R
import test_oracle_schedule_pins as S
import test_oracle_stability_pins as K
from oracle import jot_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PRINTED = json.load(open(os.path.join(ROOT, "tests", "golden", "paper_printed_values.json")))


def pin_battery():
    """A representative battery of pins as (name, thunk)."""
    b = [
        ("sum_to_one", lambda: [P.test_probabilities_sum_to_one_and_match_scipy(V) for V in (2, 16, 257)]),
        ("uniform", P.test_uniform_row),
        ("shift_inf", P.test_shift_invariance_and_minus_inf_is_deletion),
        ("bf16", P.test_bf16_is_widened_exactly),
        ("ratio_printed", lambda: P.test_ratio_closed_form_and_printed_logit_gaps(PRINTED)),
        ("top2_brute", lambda: [P.test_top2_and_argmax_brute_force_small_vocab(s) for s in range(20)]),
        ("dup_max", P.test_duplicated_maximum_gives_ratio_one_and_lowest_index),
        ("perm", P.test_vocabulary_permutation),
        ("wmax", lambda: P.test_w_max_closed_forms(PRINTED)),
        ("eq3_loop", lambda: [P.test_spatial_weight_against_double_loop(g, D) for g, D in ((0.5, 8), (0.9, 16), (1.0, 3))]),
        ("tau_special", lambda: P.test_threshold_special_cases(PRINTED)),
        ("all_masks", lambda: [P.test_every_mask_matches_brute_force(*a) for a in (
            (8, 16, O.CONF_RATIO, 7.0, 0.8, 0), (8, 5, O.CONF_MAXPROB, 0.6, 0.0, 0),
            (7, 16, O.CONF_PROBGAP, 0.5, 0.05, 0), (8, 9, O.CONF_RATIO, 3.0, 0.8, 3))]),
        ("tau_zero", lambda: [P.test_threshold_zero_finalizes_everything_in_one_step(m) for m in (0, 1, 2)]),
        ("tau_above_one", lambda: [P.test_threshold_above_one_finalizes_nothing(m) for m in (1, 2)]),
        ("invariants", lambda: [P.test_loop_invariants(b, O.CONF_RATIO, 20.0, 1.0) for b in (0, 4)]),
        ("monotone", P.test_monotonicity_in_tau_max_and_spatial_only_helps),
        ("simultaneous", P.test_simultaneous_update_within_a_step),
        ("sched_all_masks", lambda: [S.test_every_mask_matches_brute_force_with_schedule(*a) for a in (
            (7, 8, O.CONF_RATIO, 9.0, 0.8, 0, 1, 0.0), (6, 5, O.CONF_RATIO, 50.0, 0.8, 0, 0, 0.5),
            (8, 6, O.CONF_PROBGAP, 0.6, 0.05, 3, 1, 0.34))]),
        ("sched_default", S.test_no_schedule_is_the_default_and_k_zero_changes_nothing),
        ("sched_plain_topk", S.test_unreachable_threshold_degrades_to_plain_top_k_decoding),
        ("sched_fraction", S.test_fraction_one_reveals_everything_and_fraction_is_floored),
        ("sched_ties", S.test_equal_confidence_is_ranked_by_position_and_rows_without_softmax_are_skipped),
        ("sched_blocks", S.test_schedule_stays_inside_the_current_block_and_guarantees_termination),
        ("share_bound", P.test_committed_positions_leave_the_runner_up_a_small_head_to_head_share),
        ("rowwide_mean", R.test_mean_gap_and_all_or_nothing_per_row),
        ("rowwide_inclusive", R.test_threshold_is_inclusive_and_off_by_default),
        ("rowwide_or", R.test_rows_without_softmax_neither_count_nor_commit_and_rule_is_ored),
        ("rowwide_blocks", R.test_block_mode_applies_the_rule_to_the_current_block_only),
        ("kl_scipy", K.test_kl_matches_scipy_and_basic_properties),
        ("kl_two_token", K.test_two_token_closed_form_and_infinities),
        ("kl_rule", K.test_rule_needs_history_small_kl_and_enough_confidence),
        ("kl_or", K.test_rule_is_ored_with_the_others_and_off_by_default),
        ("kl_blocks", K.test_new_block_has_no_history),
        ("kl_history", K.test_history_means_the_step_just_before),
    ]
    return b


def failing_pins():
    failed = []
    for name, thunk in pin_battery():
        try:
            thunk()
        except Exception:
            failed.append(name)
    return failed


def test_battery_is_green_without_mutation():
    assert failing_pins() == []


# ---- mistakes in the numpy part ------------------------------------------------------------

def _sw_one_sided(resolved, gamma, D):
    B, L = resolved.shape
    res = resolved.astype(np.float64)
    w = np.zeros((B, L))
    for d in range(1, D + 1):
        if d < L:
            w[:, d:] += gamma ** d * res[:, :-d]
    return w


def _sw_short_window(resolved, gamma, D):
    return O.__dict__["_orig_spatial_weight"](resolved, gamma, max(D - 1, 0))


def _sw_wrong_power(resolved, gamma, D):
    B, L = resolved.shape
    res = resolved.astype(np.float64)
    w = np.zeros((B, L))
    for d in range(1, D + 1):
        if d < L:
            w[:, d:] += gamma ** (d - 1) * res[:, :-d]
            w[:, :-d] += gamma ** (d - 1) * res[:, d:]
    return w


def _thr_wrong_sign(resolved, p):
    phi = np.minimum(1.0, O.spatial_weight(resolved, p.gamma, p.D) / O.w_max(p.gamma, p.D)) if p.D else np.zeros(resolved.shape)
    return p.tau_max + (p.tau_max - p.tau_min) * phi, phi


def _conf_no_eps(p1, p2, mode, eps):
    return O.__dict__["_orig_confidence"](p1, p2, mode, 0.0 if mode == O.CONF_RATIO else eps)


def _conf_inverted(p1, p2, mode, eps):
    if mode == O.CONF_RATIO:
        return p2 / (p1 + eps)
    if mode == O.CONF_PROBGAP:
        return p1 + p2
    return p2


def _eligible_ignores_blocks(masked, p):
    return masked.copy()


PY_MUTATIONS = {
    "one_sided_window": ("spatial_weight", _sw_one_sided),
    "window_off_by_one": ("spatial_weight", _sw_short_window),
    "kernel_power_off_by_one": ("spatial_weight", _sw_wrong_power),
    "w_max_without_factor_two": ("w_max", lambda g, D: sum(g ** d for d in range(1, D + 1))),
    "threshold_sign": ("threshold", _thr_wrong_sign),
    "ratio_without_eps": ("confidence", _conf_no_eps),
    "confidence_inverted": ("confidence", _conf_inverted),
    "block_restriction_dropped": ("eligible", _eligible_ignores_blocks),
}


@pytest.mark.parametrize("name", sorted(PY_MUTATIONS))
def test_python_level_mistake_is_caught(name, monkeypatch):
    attr, repl = PY_MUTATIONS[name]
    monkeypatch.setitem(O.__dict__, "_orig_" + attr, getattr(O, attr))
    monkeypatch.setattr(O, attr, repl)
    assert failing_pins(), f"no pin notices: {name}"


def test_sequential_update_is_caught(monkeypatch):
    orig = O.OracleState.evaluate

    def evaluate_sequential(self, rows, *a, **kw):
        # decide positions one at a time, each seeing the commits made before it in the same step
        rec = orig(self, rows, *a, **kw)
        masked = self.masked.copy()
        flat = masked.reshape(-1)
        for k in range(rec.active.size):
            tau_all, phi_all = O.threshold(~masked, self.params)
            rec.tau[k] = tau_all.reshape(-1)[rec.active[k]]
            rec.commit[k] = rec.status[k] == 0 and rec.conf[k] >= rec.tau[k]
            if rec.commit[k]:
                flat[rec.active[k]] = False
        return rec

    monkeypatch.setattr(O.OracleState, "evaluate", evaluate_sequential)
    assert failing_pins()


def _sched_variant(kind):
    def _schedule(self, act, p1, ok, n_transfer, transfer_frac):
        p = self.params
        sched = np.zeros(act.size, bool)
        k_row = np.zeros(p.B, np.int64)
        if n_transfer is None and transfer_frac == 0.0:
            return sched, k_row
        n_transfer = np.zeros(p.B, np.int64) if n_transfer is None else np.asarray(n_transfer, np.int64)
        row_of = act // p.L
        if kind == "global_top_k":
            valid = np.flatnonzero(ok)
            k = int(n_transfer.sum()) + int(np.floor(transfer_frac * act.size))
            order = sorted(valid.tolist(), key=lambda j: (-p1[j], j))
            sched[order[:k]] = True
            return sched, k_row
        for b in range(p.B):
            mine = np.flatnonzero(row_of == b)
            valid = mine if kind == "selects_rows_without_softmax" else mine[ok[mine]]
            x = float(transfer_frac) * mine.size
            k = int(n_transfer[b]) + int(np.ceil(x) if kind == "fraction_rounded_up" else np.floor(x))
            k = max(0, min(k, valid.size))
            k_row[b] = k
            if kind == "least_confident_first":
                key = lambda j: (p1[j], j)
            elif kind == "ties_to_higher_index":
                key = lambda j: (-p1[j], -j)
            else:
                key = lambda j: (-np.nan_to_num(p1[j], nan=2.0), j)
            sched[sorted(valid.tolist(), key=key)[:k]] = True
        return sched, k_row
    return _schedule


@pytest.mark.parametrize("kind", ["least_confident_first", "ties_to_higher_index", "global_top_k",
                                  "fraction_rounded_up", "selects_rows_without_softmax"])
def test_schedule_mistake_is_caught(kind, monkeypatch):
    monkeypatch.setattr(O.OracleState, "_schedule", _sched_variant(kind))
    assert failing_pins(), f"no pin notices: {kind}"


def _rowwide_variant(kind):
    def _rowwide(self, act, m1, m2, ok, global_gap):
        p = self.params
        rowwide = np.zeros(act.size, bool)
        gap_row = np.full(p.B, np.nan)
        if global_gap is None:
            return rowwide, gap_row
        row_of = act // p.L
        if kind == "one_statistic_for_the_whole_batch":
            mine = np.flatnonzero(ok)
            g = float(np.mean(m1[mine] - m2[mine])) if mine.size else np.nan
            gap_row[:] = g
            if g >= global_gap:
                rowwide[mine] = True
            return rowwide, gap_row
        for b in range(p.B):
            mine = np.flatnonzero((row_of == b) & (ok if kind != "counts_rows_without_softmax" else True))
            if mine.size:
                d = m1[mine] - m2[mine]
                if kind == "largest_gap_instead_of_mean":
                    gap_row[b] = float(np.max(d))
                elif kind == "probability_gap":
                    gap_row[b] = float(np.mean(1 - np.exp(-d)))
                else:
                    gap_row[b] = float(np.nanmean(d))
                fire = gap_row[b] > global_gap if kind == "strict_comparison" else gap_row[b] >= global_gap
                if fire:
                    rowwide[mine] = True
        return rowwide, gap_row
    return _rowwide


@pytest.mark.parametrize("kind", ["one_statistic_for_the_whole_batch", "largest_gap_instead_of_mean",
                                  "probability_gap", "strict_comparison", "counts_rows_without_softmax"])
def test_rowwide_mistake_is_caught(kind, monkeypatch):
    monkeypatch.setattr(O.OracleState, "_rowwide", _rowwide_variant(kind))
    assert failing_pins(), f"no pin notices: {kind}"


def _stable_variant(kind):
    def _stable(self, act, rows, prev_rows, p1, ok, kl_threshold, kl_min_prob):
        stable = np.zeros(act.size, bool)
        kl = np.full(act.size, np.nan)
        if kl_threshold is None:
            return stable, kl
        had_prev = self.last_ok_step.reshape(-1)[act] == self.step_index
        if kind == "no_history_needed":
            had_prev = np.ones(act.size, bool)
        if kind == "any_earlier_step_counts_as_history":
            had_prev = self.last_ok_step.reshape(-1)[act] >= 0
        for k in np.flatnonzero(ok & had_prev):
            kl[k] = O.kl_row(rows[k], prev_rows[k], self.params.dtype)
        with np.errstate(invalid="ignore"):
            small = kl < kl_threshold if kind == "strict_comparison" else kl <= kl_threshold
            sure = np.ones(act.size, bool) if kind == "confidence_not_checked" else p1 >= kl_min_prob
            stable = ok & had_prev & small & sure
        return stable, kl
    return _stable


@pytest.mark.parametrize("kind", ["no_history_needed", "any_earlier_step_counts_as_history", "strict_comparison",
                                  "confidence_not_checked"])
def test_stability_mistake_is_caught(kind, monkeypatch):
    monkeypatch.setattr(O.OracleState, "_stable", _stable_variant(kind))
    assert failing_pins(), f"no pin notices: {kind}"


def test_and_instead_of_or_is_caught(monkeypatch):
    orig = O.OracleState.evaluate

    def evaluate_and(self, rows, n_transfer=None, transfer_frac=0.0, *a, **kw):
        rec = orig(self, rows, n_transfer, transfer_frac, *a, **kw)
        if n_transfer is not None or transfer_frac:
            rec.commit = rec.exit & rec.sched
        return rec

    monkeypatch.setattr(O.OracleState, "evaluate", evaluate_and)
    assert failing_pins()


# ---- mistakes in the C part ---------------------------------------------------------------

C_MUTATIONS = {
    "last_index_on_ties": (r"if \(x > best\) \{", "if (x >= best) {"),
    "second_max_includes_the_winner": (r"if \(v == arg\)\s*\n\s*continue;", ""),
    "no_max_subtraction": (r"sum \+= exp\(widen\(row, dtype, v\) - best\);", "sum += exp(widen(row, dtype, v));"),
    "sum_skips_last_entry": (r"for \(int32_t v = 0; v < V; v\+\+\)\n        sum \+=", "for (int32_t v = 0; v < V - 1; v++)\n        sum +="),
    "bf16_shift": (r"<< 16;", "<< 15;"),
    "kl_reversed": (r"kl \+= pv \* \(\(x - lse\) - \(y - plse\)\);", "kl += pv * ((y - plse) - (x - lse));"),
    "kl_without_normalizers": (r"kl \+= pv \* \(\(x - lse\) - \(y - plse\)\);", "kl += pv * (x - y);"),
    "kl_weighted_by_previous": (r"const double pv = exp\(x - m1\) / S;", "const double pv = exp(y - pm1) / pS;"),
}


@pytest.mark.parametrize("name", sorted(C_MUTATIONS))
def test_c_level_mistake_is_caught(name, monkeypatch, tmp_path):
    pat, repl = C_MUTATIONS[name]
    src = open(os.path.join(ROOT, "oracle", "jot_oracle.c")).read()
    mutated, n = re.subn(pat, repl, src)
    assert n >= 1, "mutation pattern no longer matches the oracle source"
    cfile, lib = tmp_path / "mut.c", tmp_path / "libmut.so"
    cfile.write_text(mutated)
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", str(lib), str(cfile), "-lm"])
    good = O._load()
    mut = ctypes.CDLL(str(lib))
    for fn in ("jot_oracle_row_stats", "jot_oracle_softmax_row", "jot_oracle_sample_row", "jot_oracle_kl_row",
               "jot_oracle_kl_rows"):
        getattr(mut, fn).argtypes = getattr(good, fn).argtypes
        getattr(mut, fn).restype = getattr(good, fn).restype
    monkeypatch.setattr(O, "_lib", mut)
    assert failing_pins(), f"no pin notices: {name}"
