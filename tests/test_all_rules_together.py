"""Every optional rule of a step at once, on random small problems: early exit (Eq. 6) + transfer
schedule + row-wide commit + KL stability + sampled tokens, random hyper-parameters, both element
types, block mode on and off.  The inputs are made well posed on the CPU (thresholds of the two
extra rules are placed in the widest gap of the statistics they are compared with; logits are
raised and uniform numbers redrawn where a decision would sit on an edge), then the library is
compared with the oracle step by step.  The CPU half (input preparation + oracle invariants)
also runs on its own without a GPU."""
import numpy as np
import pytest

from gen.bf16 import bf16_bits_to_f32, f32_to_bf16_bits
from harness import GUARD, GUARD_KL, GUARD_U, too_close
from oracle import jot_oracle as O
from test_gpu_edge_cases import as_rows, clear_guard_band, drifting_logits, to_device

SEEDS = list(range(40))
STEPS = 6


def widest_gap_midpoint(values, lo_q=0.15, hi_q=0.85):
    """A threshold in the widest gap between neighbouring values of the central part of `values`."""
    v = np.unique(values[np.isfinite(values)])
    if v.size < 2:
        return None
    a = int(v.size * lo_q)
    b = min(max(int(v.size * hi_q), a + 1), v.size - 1)
    w = v[a:b + 1]
    k = int(np.argmax(np.diff(w)))
    return float(np.float32((w[k] + w[k + 1]) / 2))


def random_problem(seed):
    rng = np.random.default_rng(7000 + seed)
    B = int(rng.integers(1, 5))
    L = int(rng.integers(10, 160))
    V = int(rng.choice([17, 257, 1003, 5000]))
    gs = int(rng.integers(0, L // 3 + 1))
    dtype = int(rng.choice([O.F32, O.BF16]))
    mode = int(rng.integers(0, 3))
    tau_max, tau_min = {O.CONF_RATIO: (60.0, 1.5), O.CONF_MAXPROB: (0.97, 0.3), O.CONF_PROBGAP: (0.95, 0.2)}[mode]
    p = O.OracleParams(B=B, L=L, V=V, dtype=dtype, conf_mode=mode, tau_max=float(np.float32(tau_max)),
                       tau_min=float(np.float32(tau_min)), gamma=float(np.float32(rng.uniform(0.3, 1.0))),
                       D=int(rng.integers(0, 17)), eps=float(np.float32(1e-12)), gen_start=gs,
                       block_size=int(rng.choice([0, 0, 7, 32])))
    masked = np.zeros((B, L), bool)
    masked[:, gs:] = rng.random((B, L - gs)) < 0.9
    tokens = rng.integers(0, V, (B, L)).astype(np.int32)
    seq = drifting_logits(rng, B, L, V, STEPS, scale=2.0, drift=0.1 if dtype == O.F32 else 0.3)
    if dtype == O.BF16:
        seq = [bf16_bits_to_f32(f32_to_bf16_bits(x)).reshape(x.shape) for x in seq]
    return rng, p, tokens, masked, seq


def prepare_step(st, logits, prev_logits, rng):
    """Chooses this step's options and makes every decision well posed.  Modifies `logits` in
    place (raised argmax logits).  Returns (rec, options) with the step NOT yet applied."""
    p = st.params
    nt = rng.integers(0, 3, p.B).astype(np.int32) if rng.random() < 0.6 else None
    frac = float(np.float32(rng.choice([0.0, 0.1, 0.25])))
    clear_guard_band(st, logits, nt, frac)
    act = st.active_list()
    flat = logits.reshape(p.B * p.L, p.V)
    rows = as_rows(flat[act], p.dtype)
    before = logits if prev_logits is None else prev_logits
    prev_rows = as_rows(before.reshape(p.B * p.L, p.V)[act], p.dtype)
    probe = st.evaluate(rows, nt, frac, None, 1e30, prev_rows, 0.0, 0.0)
    tau_kl = widest_gap_midpoint(probe.kl)
    if tau_kl is None:
        tau_kl = 0.05
    cand = np.isfinite(probe.kl) & (probe.kl <= tau_kl)
    min_prob = widest_gap_midpoint(probe.p1[cand]) if rng.random() < 0.5 else None
    kl = (tau_kl, 0.0 if min_prob is None else min_prob)
    # row-wide rule: mostly no row or only the most decided row clears the threshold, so that decodes last
    means = np.sort(probe.gap_row[np.isfinite(probe.gap_row)])
    pick = rng.random()
    if means.size == 0:
        gg = 3.0
    elif pick < 0.45 or (means.size < 2 and pick < 0.9):
        gg = float(np.float32(means[-1] + 0.5))                           # nobody
    elif pick < 0.9:
        gg = float(np.float32((means[-1] + means[-2]) / 2))               # the most decided row only
    else:
        gg = float(np.float32(means[0] - 0.5))                            # everybody
    u = rng.random((p.B, p.L), dtype=np.float32)
    for _ in range(100):
        rec = st.evaluate(rows, nt, frac, u, gg, prev_rows, kl[0], kl[1])
        edge = np.flatnonzero(rec.commit & (rec.cdf_margin < GUARD_U))
        if edge.size == 0:
            break
        for k in edge:
            u.reshape(-1)[act[k]] = rng.random(dtype=np.float32)
    else:
        raise AssertionError("could not move the uniform numbers off the CDF edges")
    assert too_close(rec, p.L, kl).size == 0
    assert not np.any(np.abs(rec.gap_row - gg) < GUARD * max(1.0, abs(gg)))
    return rec, dict(n_transfer=nt, transfer_frac=frac, uniforms=u, global_gap=gg, kl=kl)


@pytest.mark.parametrize("seed", SEEDS)
def test_inputs_are_well_posed_and_the_oracle_combines_the_rules_by_or(seed):
    rng, p, tokens, masked, seq = random_problem(seed)
    st = O.OracleState.init(p, tokens, masked)
    prev = None
    fired = np.zeros(4, int)
    for logits in seq:
        before_masked = st.masked.copy()
        rec, opt = prepare_step(st, logits, prev, rng)
        assert np.array_equal(rec.commit, rec.exit | rec.sched | rec.rowwide | rec.stable)
        fired += [rec.exit.sum(), rec.sched.sum(), rec.rowwide.sum(), rec.stable.sum()]
        st.apply(rec)
        gone = before_masked & ~st.masked
        assert gone.sum() == rec.commit.sum() and not (st.masked & ~before_masked).any()
        sampled = rec.final_token[rec.commit]
        assert np.array_equal(st.tokens.reshape(-1)[rec.active[rec.commit]], sampled)
        prev = logits
    assert fired.sum() > 0


@pytest.mark.gpu
@pytest.mark.parametrize("seed", SEEDS)
def test_all_rules_together_on_the_gpu(seed):
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.fail("this test needs the MI355X; there is no CPU fallback")
    import gpu_harness as G
    import paper_2602_11133_amd as J
    rng, p, tokens, masked, seq = random_problem(seed)
    print(f"[all rules] seed={seed} B={p.B} L={p.L} V={p.V} dtype={p.dtype} mode={p.conf_mode} D={p.D} "
          f"gamma={p.gamma:.3f} block={p.block_size} gen_start={p.gen_start}", flush=True)
    esz = 4 if p.dtype == O.F32 else 2
    align = 16 // esz
    stride_l = (p.V + align - 1) // align * align
    jp = J.JotParams(B=p.B, L=p.L, V=p.V, dtype=p.dtype, conf_mode=p.conf_mode, tau_max=p.tau_max,
                     tau_min=p.tau_min, gamma=p.gamma, D=p.D, eps=p.eps, gen_start=p.gen_start,
                     block_size=p.block_size)
    st = O.OracleState.init(p, tokens, masked)
    g = G.GpuJot(jp, tokens, masked)
    tol = 1e-5 if p.dtype == O.F32 else 2e-3
    prev = prev_dev = None
    for n, logits in enumerate(seq, 1):
        rec, opt = prepare_step(st, logits, prev, rng)
        act = st.active_list()
        st.apply(rec)
        dev = to_device(logits, p.dtype, stride_l)
        g.step(dev, stride_b=p.L * stride_l, stride_l=stride_l, prev_logits=dev if prev_dev is None else prev_dev,
               **opt)
        G.compare_step(g.last(), rec, act, tol)
        np.testing.assert_array_equal(g.tokens(), st.tokens)
        np.testing.assert_array_equal(g.masked(), st.masked)
        np.testing.assert_array_equal(g.active_list(), st.active_list().astype(np.int32))
        assert J.jot_anomaly_count(g.h) == st.anomalies and J.jot_step_index(g.h) == n
        prev, prev_dev = logits, dev
    np.testing.assert_array_equal(g.commit_log(), np.array(st.commit_log, np.int32).reshape(-1, 3))
    g.close()
