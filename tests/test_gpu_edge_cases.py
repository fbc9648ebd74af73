"""GPU edge cases against the oracle: ragged vocabularies and strides, rows split into pieces,
ties across pieces, -inf / NaN / +inf logits, empty and tiny canvases, many batch rows,
extreme window radii, determinism."""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from gen.bf16 import bf16_bits_to_f32, f32_to_bf16_bits  # noqa: E402
from harness import GUARD, GUARD_KL, GUARD_U, too_close  # noqa: E402
from oracle import jot_oracle as O  # noqa: E402


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the MI355X; there is no CPU fallback")
    import gpu_harness
    return gpu_harness


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def clear_guard_band(st: O.OracleState, logits: np.ndarray, n_transfer=None, frac=0.0):
    """Adjust the INPUT until no decision of the step is ill posed (confidence within the guard
    band of its threshold, or a near-tie at the edge of the schedule's selection): raise that
    row's current argmax logit by one."""
    p = st.params
    flat = logits.reshape(p.B * p.L, p.V)
    for _ in range(100):
        act = st.active_list()
        rec = st.evaluate(as_rows(flat[act], p.dtype), n_transfer, frac)
        near = np.zeros(act.size, bool)
        near[too_close(rec, p.L)] = True
        if not near.any():
            return
        for k in np.flatnonzero(near):
            v = np.float32(flat[act[k], rec.token[k]] + 1.0)
            if p.dtype == O.BF16:
                v = bf16_bits_to_f32(f32_to_bf16_bits(np.array([v], np.float32)))[0]
                if v == flat[act[k], rec.token[k]]:
                    v = np.float32(v * 2 if v > 0 else 1.0)
            flat[act[k], rec.token[k]] = v
    raise AssertionError("guard band not cleared")


def as_rows(x, dtype):
    return np.ascontiguousarray(x, np.float32) if dtype == O.F32 else f32_to_bf16_bits(np.asarray(x, np.float32))


def to_device(logits: np.ndarray, dtype: int, stride_l: int):
    """[B, L, V] host array -> device tensor with row stride stride_l >= V (padding = NaN)."""
    B, L, V = logits.shape
    tdt = torch.float32 if dtype == O.F32 else torch.bfloat16
    dev = torch.full((B, L, stride_l), float("nan"), dtype=tdt, device="cuda")
    dev[:, :, :V] = torch.from_numpy(logits).to("cuda").to(tdt)
    return dev


def check_case(gpu, p: O.OracleParams, tokens, masked, logit_seq, stride_pad=0, tol=None, clear=True,
               schedule=None, uniforms=None, global_gap=None, kl=None, compact=False):
    """compact: give the library a [n_examined, stride] tensor with the examined rows in list order.
    kl: optional list, per step, of (kl_threshold, kl_min_prob) or None: the KL stability rule
    against the logits of the step before.  schedule: optional list of (n_transfer, frac) per step.  uniforms: optional list of [B, L]
    float32 arrays per step (sampling-based finalization); numbers that fall within GUARD_U of
    an edge of the chosen token's CDF interval are redrawn here (they are inputs)."""
    import paper_2602_11133_amd as J
    esz = 4 if p.dtype == O.F32 else 2
    align = 16 // esz
    stride_l = (p.V + align - 1) // align * align + stride_pad * align
    jp = J.JotParams(B=p.B, L=p.L, V=p.V, dtype=p.dtype, conf_mode=p.conf_mode, tau_max=p.tau_max,
                     tau_min=p.tau_min, gamma=p.gamma, D=p.D, eps=p.eps, gen_start=p.gen_start,
                     block_size=p.block_size)
    # the library holds gamma, tau and eps as binary32: give the oracle the same real numbers
    p = O.OracleParams(**{**p.__dict__, "gamma": float(np.float32(p.gamma)), "tau_max": float(np.float32(p.tau_max)),
                          "tau_min": float(np.float32(p.tau_min)), "eps": float(np.float32(p.eps))})
    st = O.OracleState.init(p, tokens, masked)
    g = gpu.GpuJot(jp, tokens, masked)
    tol = tol or (1e-5 if p.dtype == O.F32 else 2e-3)
    np.testing.assert_array_equal(g.active_list(), st.active_list().astype(np.int32))
    prev_logits = prev_dev = None
    for n, logits in enumerate(logit_seq, 1):
        logits = np.array(logits, np.float32)
        if p.dtype == O.BF16:
            logits = bf16_bits_to_f32(f32_to_bf16_bits(logits)).reshape(logits.shape)
        nt, frac = schedule[n - 1] if schedule else (None, 0.0)
        frac = float(np.float32(frac))
        gg = None if global_gap is None else float(np.float32(global_gap[n - 1]))
        if clear:
            clear_guard_band(st, logits, nt, frac)
            if p.dtype == O.BF16:
                assert np.array_equal(bf16_bits_to_f32(f32_to_bf16_bits(logits)).reshape(logits.shape), logits)
        act = st.active_list()
        u = None
        if uniforms is not None:
            u = np.array(uniforms[n - 1], np.float32)
            redraw = np.random.default_rng(1000 + n)
            for _ in range(100):
                probe = st.evaluate(as_rows(logits.reshape(p.B * p.L, p.V)[act], p.dtype), nt, frac, u, gg)
                edge = np.flatnonzero(probe.commit & (probe.cdf_margin < GUARD_U))
                if edge.size == 0:
                    break
                for k in edge:
                    u.reshape(-1)[act[k]] = redraw.random(dtype=np.float32)
        klo = kl[n - 1] if kl else None
        kl_kw = {}
        if klo is not None:
            klo = (float(np.float32(klo[0])), float(np.float32(klo[1])))
            before = logits if prev_logits is None else prev_logits
            kl_kw = dict(prev_rows=as_rows(before.reshape(p.B * p.L, p.V)[act], p.dtype), kl_threshold=klo[0],
                         kl_min_prob=klo[1])
        rec = st.step(as_rows(logits.reshape(p.B * p.L, p.V)[act], p.dtype), nt, frac, u, gg, **kl_kw)
        if klo is not None:
            assert too_close(rec, p.L, klo).size == 0 or clear, "a divergence sits on its threshold"
            fin = np.isfinite(rec.kl)
            assert not np.any(np.abs(rec.kl[fin] - klo[0]) < GUARD_KL * max(1.0, klo[0])), "a divergence sits on its threshold"
        if gg is not None:
            assert np.all(~(np.abs(rec.gap_row - gg) < GUARD * max(1.0, abs(gg)))), "row mean sits on the threshold"
        dev = to_device(logits, p.dtype, stride_l)
        if compact:
            small = gpu.gather_compact(dev[:, :, :p.V].contiguous(), J.jot_active_list(g.h), g.active_count(),
                                       pad_elems=stride_l - p.V)
            g.step(small, n_transfer=nt, transfer_frac=frac, uniforms=u, global_gap=gg, compact=True)
        else:
            g.step(dev, stride_b=p.L * stride_l, stride_l=stride_l, n_transfer=nt, transfer_frac=frac, uniforms=u,
                   global_gap=gg, kl=klo, prev_logits=dev if prev_dev is None else prev_dev)
        prev_logits, prev_dev = logits, dev
        gpu.compare_step(g.last(), rec, act, tol)
        np.testing.assert_array_equal(g.tokens(), st.tokens)
        np.testing.assert_array_equal(g.masked(), st.masked)
        np.testing.assert_array_equal(g.active_list(), st.active_list().astype(np.int32))
        assert g.active_count() == st.active_count()
        assert J.jot_anomaly_count(g.h) == st.anomalies
        assert J.jot_step_index(g.h) == n
    want = np.array(st.commit_log, np.int32).reshape(-1, 3)
    np.testing.assert_array_equal(g.commit_log(), want)
    out = (g.tokens(), g.masked(), g.commit_log(), g.last())
    g.close()
    return out


def random_case(seed, B, L, V, gs, dtype=O.F32, steps=3, scale=3.0, **kw):
    rng = np.random.default_rng(seed)
    p = O.OracleParams(B=B, L=L, V=V, dtype=dtype, gen_start=gs, **kw)
    masked = np.zeros((B, L), bool)
    masked[:, gs:] = rng.random((B, L - gs)) < 0.85
    tokens = rng.integers(0, V, (B, L)).astype(np.int32)
    seq = []
    target = rng.integers(0, V, (B, L))
    for n in range(steps):
        lg = (rng.standard_normal((B, L, V)) * scale).astype(np.float32)
        boost = rng.uniform(0, 14, (B, L)).astype(np.float32) * (n + 1) / steps
        np.put_along_axis(lg, target[..., None], boost[..., None] + 6.0, -1)
        seq.append(lg)
    return p, tokens, masked, seq


@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
@pytest.mark.parametrize("V", [2, 3, 7, 8, 9, 1003, 2048, 2049, 8191, 20011])
def test_ragged_vocabulary_and_padded_strides(gpu, dtype, V):
    say(f"[edge] ragged V={V} dtype={dtype}")
    p, tokens, masked, seq = random_case(V, B=2, L=37, V=V, gs=5, dtype=dtype, conf_mode=O.CONF_RATIO,
                                         tau_max=20.0, tau_min=1.0, gamma=0.5, D=4)
    check_case(gpu, p, tokens, masked, seq, stride_pad=1)


@pytest.mark.parametrize("mode,tau_max,tau_min", [(O.CONF_RATIO, 90.0, 1.0), (O.CONF_MAXPROB, 0.9, 0.0),
                                                   (O.CONF_PROBGAP, 0.8, 0.1)])
@pytest.mark.parametrize("gamma,D", [(0.5, 8), (0.3, 4), (0.9, 16), (1.0, 32), (0.7, 1), (0.5, 0)])
def test_spatial_parameters(gpu, mode, tau_max, tau_min, gamma, D):
    say(f"[edge] spatial mode={mode} gamma={gamma} D={D}")
    p, tokens, masked, seq = random_case(D * 7 + mode, B=3, L=131, V=512, gs=40, conf_mode=mode,
                                         tau_max=tau_max, tau_min=tau_min, gamma=gamma, D=D, steps=4)
    check_case(gpu, p, tokens, masked, seq)


@pytest.mark.parametrize("block", [1, 5, 32, 64, 500])
def test_block_mode(gpu, block):
    say(f"[edge] block={block}")
    p, tokens, masked, seq = random_case(block, B=4, L=200, V=300, gs=30, conf_mode=O.CONF_MAXPROB,
                                         tau_max=0.7, tau_min=0.0, gamma=0.5, D=8, block_size=block, steps=8)
    masked[1, 10:20] = True          # masked positions inside the prompt region too
    check_case(gpu, p, tokens, masked, seq)


@pytest.mark.parametrize("block", [0, 1, 32, 500])
def test_single_row_canvas_longer_than_a_workgroup(gpu, block):
    # one batch row: decisions, compaction and the closing of the step run in one workgroup of one
    # launch, which walks the row in several chunks and, in block mode, looks for the block first
    say(f"[edge] single row, block={block}")
    p, tokens, masked, seq = random_case(40 + block, B=1, L=700, V=300, gs=45, conf_mode=O.CONF_MAXPROB,
                                         tau_max=0.7, tau_min=0.0, gamma=0.5, D=8, block_size=block, steps=8)
    masked[0, 10:20] = True          # masked positions inside the prompt region too
    check_case(gpu, p, tokens, masked, seq)


def test_rows_split_into_pieces_with_ties_across_pieces(gpu):
    # few examined rows and a long vocabulary: each row is cut into several pieces that are
    # merged afterwards; equal maxima sit in different pieces
    B, L, V = 1, 6, 100_003
    rng = np.random.default_rng(9)
    p = O.OracleParams(B=B, L=L, V=V, dtype=O.F32, conf_mode=O.CONF_RATIO, tau_max=5.0, tau_min=0.5,
                       gamma=0.5, D=2, gen_start=1)
    masked = np.array([[False, True, True, True, True, True]])
    tokens = np.zeros((B, L), np.int32)
    lg = rng.standard_normal((B, L, V)).astype(np.float32)
    lg[0, 1, [99_999, 50_000, 123]] = 9.0          # three-way tie: index 123 wins, m2 = m1
    lg[0, 2, 77_777] = 12.0                        # clear winner in a late piece
    lg[0, 2, 3] = 11.0                             # runner-up in the first piece
    lg[0, 3, V - 1] = 15.0                         # winner in the ragged tail
    lg[0, 4, :] = -np.inf
    lg[0, 4, 60_000] = 0.0                         # a single finite entry: p1 = 1, p2 = 0
    lg[0, 5, 0] = 10.0
    lg[0, 5, 1] = 10.0                             # tie inside one vector
    toks, msk, log, last = check_case(gpu, p, tokens, masked, [lg], clear=False)
    assert last["token"].tolist() == [123, 77_777, V - 1, 60_000, 0]
    assert last["p2"][3] == 0.0 and last["p1"][3] == 1.0


@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
def test_rows_without_softmax_and_minus_inf_entries(gpu, dtype):
    B, L, V = 2, 12, 5000
    rng = np.random.default_rng(4)
    p = O.OracleParams(B=B, L=L, V=V, dtype=dtype, conf_mode=O.CONF_MAXPROB, tau_max=0.5, tau_min=0.0,
                       gamma=0.5, D=3, gen_start=2)
    masked = np.zeros((B, L), bool)
    masked[:, 2:] = True
    lg = rng.standard_normal((B, L, V)).astype(np.float32)
    lg[:, :, 17] = 14.0                              # everything would finalize ...
    lg[0, 3, 4000] = np.nan                          # ... except rows without a softmax
    lg[0, 4, 99] = np.inf
    lg[0, 5, :] = -np.inf
    lg[1, 6, ::2] = -np.inf                          # masked-out tokens are fine
    lg[1, 7, :] = -200.0                             # very negative everywhere: shift invariance
    lg[1, 7, 17] = -190.0
    lg[1, 8, :] = 3.0e4 if dtype == O.F32 else 3.0e4  # huge but finite
    lg[1, 8, 17] = 3.0e4 + 64
    toks, msk, log, last = check_case(gpu, p, np.zeros((B, L), np.int32), masked, [lg, lg], clear=False)
    assert msk[0, 3] and msk[0, 4] and msk[0, 5]
    assert not msk[1, 6] and not msk[1, 7] and not msk[1, 8]


def test_empty_and_tiny_canvases(gpu):
    import paper_2602_11133_amd as J
    # nothing masked: zero examined positions, steps are no-ops
    p = O.OracleParams(B=2, L=5, V=16, gen_start=5)
    tokens = np.arange(10, dtype=np.int32).reshape(2, 5)
    masked = np.zeros((2, 5), bool)
    lg = np.zeros((2, 5, 16), np.float32)
    toks, msk, log, last = check_case(gpu, p, tokens, masked, [lg, lg], clear=False)
    assert log.shape == (0, 3) and last["active"].size == 0
    np.testing.assert_array_equal(toks, tokens)
    # one position, two tokens
    p = O.OracleParams(B=1, L=1, V=2, conf_mode=O.CONF_RATIO, tau_max=3.0, tau_min=1.0, D=8)
    lg = np.array([[[0.0, 2.0]]], np.float32)
    toks, msk, log, last = check_case(gpu, p, np.zeros((1, 1), np.int32), np.ones((1, 1), bool), [lg])
    assert toks[0, 0] == 1 and log.tolist() == [[1, 0, 1]]


def test_many_batch_rows(gpu):
    # more batch rows than threads in a workgroup: the prefix over rows takes several strides
    p, tokens, masked, seq = random_case(31, B=700, L=9, V=40, gs=2, conf_mode=O.CONF_MAXPROB,
                                         tau_max=0.6, tau_min=0.0, gamma=0.5, D=2, steps=3)
    check_case(gpu, p, tokens, masked, seq)


def test_long_rows_cross_word_boundaries(gpu):
    # L not a multiple of 64 or 256; windows straddle 64-bit words of the mask image
    p, tokens, masked, seq = random_case(12, B=2, L=333, V=64, gs=61, conf_mode=O.CONF_RATIO,
                                         tau_max=40.0, tau_min=1.0, gamma=0.9, D=32, steps=5)
    check_case(gpu, p, tokens, masked, seq)


def test_bf16_ties_are_broken_by_lowest_index(gpu):
    B, L, V = 1, 40, 30_000
    rng = np.random.default_rng(8)
    p = O.OracleParams(B=B, L=L, V=V, dtype=O.BF16, conf_mode=O.CONF_RATIO, tau_max=0.9, tau_min=0.5,
                       gamma=0.5, D=8, gen_start=0)
    masked = np.ones((B, L), bool)
    lg = np.round(rng.standard_normal((B, L, V)) * 2).astype(np.float32)     # integers: many ties at the top
    toks, msk, log, last = check_case(gpu, p, np.zeros((B, L), np.int32), masked, [lg], clear=False)
    assert np.array_equal(last["token"], np.argmax(lg[0], -1))


def test_two_runs_are_bitwise_identical(gpu):
    p, tokens, masked, seq = random_case(77, B=3, L=90, V=9000, gs=10, dtype=O.BF16, conf_mode=O.CONF_RATIO,
                                         tau_max=30.0, tau_min=1.0, gamma=0.5, D=8, steps=4)
    a = check_case(gpu, p, tokens, masked, seq)
    b = check_case(gpu, p, tokens, masked, seq)
    for x, y in zip(a[:3], b[:3]):
        np.testing.assert_array_equal(x, y)
    for k in a[3]:
        np.testing.assert_array_equal(a[3][k].view(np.uint8), b[3][k].view(np.uint8))


# --------------------------------------------------------------------------- transfer schedule

@pytest.mark.parametrize("mode,tau_max,tau_min", [(O.CONF_RATIO, 90.0, 1.0), (O.CONF_MAXPROB, 0.9, 0.0),
                                                   (O.CONF_RATIO, 1e9, 1e9)])
def test_schedule_counts_and_fractions(gpu, mode, tau_max, tau_min):
    say(f"[edge] schedule mode={mode} tau_max={tau_max}")
    p, tokens, masked, seq = random_case(41 + mode, B=5, L=150, V=300, gs=20, conf_mode=mode, tau_max=tau_max,
                                         tau_min=tau_min, gamma=0.5, D=8, steps=7)
    sched = [([1, 0, 3, 200, 7], 0.0), (None, 0.25), ([0, 0, 0, 0, 0], 0.0), ([2, 2, 2, 2, 2], 0.1),
             ([1, 1, 1, 1, 1], 0.0), (None, 0.5), (None, 1.0)]
    toks, msk, log, last = check_case(gpu, p, tokens, masked, seq, schedule=sched)
    assert not msk.any()                      # the last step (fraction 1) reveals everything


def test_schedule_in_block_mode(gpu):
    p, tokens, masked, seq = random_case(43, B=3, L=100, V=200, gs=12, conf_mode=O.CONF_RATIO, tau_max=30.0,
                                         tau_min=1.0, gamma=0.5, D=8, block_size=16, steps=12)
    check_case(gpu, p, tokens, masked, seq, schedule=[([2, 1, 3], 0.0)] * 12)


def test_schedule_with_equal_confidences_and_rows_without_softmax(gpu):
    B, L, V = 2, 300, 64
    p = O.OracleParams(B=B, L=L, V=V, dtype=O.F32, conf_mode=O.CONF_MAXPROB, tau_max=2.0, tau_min=1.5, D=0)
    lg = np.zeros((B, L, V), np.float32)
    lg[:, :, 5] = 4.0                          # identical rows: every p1 is the same bit pattern
    lg[0, 7, 9] = np.nan
    lg[0, 8, :] = -np.inf
    lg[1, 100:110, 6] = 6.0                    # ten rows with a larger p1 ...
    lg[1, 200:205, 5] = 9.0                    # ... and five with a still larger one
    masked = np.ones((B, L), bool)
    sched = [([3, 7], 0.0), ([290, 0], 0.0), ([1000, 1000], 0.0)]
    toks, msk, log, last = check_case(gpu, p, np.zeros((B, L), np.int32), masked, [lg, lg, lg], clear=False,
                                      schedule=sched)
    assert log[:3, 1].tolist() == [0, 1, 2]                       # equal confidence: lowest positions first
    assert sorted(log[3:10, 1].tolist()) == [L + 100, L + 101, L + 200, L + 201, L + 202, L + 203, L + 204]
    assert msk[0, 7] and msk[0, 8] and msk.sum() == 2             # rows without a softmax are never revealed


def test_schedule_on_a_long_row(gpu):
    # several 256-wide chunks per row in the selection kernel, L not a multiple of anything
    p, tokens, masked, seq = random_case(47, B=2, L=2500, V=48, gs=3, conf_mode=O.CONF_MAXPROB, tau_max=0.95,
                                         tau_min=0.0, gamma=0.5, D=8, steps=3)
    check_case(gpu, p, tokens, masked, seq, schedule=[([1, 1999], 0.0), (None, 0.37), ([5, 5], 0.5)])


# --------------------------------------------------------------------------- sampling-based finalization

@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
@pytest.mark.parametrize("V", [2, 9, 1003, 8192, 8200, 40_003, 600_001])     # the last: more batches than the kernel keeps totals of
def test_sampled_tokens(gpu, dtype, V):
    say(f"[edge] sampling V={V} dtype={dtype}")
    # flat-ish rows (scale 1.5) so that samples differ from the argmax; tau = 0: everything is finalized
    rng = np.random.default_rng(V + dtype)
    B, L = 2, 23
    p = O.OracleParams(B=B, L=L, V=V, dtype=dtype, conf_mode=O.CONF_MAXPROB, tau_max=0.0, tau_min=0.0, D=0)
    lg = (rng.standard_normal((B, L, V)) * 1.5).astype(np.float32)
    lg[0, 3, : V // 2] = -np.inf                       # zero-probability prefix
    lg[1, 4, :] = -30.0
    lg[1, 4, V - 1] = 5.0                              # all the mass on the last token (ragged tail when V % 8 != 0)
    lg[1, 5, :] = -30.0
    lg[1, 5, 0] = 5.0                                  # all the mass on the first token
    u = rng.random((B, L), dtype=np.float32)
    u[0, 0], u[0, 1], u[0, 2] = 0.0, 1e-7, 0.9999999   # extremes
    toks, msk, log, last = check_case(gpu, p, np.zeros((B, L), np.int32), np.ones((B, L), bool), [lg],
                                      clear=False, uniforms=[u])
    assert not msk.any()
    assert toks[1, 4] == V - 1 and toks[1, 5] == 0 and toks[0, 3] >= V // 2
    if V > 100:
        assert (last["final"] != last["token"]).mean() > 0.3      # sampling really differs from argmax


@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
def test_sampling_at_the_upper_edge_of_the_uniform_range(gpu, dtype):
    """Uniform numbers at and next to 1 (the input recipe of the other tests keeps them away from
    there): the largest binary32 number below 1 selects by the ordinary rule; a number the
    cumulative sum never exceeds (1.0, not a valid draw) selects the last token with a non-zero
    probability, in the oracle and in the library alike."""
    import paper_2602_11133_amd as J
    V, L = 40_000, 6
    rng = np.random.default_rng(90)
    lg = rng.standard_normal((1, L, V)).astype(np.float32)
    lg[0, 0, 777] = 40.0                              # peaked: all but ~1e-13 of the mass on one token
    lg[0, 1, 777] = 40.0
    lg[0, 1, 39_000:] = -np.inf                       # zero-probability tail
    lg[0, 2, 30_001:] = -np.inf
    lg[0, 3, :] = 0.0                                 # flat
    lg[0, 3, V - 3:] = -np.inf
    lg[0, 4, V - 1] = 40.0                            # peaked on the last token
    lg[0, 5, 0] = 40.0                                # peaked on the first token
    if dtype == O.BF16:
        lg = bf16_bits_to_f32(f32_to_bf16_bits(lg)).reshape(lg.shape)
    below_one = np.nextafter(np.float32(1.0), np.float32(0.0))
    u = np.array([[below_one, 1.0, 1.0, 1.0, below_one, 1.0]], np.float32)
    p = O.OracleParams(B=1, L=L, V=V, dtype=dtype, conf_mode=O.CONF_MAXPROB, tau_max=0.0, tau_min=0.0, D=0)
    st = O.OracleState.init(p, np.zeros((1, L), np.int32), np.ones((1, L), bool))
    rec = st.step(as_rows(lg.reshape(L, V), dtype), sample_u=u)
    assert rec.commit.all()
    assert rec.final_token.tolist()[:3] == [777, 38_999, 30_000] and rec.final_token[3] == V - 4
    assert rec.final_token[4] == V - 1
    jp = J.JotParams(B=1, L=L, V=V, dtype=dtype, conf_mode=O.CONF_MAXPROB, tau_max=0.0, tau_min=0.0, gamma=0.5,
                     D=0, eps=1e-12, gen_start=0, block_size=0)
    g = gpu.GpuJot(jp, np.zeros((1, L), np.int32), np.ones((1, L), bool))
    g.step(to_device(lg, dtype, V), stride_b=L * V, stride_l=V, uniforms=u)
    np.testing.assert_array_equal(g.last()["final"], rec.final_token)
    np.testing.assert_array_equal(g.tokens(), st.tokens)
    g.close()


def test_sampling_leaves_unfinalized_positions_alone(gpu):
    p, tokens, masked, seq = random_case(51, B=2, L=60, V=500, gs=8, conf_mode=O.CONF_RATIO, tau_max=50.0,
                                         tau_min=1.0, gamma=0.5, D=8, steps=5)
    rng = np.random.default_rng(52)
    us = [rng.random((2, 60), dtype=np.float32) for _ in range(5)]
    check_case(gpu, p, tokens, masked, seq, uniforms=us, schedule=[([1, 2], 0.0)] * 5)


# --------------------------------------------------------------------------- sizes, streams, run-time errors

def test_active_count_can_be_polled_without_waiting(gpu):
    """jot_active_count_poll never blocks: it returns the count of the last COMPLETED step and how
    many steps have completed; polled until the enqueued step shows up it agrees with the waiting
    call, and it is consistent (never a count of one step labelled with another)."""
    import time
    import paper_2602_11133_amd as J
    p, tokens, masked, seq = random_case(77, B=3, L=90, V=4000, gs=10, conf_mode=O.CONF_RATIO, tau_max=40.0,
                                         tau_min=1.0, gamma=0.5, D=8, steps=4)
    jp = J.JotParams(B=p.B, L=p.L, V=p.V, dtype=p.dtype, conf_mode=p.conf_mode, tau_max=p.tau_max, tau_min=p.tau_min,
                     gamma=p.gamma, D=p.D, eps=p.eps, gen_start=p.gen_start, block_size=p.block_size)
    st = O.OracleState.init(p, tokens, masked)
    g = gpu.GpuJot(jp, tokens, masked)
    n0, done0 = J.jot_active_count_poll(g.h)
    assert (n0, done0) == (st.active_count(), 0)
    for n, logits in enumerate(seq, 1):
        lg = np.array(logits, np.float32)
        clear_guard_band(st, lg)
        st.step(as_rows(lg.reshape(p.B * p.L, p.V)[st.active_list()], p.dtype))
        sl = p.V + (-p.V) % 4
        g.step(to_device(lg, p.dtype, sl), stride_b=p.L * sl, stride_l=sl)
        deadline = time.time() + 20.0
        seen = set()
        while True:
            cnt, done = J.jot_active_count_poll(g.h)
            seen.add((cnt, done))
            if done == n or time.time() > deadline:
                break
        assert done == n and cnt == st.active_count()
        assert seen <= {(n0, n - 1), (cnt, n)}               # only the old or the new snapshot, never a mix
        n0 = cnt
        assert J.jot_active_count(g.h) == cnt and J.jot_step_index(g.h) == n
    g.close()


def test_very_long_vocabulary_single_rows(gpu):
    # one row of 3 000 001 logits (12 MB): many pieces per row, 64-bit-safe index arithmetic, ragged end
    B, L, V = 1, 3, 3_000_001
    rng = np.random.default_rng(61)
    p = O.OracleParams(B=B, L=L, V=V, dtype=O.F32, conf_mode=O.CONF_RATIO, tau_max=20.0, tau_min=1.0, D=1)
    lg = rng.standard_normal((B, L, V)).astype(np.float32)
    lg[0, 0, V - 1] = 12.0
    lg[0, 1, 1_500_000] = 11.0
    lg[0, 2, 0] = 2.0
    toks, msk, log, last = check_case(gpu, p, np.zeros((B, L), np.int32), np.ones((B, L), bool), [lg])
    assert toks[0, 0] == V - 1 and toks[0, 1] == 1_500_000


def test_large_canvas_with_few_masked_positions(gpu):
    # 1.5 million canvas positions, about 1 % masked, scattered: frozen positions cost nothing
    B, L, V = 300, 5000, 24
    rng = np.random.default_rng(62)
    p = O.OracleParams(B=B, L=L, V=V, dtype=O.BF16, conf_mode=O.CONF_MAXPROB, tau_max=0.5, tau_min=0.0,
                       gamma=0.7, D=16, gen_start=100)
    masked = rng.random((B, L)) < 0.01
    masked[:, :100] = False
    tokens = rng.integers(0, V, (B, L)).astype(np.int32)
    seq = [np.round(rng.standard_normal((B, L, V)) * 8) / 4 for _ in range(2)]
    check_case(gpu, p, tokens, masked, seq)


def test_step_argument_errors_have_no_effect(gpu):
    import paper_2602_11133_amd as J
    p, tokens, masked, seq = random_case(63, B=2, L=20, V=100, gs=4, conf_mode=O.CONF_RATIO, tau_max=5.0,
                                         tau_min=1.0, gamma=0.5, D=4, steps=1)
    jp = J.JotParams(B=2, L=20, V=100, dtype=0, conf_mode=0, tau_max=5.0, tau_min=1.0, gamma=0.5, D=4,
                     eps=1e-12, gen_start=4, block_size=0)
    g = gpu.GpuJot(jp, tokens, masked)
    dev = to_device(seq[0], O.F32, 100)
    before = (g.tokens().copy(), g.masked().copy(), g.active_list().copy())
    lib = J.load_library()
    st = g.stream
    assert lib.jot_step(g.h, dev.data_ptr(), 2000, 99, st) == -1            # stride_l < V
    assert lib.jot_step(g.h, dev.data_ptr(), 1000, 100, st) == -1           # rows of different batches overlap
    assert lib.jot_step(g.h, dev.data_ptr() + 4, 2000, 100, st) == -5       # misaligned base
    assert lib.jot_step(g.h, dev.data_ptr(), 2048, 102, st) == -5           # misaligned row stride
    assert lib.jot_step(g.h, None, 2000, 100, st) == -2
    assert lib.jot_step_scheduled(g.h, dev.data_ptr(), 2000, 100, None, 1.5, st) == -1
    assert lib.jot_step_scheduled(g.h, dev.data_ptr(), 2000, 100, None, float("nan"), st) == -1
    assert J.jot_step_index(g.h) == 0
    np.testing.assert_array_equal(g.tokens(), before[0])
    np.testing.assert_array_equal(g.masked(), before[1])
    np.testing.assert_array_equal(g.active_list(), before[2])
    g.close()


def test_two_states_interleaved_on_a_side_stream(gpu):
    # two independent decodes stepped alternately on a non-default stream
    import paper_2602_11133_amd as J
    cases = [random_case(64 + k, B=2, L=50, V=700, gs=6, conf_mode=O.CONF_RATIO, tau_max=10.0, tau_min=1.0,
                         gamma=0.5, D=8, steps=3) for k in range(2)]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        oracles, gpus = [], []
        for (p, tokens, masked, seq) in cases:
            jp = J.JotParams(B=p.B, L=p.L, V=p.V, dtype=p.dtype, conf_mode=p.conf_mode, tau_max=p.tau_max,
                             tau_min=p.tau_min, gamma=p.gamma, D=p.D, eps=p.eps, gen_start=p.gen_start,
                             block_size=p.block_size)
            oracles.append(O.OracleState.init(p, tokens, masked))
            gpus.append(gpu.GpuJot(jp, tokens, masked))
            assert gpus[-1].stream == side.cuda_stream
        for n in range(3):
            devs = []
            for k, (p, tokens, masked, seq) in enumerate(cases):
                lg = np.array(seq[n], np.float32)
                clear_guard_band(oracles[k], lg)
                devs.append(to_device(lg, p.dtype, p.V + (-p.V) % 4))
                act = oracles[k].active_list()
                oracles[k].step(as_rows(lg.reshape(p.B * p.L, p.V)[act], p.dtype))
            for k in (0, 1):                                   # both enqueued before either is read
                sl = devs[k].stride(1)
                gpus[k].step(devs[k], stride_b=cases[k][0].L * sl, stride_l=sl)
            for k in (1, 0):
                np.testing.assert_array_equal(gpus[k].tokens(), oracles[k].tokens)
                np.testing.assert_array_equal(gpus[k].active_list(), oracles[k].active_list().astype(np.int32))
        for g in gpus:
            g.close()


@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
def test_adversarial_rows(gpu, dtype):
    # rows built to stress the running reference of the exponent sums and the tie rules
    V, L = 20_000, 12
    p = O.OracleParams(B=1, L=L, V=V, dtype=dtype, conf_mode=O.CONF_RATIO, tau_max=3.0, tau_min=1.0, D=0)
    v = np.arange(V, dtype=np.float32)
    lg = np.zeros((1, L, V), np.float32)
    lg[0, 0] = v * 0.5                                   # steady climb to 1e4: the reference moves many times
    lg[0, 1] = -v * 0.5                                  # steady fall: maximum first
    lg[0, 2] = np.where(v % 2 == 0, 1.0e4, -1.0e4)       # alternating extremes, tied maxima
    lg[0, 3] = 3.0e6                                     # constant at the edge of the supported range
    lg[0, 4] = np.where(v % 5 == 0, -3.0e6, -3.0e6 - 8)
    lg[0, 5] = np.where(v == 777, 2.0, np.where(v > 9000, -1.0e30, -3.0e38))   # fill values around one real logit
    lg[0, 6] = 1.0e-40                                   # subnormal in binary32
    lg[0, 7] = np.where(v % 3 == 0, -0.0, 0.0)           # signed zeros are equal: lowest index wins
    lg[0, 8] = np.sin(v) * 50.0                          # oscillating, several near-maxima
    lg[0, 9] = np.minimum(v, 100.0)                      # long plateau of equal maxima from index 100
    lg[0, 10] = np.where(v < V - 1, -np.inf, 3.0)        # one finite entry at the very end
    lg[0, 11] = (v % 97) * 0.25 - 1.0e3                  # sawtooth far below zero
    toks, msk, log, last = check_case(gpu, p, np.zeros((1, L), np.int32), np.ones((1, L), bool), [lg], clear=False)
    assert last["token"][3] == 0 and last["token"][5] == 777 and last["token"][7] == 0
    assert last["p1"][5] == 1.0 and last["p2"][5] == 0.0
    assert last["token"][9] == 100 and last["token"][10] == V - 1
    if dtype == O.F32:                                   # (in bf16 the top of the ramp is a plateau of equal values)
        assert last["token"][0] == V - 1


@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
def test_fill_values_of_any_size(gpu, dtype):
    # masked-token fill values of any size count as probability 0
    V, L = 70_000, 6
    rng = np.random.default_rng(70)
    p = O.OracleParams(B=1, L=L, V=V, dtype=dtype, conf_mode=O.CONF_MAXPROB, tau_max=0.0, tau_min=0.0, D=0)
    lg = rng.standard_normal((1, L, V)).astype(np.float32)
    lg[0, 0, 30_000:] = -1.0e9                           # a whole region masked with a finite fill value
    lg[0, 1, :60_000] = -1.0e30
    lg[0, 2, ::3] = -3.0e38
    lg[0, 3, 10_000:50_000] = -np.inf
    lg[0, 4, 5] = 3.9e6                                  # far above the rest
    lg[0, 5, :] = np.where(np.arange(V) % 7 == 0, -3.9e6, -3.9e6 - 16)   # far below zero as a whole
    toks, msk, log, last = check_case(gpu, p, np.zeros((1, L), np.int32), np.ones((1, L), bool), [lg], clear=False)
    assert not msk.any()
    assert toks[0, 4] == 5 and toks[0, 0] < 30_000 and toks[0, 1] >= 60_000 and toks[0, 5] == 0


def far_rows(rng, V, L):
    """Rows whose entries lie far from zero (beyond +-4e6, where the reduction's one-pass base-2
    sums stop being accurate and it sums the row a second time against its maximum): Section 4.1
    defines their softmax like any other, from the differences to the row maximum."""
    lg = rng.standard_normal((1, L, V)).astype(np.float32)
    lg[0, 0, :] = 1.0e30                                  # constant, huge: uniform distribution
    lg[0, 1, 123] = 5.0e6                                 # one huge outlier: p1 = 1
    lg[0, 2, :] = -1.0e9                                  # constant, very negative: uniform
    lg[0, 3, :] = (-5.0e6 - 0.5 * (np.arange(V) % 11)).astype(np.float32)    # structure 5e6 below zero
    lg[0, 4, :] = (2.0 ** 24 + 2.0 * (np.arange(V) % 7)).astype(np.float32)  # ... and 1.7e7 above
    lg[0, 5, :] = -3.0e38
    lg[0, 5, V // 2] = -6.0e6                             # fill values around one very negative real logit
    lg[0, 6, :] = np.where(np.arange(V) % 2 == 0, 4.5e6, -4.5e6)            # both ends of the range
    lg[0, 7, V - 1] = 1.0e10                              # the outlier sits in the ragged tail
    return lg


@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
@pytest.mark.parametrize("V", [70_000, 300_007])          # whole rows / rows cut into pieces
def test_rows_far_from_zero(gpu, dtype, V):
    L = 8
    rng = np.random.default_rng(71)
    p = O.OracleParams(B=1, L=L, V=V, dtype=dtype, conf_mode=O.CONF_MAXPROB, tau_max=0.9, tau_min=0.9, D=0)
    lg = far_rows(rng, V, L)
    u = rng.random((1, L), dtype=np.float32)
    toks, msk, log, last = check_case(gpu, p, np.zeros((1, L), np.int32), np.ones((1, L), bool), [lg], clear=False,
                                      uniforms=[u])
    assert msk[0].tolist() == [True, False, True, True, True, False, True, False]
    assert toks[0, 1] == 123 and toks[0, 5] == V // 2 and toks[0, 7] == V - 1
    assert last["token"].tolist()[:4] == [0, 123, 0, 0] and last["token"][4] == (6 if dtype == O.F32 else 0)


@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
def test_stability_rule_on_rows_far_from_zero(gpu, dtype):
    # the cross term of the divergence rides along with the second summation of such rows
    V, L = 70_000, 8
    rng = np.random.default_rng(72)
    p = O.OracleParams(B=1, L=L, V=V, dtype=dtype, conf_mode=O.CONF_MAXPROB, tau_max=2.0, tau_min=2.0, D=0)
    a = far_rows(rng, V, L)
    b = a.copy()
    b[0, 3, ::5] -= 1.0                                   # moved (in steps binary32 resolves at 5e6)
    b[0, 4, ::3] += 4.0
    b[0, 6, 1::2] = -4.6e6                                # moved where the weight is 0: no change
    toks, msk, log, last = check_case(gpu, p, np.zeros((1, L), np.int32), np.ones((1, L), bool), [a, b, b],
                                      clear=False, kl=[(0.05, 0.0)] * 3)
    assert np.isfinite(last["kl"]).all() and len(log) > 0


# --------------------------------------------------------------------------- row-wide early commit

@pytest.mark.parametrize("L,block", [(70, 0), (2600, 0), (300, 32)])
def test_rowwide_rule(gpu, L, block):
    # rows with very different mean gaps: some fire, some do not; long rows take the separate kernels
    B, V = 4, 60
    rng = np.random.default_rng(80 + L)
    p = O.OracleParams(B=B, L=L, V=V, dtype=O.F32, conf_mode=O.CONF_RATIO, tau_max=1e6, tau_min=1e6, D=4,
                       gen_start=6, block_size=block)
    masked = np.zeros((B, L), bool)
    masked[:, 6:] = rng.random((B, L - 6)) < 0.9
    lg = rng.standard_normal((B, L, V)).astype(np.float32)
    lg[1, :, 7] += 9.0                                   # decided row
    lg[3, :, 2] += 4.0                                   # in between
    lg[2, 10, 5] = np.nan                                # a row without a softmax does not count
    lg[2, 11, :] = -np.inf
    lg[2, 11, 3] = 0.0                                   # one finite logit: gap = +inf, the mean too
    toks, msk, log, last = check_case(gpu, p, np.zeros((B, L), np.int32), masked, [lg, lg, lg], clear=False,
                                      global_gap=[6.0, 3.0, 1.0])
    assert (last["flags"] & 4).any()


# --------------------------------------------------------------------------- KL stability rule

def drifting_logits(rng, B, L, V, steps, scale=2.0, drift=0.05):
    """A sequence of logit tensors whose rows move by small random amounts per step, a few rows by
    large ones, around a planted token of varying strength."""
    base = (rng.standard_normal((B, L, V)) * scale).astype(np.float32)
    target = rng.integers(0, V, (B, L))
    boost = rng.uniform(0.0, 12.0, (B, L)).astype(np.float32)
    np.put_along_axis(base, target[..., None], boost[..., None], -1)
    seq = []
    for n in range(steps):
        amount = np.where(rng.random((B, L, 1)) < 0.2, 1.0, drift).astype(np.float32)
        base = base + (rng.standard_normal((B, L, V)).astype(np.float32) * amount)
        seq.append(base.copy())
    return seq


@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
@pytest.mark.parametrize("V", [2, 9, 1003, 8200, 40_003])
def test_stability_rule(gpu, dtype, V):
    B, L = 3, 40
    rng = np.random.default_rng(900 + V)
    p = O.OracleParams(B=B, L=L, V=V, dtype=dtype, conf_mode=O.CONF_MAXPROB, tau_max=2.0, tau_min=2.0, D=4,
                       gen_start=5)                       # the early exit never fires: only the rule under test
    masked = np.zeros((B, L), bool)
    masked[:, 5:] = rng.random((B, L - 5)) < 0.9
    seq = drifting_logits(rng, B, L, V, 4, drift=0.05 if dtype == O.F32 else 0.25)
    thr = 0.004 if dtype == O.F32 else 0.09
    toks, msk, log, last = check_case(gpu, p, np.zeros((B, L), np.int32), masked, seq, clear=False, stride_pad=1,
                                      kl=[(thr, 0.0), (thr, 0.3), None, (thr * 2, 0.0)])
    assert len(log) > 0 and (msk.any() or V < 100)         # some positions were stable, some (long rows) were not


def test_stability_rule_when_rows_are_cut_into_pieces(gpu):
    B, L, V = 1, 7, 300_007
    rng = np.random.default_rng(77)
    p = O.OracleParams(B=B, L=L, V=V, dtype=O.F32, conf_mode=O.CONF_MAXPROB, tau_max=2.0, tau_min=2.0, D=2,
                       gen_start=1)
    masked = np.ones((B, L), bool)
    masked[0, 0] = False
    a = (rng.standard_normal((B, L, V)) * 2).astype(np.float32)
    a[0, 1, 250_000] = 14.0                               # decided row, planted in a late piece
    a[0, 2, 5] = 30.0                                     # very decided: the other pieces carry almost no weight
    b = a + (rng.standard_normal((B, L, V)) * 0.02).astype(np.float32)
    b[0, 3] = a[0, 3] + (rng.standard_normal(V) * 0.8).astype(np.float32)     # this one moved
    b[0, 4, V - 3:] += 6.0                                # movement confined to the ragged tail
    toks, msk, log, last = check_case(gpu, p, np.zeros((B, L), np.int32), masked, [a, b, b], clear=False,
                                      kl=[(0.001, 0.0), (0.001, 0.0), (0.0005, 0.0)])
    got = {int(pos): int(step) for step, pos, tok in log}
    assert got[1] == 2 and got[2] == 2 and got[5] == 2 and got[6] == 2        # still within 0.001 of their past
    assert got[3] == 3 and got[4] == 3                                         # identical rows: divergence 0
    assert np.all(np.abs(last["kl"]) < 1e-5)               # (the rows are cut differently in the two steps)


@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
def test_stability_rule_with_vocabulary_masks_and_broken_rows(gpu, dtype):
    B, L, V = 2, 12, 520
    rng = np.random.default_rng(31)
    p = O.OracleParams(B=B, L=L, V=V, dtype=dtype, conf_mode=O.CONF_MAXPROB, tau_max=2.0, tau_min=2.0, D=2,
                       gen_start=2, block_size=5)
    masked = np.zeros((B, L), bool)
    masked[:, 2:] = True
    a = rng.standard_normal((B, L, V)).astype(np.float32)
    a[:, :, 9] += 8.0
    a[:, :, 100:200] = -np.inf                            # a static vocabulary mask, the same in every step
    a[:, :, 300:310] = -1e30                              # ... and fill values
    b = a.copy()
    b[:, :, :100] += (rng.standard_normal((B, L, 100)) * 0.05).astype(np.float32)
    b[0, 3, 150] = -20.0                                  # weight appears where there was none: divergence +inf
    b[0, 4, 50] = np.nan                                  # no softmax now
    a[1, 2, 7] = np.nan                                   # no softmax before
    a[1, 3, 400] = np.inf                                 # no softmax before either
    c = b.copy()
    c[0, 4, 50] = 0.0                                     # mended, but its previous step had none
    toks, msk, log, last = check_case(gpu, p, np.zeros((B, L), np.int32), masked, [a, b, c, c, c], clear=False,
                                      kl=[(0.5, 0.5)] * 5)
    assert len(log) > 0


def test_stability_rule_argument_errors(gpu):
    import paper_2602_11133_amd as J
    p, tokens, masked, seq = random_case(64, B=2, L=20, V=100, gs=4, conf_mode=O.CONF_RATIO, tau_max=5.0,
                                         tau_min=1.0, gamma=0.5, D=4, steps=1)
    jp = J.JotParams(B=2, L=20, V=100, dtype=0, conf_mode=0, tau_max=5.0, tau_min=1.0, gamma=0.5, D=4,
                     eps=1e-12, gen_start=4, block_size=0)
    g = gpu.GpuJot(jp, tokens, masked)
    dev = to_device(seq[0], O.F32, 100)
    lib = J.load_library()

    def call(**kw):
        opt = J.JotStepOptions()
        opt.enable_kl = 1
        opt.prev_logits_dev = dev.data_ptr()
        opt.kl_threshold, opt.kl_min_prob = 0.1, 0.5
        for k, v in kw.items():
            setattr(opt, k, v)
        import ctypes
        return lib.jot_step_ex(g.h, dev.data_ptr(), 2000, 100, ctypes.byref(opt), g.stream)

    assert call(prev_logits_dev=None) == -2
    assert call(prev_logits_dev=dev.data_ptr() + 4) == -5
    assert call(kl_threshold=-0.1) == -1
    assert call(kl_threshold=float("nan")) == -1
    assert call(kl_min_prob=1.5) == -1
    assert J.jot_step_index(g.h) == 0
    assert call() == 0 and J.jot_step_index(g.h) == 1
    g.close()


# --------------------------------------------------------------------------- compact logits

@pytest.mark.parametrize("dtype", [O.F32, O.BF16])
@pytest.mark.parametrize("V,L,block", [(9, 30, 0), (1003, 70, 0), (8200, 50, 5), (40_003, 20, 0), (300_007, 6, 0)])
def test_compact_logits(gpu, dtype, V, L, block):
    # one row per examined entry, padded row stride, schedule on; long vocabularies are cut into pieces
    p, tokens, masked, seq = random_case(300 + V, B=3, L=L, V=V, gs=L // 4, dtype=dtype, conf_mode=O.CONF_MAXPROB,
                                         tau_max=0.9, tau_min=0.2, gamma=0.6, D=6, steps=3, block_size=block)
    check_case(gpu, p, tokens, masked, seq, stride_pad=1, compact=True,
               schedule=[(np.array([1, 0, 2], np.int32), 0.0), (None, 0.25), (None, 0.0)])


def test_compact_logits_sampled_and_errors(gpu):
    import ctypes
    import paper_2602_11133_amd as J
    rng = np.random.default_rng(5)
    B, L, V = 2, 17, 520
    p = O.OracleParams(B=B, L=L, V=V, dtype=O.F32, conf_mode=O.CONF_MAXPROB, tau_max=0.0, tau_min=0.0, D=0)
    lg = (rng.standard_normal((B, L, V)) * 1.5).astype(np.float32)
    masked = rng.random((B, L)) < 0.7
    u = rng.random((B, L)).astype(np.float32)
    check_case(gpu, p, np.zeros((B, L), np.int32), masked, [lg], uniforms=[u], compact=True, clear=False)
    # compact logits cannot be combined with the KL rule
    jp = J.JotParams(B=B, L=L, V=V, dtype=0, conf_mode=1, tau_max=0.5, tau_min=0.5, gamma=0.5, D=0, eps=0.0,
                     gen_start=0, block_size=0)
    g = gpu.GpuJot(jp, np.zeros((B, L), np.int32), masked)
    dev = to_device(lg, O.F32, V)
    opt = J.JotStepOptions()
    opt.logits_compact = 1
    opt.enable_kl = 1
    opt.prev_logits_dev = dev.data_ptr()
    opt.kl_threshold = 0.1
    assert J.load_library().jot_step_ex(g.h, dev.data_ptr(), 0, V, ctypes.byref(opt), g.stream) == -1
    assert J.jot_step_index(g.h) == 0
    g.close()
