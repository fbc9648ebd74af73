"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI.

Bar: bit-exact argmax tokens, masks, commit order and active lists; confidences within 1e-5
relative for fp32 logits and 2e-3 relative for bf16 logits.  Every confidence of the oracle is
kept at least 1e-4 (relative to max(1, tau)) away from its threshold by the input recipe, so
the fp32 decision on the GPU and the fp64 decision of the oracle are the same decision.
"""
import os
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from gen.configs import BF16, CONF_MAXPROB, CONF_PROBGAP, CONF_RATIO, CONFIGS, F32  # noqa: E402
from harness import LockstepRun  # noqa: E402

THREADS = int(os.environ.get("JOT_TEST_THREADS", "16"))
TOL = {F32: 1e-5, BF16: 2e-3}
# (kl_threshold, kl_min_prob) per workload, placed inside the bulk of the divergences the workload's
# consecutive steps show (independent noise of variance ~1 per step: about 1; the low-noise
# large-vocabulary workload: about 1.2e-3), so that the rule decides both ways
KL_CASES = {2: (1.0, 0.0), 3: (0.995, 0.0), 4: (1.0, 0.0), 5: (0.0014, 0.0)}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the MI355X; there is no CPU fallback")
    import gpu_harness
    return gpu_harness


def check_every_row(g, cfg, tokens0, masked0):
    """What must hold in batch rows the oracle did not follow (and in the others too): the
    finalization log is ordered and names every position at most once, the mask only shrinks,
    tokens of positions that were never finalized are untouched, the list of positions the next
    step examines is ascending and made of masked positions only."""
    tok, msk, cst, log = g.tokens(), g.masked(), g.commit_step(), g.commit_log()
    n = cfg.B * cfg.L
    steps, pos, tk = log[:, 0].astype(np.int64), log[:, 1].astype(np.int64), log[:, 2]
    assert np.all(np.diff(steps * n + pos) > 0)                      # step-major, ascending position, no repeats
    assert np.unique(pos).size == pos.size
    assert masked0.reshape(-1)[pos].all() and (tk >= 0).all() and (tk < cfg.V).all()
    want_msk = masked0.reshape(-1).copy()
    want_msk[pos] = False
    np.testing.assert_array_equal(msk.reshape(-1), want_msk)
    want_tok = tokens0.reshape(-1).copy()
    want_tok[pos] = tk
    np.testing.assert_array_equal(tok.reshape(-1), want_tok)
    want_cst = np.zeros(n, np.int32)
    want_cst[pos] = steps
    np.testing.assert_array_equal(cst.reshape(-1), want_cst)
    act = g.active_list().astype(np.int64)
    assert np.all(np.diff(act) > 0) and msk.reshape(-1)[act].all()
    if cfg.block_size <= 0:
        np.testing.assert_array_equal(act, np.flatnonzero(msk.reshape(-1)))


def run_parity(gpu, cfg, batch_rows=None, max_steps=None, use_device_gen=True, schedule=None, sample=False,
               global_gap=None, kl=None, compact=False, shards=None):
    """Lock-step decode: oracle on the host (optionally on a subset of batch rows), library on
    the GPU over the whole batch; compares every step and the final state.
    shards: optional list of lists of batch rows; the oracle then follows each list as a sub-batch
    of its own (bounds host memory), all of them at every step.
    global_gap: optional function step -> threshold of the row-wide early-commit rule.
    kl: optional (kl_threshold, kl_min_prob) of the KL stability rule, applied at every step.
    compact: hand the library a [n_examined, V] tensor (rows in list order) instead of [B, L, V]."""
    from gen.device import DeviceGenerator
    import paper_2602_11133_amd as J
    if shards is None:
        shards = [batch_rows]
    say(f"[parity] {cfg.name} B={cfg.B} L={cfg.L} V={cfg.V} dtype={cfg.dtype} mode={cfg.conf_mode} "
        f"tau=({cfg.tau_max},{cfg.tau_min}) block={cfg.block_size} rows={shards}")
    runs = [LockstepRun(cfg, threads=THREADS, batch_rows=shards[0])]
    runs += [LockstepRun(cfg, threads=THREADS, batch_rows=rows, share=runs[0]) for rows in shards[1:]]
    assert use_device_gen or len(runs) == 1
    traj = runs[0].traj
    tokens0, masked0 = traj.initial_canvas()
    g = gpu.GpuJot(gpu.params_of(cfg), tokens0, masked0)
    dgen = DeviceGenerator(cfg, traj.target, traj.rival)
    bufs = [dgen.alloc_logits(poison=True), dgen.alloc_logits(poison=True) if kl else None]
    n_stable = 0
    in_run = np.full(cfg.B, -1)
    for k, run in enumerate(runs):
        assert (in_run[run.batch_rows] < 0).all(), "sub-batches overlap"
        in_run[run.batch_rows] = k
    all_followed = bool((in_run >= 0).all())
    steps = cfg.steps + 16 if max_steps is None else max_steps
    n_done = 0
    for n in range(1, steps + 1):
        if all(run.state.active_count() == 0 for run in runs):
            break
        nt, frac = schedule(n) if schedule else (None, 0.0)
        frac = float(np.float32(frac))
        u = runs[0].draw_uniforms(n) if sample else None
        gg = None if global_gap is None else float(np.float32(global_gap(n)))
        want = []
        for run in runs:                          # the oracle, one sub-batch after the other
            act_full = run.active_full()
            rec, _, _, rows = run.next_step(nt, frac, u, gg, kl)
            want.append((act_full, rec))
            n_stable += int(rec.stable.sum())
        T, R = traj.planted(n)                    # with every adjustment the sub-batches made to this step
        logits, prev = (bufs[n % 2], bufs[(n - 1) % 2]) if kl else (bufs[0], None)   # ping-pong under the KL rule
        n_gpu = g.active_count()
        if use_device_gen:
            dgen.set_planted(T, R)
            dgen.fill(logits, n, J.jot_active_list(g.h), n_gpu)
        else:
            gpu.upload_rows(logits, want[0][0], rows, cfg.dtype)
        if compact:
            small = gpu.gather_compact(logits, J.jot_active_list(g.h), n_gpu)
            g.step(small, n_transfer=nt, transfer_frac=frac, uniforms=u, global_gap=gg, compact=True)
        else:
            g.step(logits, n_transfer=nt, transfer_frac=frac, uniforms=u, global_gap=gg, kl=kl, prev_logits=prev)
        last = g.last()
        assert np.all(np.diff(last["active"].astype(np.int64)) > 0)           # every row: ascending positions
        row_of = in_run[last["active"] // cfg.L]
        for k, (act_full, rec) in enumerate(want):
            sel = (row_of == k) if not (all_followed and len(runs) == 1) else None
            gpu.compare_step(last, rec, act_full, TOL[cfg.dtype], sel)
        if all_followed:
            assert last["active"].size == sum(a.size for a, _ in want)
            assert g.active_count() == sum(run.state.active_count() for run in runs)
        n_done = n
        if n % 32 == 0:
            say(f"  step {n}: examined {last['active'].size}, oracle rows {sum(a.size for a, _ in want)}")
    say(f"  finished after {n_done} steps, bumps={sum(r.n_bumps for r in runs)}, stable={n_stable}")
    if kl:
        assert n_stable > 0, "the stability rule never fired: the case tests nothing"
    # final state of the followed rows
    tok, msk, cst = g.tokens(), g.masked(), g.commit_step()
    log = g.commit_log()
    log_run = in_run[log[:, 1] // cfg.L]
    for k, run in enumerate(runs):
        st = run.state
        np.testing.assert_array_equal(tok[run.batch_rows], st.tokens)
        np.testing.assert_array_equal(msk[run.batch_rows], st.masked)
        want_log = np.array([(s, p, t) for (s, p, t) in st.commit_log], np.int64).reshape(-1, 3)
        want_log[:, 1] = run.to_full(want_log[:, 1])
        np.testing.assert_array_equal(log[log_run == k], want_log.astype(np.int32))
    # every batch row, followed or not
    check_every_row(g, cfg, tokens0, masked0)
    # generated inputs never hold NaN or +inf, and rows the step does not examine are poisoned: a
    # read of a frozen row, in any batch row, would be counted here
    assert J.jot_anomaly_count(g.h) == 0
    if all_followed:
        want_act = np.sort(np.concatenate([run.active_full() for run in runs])).astype(np.int32)
        np.testing.assert_array_equal(g.active_list(), want_act)
        assert g.active_count() == want_act.size
    g.close()
    return n_done


# --------------------------------------------------------------------------- generator identity

@pytest.mark.parametrize("cid", [1, 2, 5])
def test_device_generator_is_byte_identical_to_host(gpu, cid):
    from gen.device import DeviceGenerator
    from gen.host import HostGenerator
    from gen.trajectory import Trajectory
    cfg = CONFIGS[cid]
    if cid == 5:
        cfg = cfg.replace(B=2)
    tr = Trajectory(cfg)
    T, R = tr.planted(3)
    hg = HostGenerator(cfg, tr.target, tr.rival, threads=THREADS)
    dg = DeviceGenerator(cfg, tr.target, tr.rival)
    dg.set_planted(T, R)
    logits = dg.alloc_logits(poison=True)
    pos = np.unique(np.concatenate([[cfg.gen_start, cfg.B * cfg.L - 1],
                                    np.random.default_rng(cid).integers(cfg.gen_start, cfg.L, 20)]))
    pos = pos[(pos % cfg.L) >= cfg.gen_start]
    pos_dev = torch.from_numpy(pos.astype(np.int32)).cuda()
    dg.fill(logits, 3, pos_dev.data_ptr(), pos.size)
    torch.cuda.synchronize()
    got = logits.view(cfg.B * cfg.L, cfg.V)[torch.from_numpy(pos).cuda()].cpu()
    want = hg.rows(3, pos, T, R)
    if cfg.dtype == F32:
        np.testing.assert_array_equal(got.numpy().view(np.uint32), want.view(np.uint32))
    else:
        np.testing.assert_array_equal(got.view(torch.int16).numpy().view(np.uint16), want)
    # rows that were not generated still hold the poison
    other = cfg.gen_start + 1 if (cfg.gen_start + 1) not in pos else cfg.gen_start - 1
    assert torch.isnan(logits.view(cfg.B * cfg.L, cfg.V)[other].float()).all()


# --------------------------------------------------------------------------- the five workloads

@pytest.mark.parametrize("mode,tau_max,tau_min", [(CONF_MAXPROB, 0.9, 0.0), (CONF_RATIO, 90.0, 1.0),
                                                   (CONF_PROBGAP, 0.9, 0.0)])
def test_config1_single_step(gpu, mode, tau_max, tau_min):
    cfg = CONFIGS[1].replace(conf_mode=mode, tau_max=tau_max, tau_min=tau_min)
    assert run_parity(gpu, cfg, max_steps=1) == 1


def test_config1_bare_offset_finalizes_none_or_all(gpu):
    cfg = CONFIGS[1].replace(base="literal")
    assert run_parity(gpu, cfg, max_steps=1) == 1
    assert run_parity(gpu, cfg.replace(conf_mode=CONF_RATIO, tau_max=0.9, tau_min=0.9), max_steps=1) == 1


def test_config1_host_uploaded_rows(gpu):
    # same case with rows generated on the host and copied in: independent of the device generator
    assert run_parity(gpu, CONFIGS[1], max_steps=1, use_device_gen=False) == 1


def test_config2_full_loop(gpu):
    run_parity(gpu, CONFIGS[2])


@pytest.mark.parametrize("mode,tau_max,tau_min", [(CONF_RATIO, 90.0, 1.0), (CONF_PROBGAP, 0.9, 0.0)])
def test_config2_other_signals_short(gpu, mode, tau_max, tau_min):
    cfg = CONFIGS[2].replace(conf_mode=mode, tau_max=tau_max, tau_min=tau_min, steps=24, L=64 + 96)
    run_parity(gpu, cfg)


@pytest.mark.parametrize("tau_max", [0.7, 0.8, 0.9])
def test_config3_threshold_sweep(gpu, tau_max):
    run_parity(gpu, CONFIGS[3].replace(tau_max=tau_max))         # all 8 batch rows under the oracle


def test_config4_blockwise(gpu):
    run_parity(gpu, CONFIGS[4])                                   # all 32 batch rows, the whole decode


def test_config4_blockwise_ratio_llada_defaults_short(gpu):
    cfg = CONFIGS[4].replace(conf_mode=CONF_RATIO, tau_max=30.0, tau_min=1.0, B=4, L=128 + 128, steps=128)
    run_parity(gpu, cfg)


def test_config5_full_size_every_row_first_steps(gpu):
    # the launch shape the benchmark times; the oracle follows all 64 batch rows (as eight
    # sub-batches of eight, to bound host memory) through the first four steps
    run_parity(gpu, CONFIGS[5], shards=[list(range(k, k + 8)) for k in range(0, 64, 8)], max_steps=4)


def test_config5_full_size_whole_decode(gpu):
    # the whole batch runs on the GPU; the oracle follows eight batch rows spread over the batch
    # through all steps (rows are independent decodes); the other rows are held to the invariants
    run_parity(gpu, CONFIGS[5], batch_rows=[3, 12, 21, 30, 41, 47, 56, 63])


def test_config5_full_size_probgap_first_steps(gpu):
    cfg = CONFIGS[5].replace(conf_mode=CONF_PROBGAP, tau_max=0.9, tau_min=0.0, base="partition")
    run_parity(gpu, cfg, batch_rows=[7, 58], max_steps=3)


def test_config5_probgap_short(gpu):
    cfg = CONFIGS[5].replace(conf_mode=CONF_PROBGAP, tau_max=0.9, tau_min=0.0, B=2, L=256 + 128,
                             steps=32, base="partition", noise_scale=0.02)
    run_parity(gpu, cfg)


@pytest.mark.parametrize("scale", [1.0, 0.1])
@pytest.mark.parametrize("dtype", [F32, BF16])
def test_config5_heavy_tails_at_larger_noise_scale_short(gpu, dtype, scale):
    # the large workload scales its Student-t noise by 0.02 (so that outliers alone rarely clear the
    # ratio threshold); here the noise has unit scale, so single outliers of tens of logits decide
    # many rows, the lane maxima keep climbing late in a row and the runner-up is often an outlier too
    # (at scale 1 the outliers finalize everything within a few steps; 0.1 gives a longer decode)
    cfg = CONFIGS[5].replace(B=2, L=256 + 192, steps=24, noise_scale=scale, dtype=dtype)
    run_parity(gpu, cfg, max_steps=24)


# --------------------------------------------------------------------------- with a transfer schedule

def test_config2_with_fractional_schedule(gpu):
    # a decoder that reveals remaining/steps_left positions per step (so it ends on the last
    # configured step at the latest), with the early exit on top
    cfg = CONFIGS[2].replace(steps=48, L=64 + 192)
    n = run_parity(gpu, cfg, schedule=lambda n: (None, 1.0 / max(1, cfg.steps - n + 1)))
    assert n <= cfg.steps


def test_config4_with_one_token_per_step_schedule(gpu):
    # block-wise decoder: one position per row per step from the schedule, early exit on top
    cfg = CONFIGS[4].replace(B=8, L=128 + 128, steps=128)
    n = run_parity(gpu, cfg, batch_rows=[0, 3, 7], schedule=lambda n: (np.ones(cfg.B, np.int32), 0.0))
    assert n <= cfg.n_gen


def test_config5_ratio_with_schedule_short(gpu):
    cfg = CONFIGS[5].replace(B=4, steps=24)
    run_parity(gpu, cfg, batch_rows=[1, 2], max_steps=24, schedule=lambda n: (np.full(cfg.B, 8, np.int32), 0.02))


# --------------------------------------------------------------------------- sampling-based finalization

def test_config1_sampled(gpu):
    assert run_parity(gpu, CONFIGS[1], max_steps=1, sample=True) == 1


def test_config2_sampled_with_schedule(gpu):
    cfg = CONFIGS[2].replace(steps=32, L=64 + 128)
    run_parity(gpu, cfg, sample=True, schedule=lambda n: (None, 1.0 / max(1, cfg.steps - n + 1)))


def test_config5_sampled_short(gpu):
    cfg = CONFIGS[5].replace(B=4, steps=16)
    run_parity(gpu, cfg, batch_rows=[0, 3], max_steps=16, sample=True,
               schedule=lambda n: (np.full(cfg.B, 16, np.int32), 0.0))


# --------------------------------------------------------------------------- replay from a HIP graph

@pytest.mark.parametrize("cid,scheduled", [(2, False), (1, False), (4, True)])
def test_step_replayed_from_a_captured_graph(gpu, cid, scheduled):
    """One jot_step is captured into a HIP graph and replayed for every later step of the decode
    (step number and buffer parity live on the device, so nothing is baked into the launches).
    Between replays the program does eager work (generating the next logits, reading results
    back), and every replay is compared with the oracle."""
    import paper_2602_11133_amd as J
    from gen.device import DeviceGenerator
    cfg = {1: CONFIGS[1].replace(L=32 + 40, steps=6, traj="sigmoid", conv="uniform"),
           2: CONFIGS[2].replace(steps=20, L=64 + 96),
           4: CONFIGS[4].replace(B=3, L=128 + 64, steps=64)}[cid]
    say(f"[graph] {cfg.name} scheduled={scheduled}")
    run = LockstepRun(cfg, threads=THREADS)
    tokens0, masked0 = run.traj.initial_canvas()
    g = gpu.GpuJot(gpu.params_of(cfg), tokens0, masked0)
    dgen = DeviceGenerator(cfg, run.traj.target, run.traj.rival)
    logits = dgen.alloc_logits(poison=True)
    nt_host = np.ones(cfg.B, np.int32) if scheduled else None
    nt_dev = torch.from_numpy(nt_host).cuda() if scheduled else None

    def oracle_and_fill(n):
        act_full = run.active_full()
        rec, T, R, _ = run.next_step(nt_host, 0.0)
        dgen.set_planted(T, R)
        dgen.fill(logits, n, J.jot_active_list(g.h), g.active_count())
        return act_full, rec

    # step 1 eagerly
    act_full, rec = oracle_and_fill(1)
    g.step(logits, n_transfer=nt_host)
    gpu.compare_step(g.last(), rec, act_full, TOL[cfg.dtype])
    torch.cuda.synchronize()

    # capture one step
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        st = torch.cuda.current_stream().cuda_stream
        if scheduled:
            J.jot_step_scheduled(g.h, logits.data_ptr(), cfg.L * cfg.V, cfg.V, nt_dev.data_ptr(), 0.0, st)
        else:
            J.jot_step(g.h, logits.data_ptr(), cfg.L * cfg.V, cfg.V, st)
    torch.cuda.synchronize()

    replays = 0
    for n in range(2, cfg.steps + 16):
        if run.state.active_count() == 0:
            break
        act_full, rec = oracle_and_fill(n)
        torch.cuda.synchronize()
        graph.replay()
        if n % 2:
            torch.cuda.synchronize()
        else:       # tell the library where the replay runs: its read-backs then wait for that stream only
            J.jot_wait_on_stream(g.h, torch.cuda.current_stream().cuda_stream)
        replays += 1
        gpu.compare_step(g.last(), rec, act_full, TOL[cfg.dtype])
        assert g.active_count() == run.state.active_count()
        assert J.jot_step_index(g.h) == n                      # counted on the device, replays included
    assert replays >= 3
    np.testing.assert_array_equal(g.tokens(), run.state.tokens)
    np.testing.assert_array_equal(g.masked(), run.state.masked)
    want = np.array(run.state.commit_log, np.int32).reshape(-1, 3)
    np.testing.assert_array_equal(g.commit_log(), want)          # step numbers keep counting on the device
    g.close()


def test_config5_full_size_repeats_bit_for_bit(gpu):
    """Two decodes of the largest workload from the same inputs give identical bits everywhere
    (confidences included): no result depends on the arrival order of workgroups or atomics."""
    import paper_2602_11133_amd as J
    from gen.device import DeviceGenerator
    from gen.trajectory import Trajectory
    cfg = CONFIGS[5]
    tr = Trajectory(cfg)
    tokens0, masked0 = tr.initial_canvas()
    dgen = DeviceGenerator(cfg, tr.target, tr.rival)
    logits = dgen.alloc_logits(poison=True)
    nt = np.full(cfg.B, 4, np.int32)
    u = np.random.default_rng(5).random((cfg.B, cfg.L), dtype=np.float32)
    outs = []
    for rep in range(2):
        g = gpu.GpuJot(gpu.params_of(cfg), tokens0, masked0)
        per_step = []
        for n in range(1, 4):
            T, R = tr.planted(n)
            dgen.set_planted(T, R)
            dgen.fill(logits, n, J.jot_active_list(g.h), g.active_count())
            g.step(logits, n_transfer=nt, transfer_frac=0.01, uniforms=u)
            last = g.last()
            per_step.append({k: v.copy() for k, v in last.items()})
        outs.append((per_step, g.tokens().copy(), g.commit_log().copy(), g.active_list().copy()))
        say(f"  repetition {rep}: {outs[-1][2].shape[0]} finalized in 3 steps")
        g.close()
    a, b = outs
    for sa, sb in zip(a[0], b[0]):
        for k in sa:
            np.testing.assert_array_equal(sa[k].view(np.uint8), sb[k].view(np.uint8))
    for x, y in zip(a[1:], b[1:]):
        np.testing.assert_array_equal(x, y)
    assert a[2].shape[0] > 3 * cfg.B * 4


# --------------------------------------------------------------------------- row-wide early commit

def test_config2_with_rowwide_rule_staged_thresholds(gpu):
    # thresholds falling with progress (7.5, 5, 2.5 on the logit scale, the values Section 6.1
    # quotes for the global rule), early exit on top
    cfg = CONFIGS[2].replace(steps=36, L=64 + 128, conf_mode=CONF_RATIO, tau_max=90.0, tau_min=1.0)
    stage = lambda n: 7.5 if n <= 12 else (5.0 if n <= 24 else 2.5)
    n = run_parity(gpu, cfg, global_gap=stage)
    assert n <= cfg.steps + 16


def test_config4_rowwide_rule_with_schedule_and_sampling(gpu):
    cfg = CONFIGS[4].replace(B=4, L=128 + 96, steps=96)
    run_parity(gpu, cfg, batch_rows=[0, 3], sample=True, global_gap=lambda n: 6.0,
               schedule=lambda n: (np.ones(cfg.B, np.int32), 0.0))


def test_config5_rowwide_rule_short(gpu):
    cfg = CONFIGS[5].replace(B=3, steps=40, conv="mixture")
    run_parity(gpu, cfg, batch_rows=[0, 2], max_steps=40, global_gap=lambda n: 3.0)


# --------------------------------------------------------------------------- KL stability rule

def test_config2_with_stability_rule(gpu):
    cfg = CONFIGS[2].replace(steps=40, L=64 + 128)
    run_parity(gpu, cfg, kl=(KL_CASES[2]))


def test_config4_blockwise_stability_rule_with_schedule_and_sampling(gpu):
    cfg = CONFIGS[4].replace(B=4, L=128 + 96, steps=96)
    run_parity(gpu, cfg, batch_rows=[1, 2], sample=True, kl=KL_CASES[4],
               schedule=lambda n: (np.ones(cfg.B, np.int32), 0.0))


def test_config5_stability_rule_short(gpu):
    cfg = CONFIGS[5].replace(B=3, L=256 + 192, steps=40, conv="mixture")
    run_parity(gpu, cfg, batch_rows=[0, 2], max_steps=4, kl=KL_CASES[5])


def test_config3_bf16_stability_rule_short(gpu):
    cfg = CONFIGS[3].replace(B=2, steps=32, dtype=BF16)
    run_parity(gpu, cfg, max_steps=32, kl=KL_CASES[3])


def test_config5_full_size_stability_rule_first_steps(gpu):
    # full batch, the launch shape bench.py --kl times; the oracle follows one batch row
    # (a threshold just above the bulk of the divergences: fewer inputs to move off the guard band)
    # for four steps, three of which have a previous distribution
    run_parity(gpu, CONFIGS[5], batch_rows=[17, 44], max_steps=4, kl=(0.002, 0.0))


def test_config4_full_size_blockwise_stability_rule(gpu):
    # the bf16 two-tensor reduction in its real launch shape, block-wise: positions of a block that
    # has just become current have no history
    run_parity(gpu, CONFIGS[4], batch_rows=[0, 13, 31], max_steps=48, kl=KL_CASES[4])


def test_config3_full_size_stability_rule(gpu):
    run_parity(gpu, CONFIGS[3], max_steps=16, kl=KL_CASES[3])


def test_config5_full_size_schedule_and_sampling_first_steps(gpu):
    cfg = CONFIGS[5]
    run_parity(gpu, cfg, batch_rows=[5, 40], max_steps=3, sample=True,
               schedule=lambda n: (np.full(cfg.B, 4, np.int32), 0.01))


# --------------------------------------------------------------------------- compact logits

def test_config2_compact_logits_with_schedule_and_sampling(gpu):
    cfg = CONFIGS[2].replace(steps=40, L=64 + 160)
    run_parity(gpu, cfg, compact=True, sample=True, schedule=lambda n: (None, 1.0 / max(1, cfg.steps - n + 1)))


def test_config4_compact_logits_blockwise_with_rowwide_rule(gpu):
    cfg = CONFIGS[4].replace(B=6, L=128 + 96, steps=96)
    run_parity(gpu, cfg, batch_rows=[0, 2, 5], compact=True, global_gap=lambda n: 6.5)


def test_config5_compact_logits_short(gpu):
    cfg = CONFIGS[5].replace(B=3, steps=24)
    run_parity(gpu, cfg, batch_rows=[1], max_steps=24, compact=True)
