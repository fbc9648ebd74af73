"""The Algorithm 1 loop driver on the GPU: a fixed schedule alone ends exactly on the step
budget, the early exit on top of it ends sooner and decodes the same planted tokens, and the
driver does what the same calls made by hand do."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from gen.configs import CONFIGS  # noqa: E402


@pytest.fixture(scope="module")
def loop():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the MI355X; there is no CPU fallback")
    from paper_2602_11133_amd import decode_loop
    return decode_loop


@pytest.mark.parametrize("cid,small", [(2, dict(steps=48, L=64 + 96)), (4, dict(B=4, L=128 + 128, steps=128)),
                                       (5, dict(B=2, L=256 + 96, steps=32))])
def test_step_budget_and_step_reduction(loop, cid, small):
    cfg = CONFIGS[cid].replace(**small)
    budget = 2 * cfg.steps            # a decoder configured with twice the steps the sequence needs
    fixed = loop._synthetic_run(cfg, early_exit=False, budget=budget)
    early = loop._synthetic_run(cfg, early_exit=True, budget=budget)
    print(f"[loop] {cfg.name}: schedule only {fixed['steps']} steps, with early exit {early['steps']}", flush=True)
    want = budget                      # the schedule alone spends its whole budget ...
    if cfg.block_size > 0:             # ... or, revealing at least one position per row and step, one step per position
        n_blocks = -(-cfg.n_gen // cfg.block_size)
        per_step = -(-cfg.block_size // max(1, budget // n_blocks))
        want = n_blocks * -(-cfg.block_size // per_step)
    assert fixed["steps"] == want and fixed["still_masked"] == 0
    assert early["steps"] < fixed["steps"] and early["still_masked"] == 0    # the early exit saves steps
    assert sum(early["examined_per_step"]) < sum(fixed["examined_per_step"])
    # synthetic trajectories converge to their planted token: stopping early keeps (nearly) all of them.
    # (The heavy-tailed noise of workload 5 is made to plant outliers that clear the ratio threshold
    # on their own, so a share of its positions is finalized to a noise token by design.)
    print(f"       planted tokens kept: schedule only {fixed['tokens_equal_to_planted_targets']:.3f}, "
          f"with early exit {early['tokens_equal_to_planted_targets']:.3f}", flush=True)
    assert early["tokens_equal_to_planted_targets"] >= (0.6 if cid == 5 else 0.97)
    assert early["examined_per_step"] == sorted(early["examined_per_step"], reverse=True) or cfg.block_size > 0


def test_driver_equals_the_same_calls_made_by_hand(loop):
    import gpu_harness as G
    import paper_2602_11133_amd as J
    from gen.device import DeviceGenerator
    from gen.trajectory import Trajectory
    cfg = CONFIGS[2].replace(steps=24, L=64 + 64)
    traj = Trajectory(cfg)
    dgen = DeviceGenerator(cfg, traj.target, traj.rival)
    tokens0, masked0 = traj.initial_canvas()
    logits = dgen.alloc_logits(poison=True)

    def logits_fn(step, active_dev, n_active):
        dgen.set_planted(*traj.planted(step))
        dgen.fill(logits, step, active_dev, n_active)
        return logits.data_ptr(), cfg.L * cfg.V, cfg.V

    a = G.GpuJot(G.params_of(cfg), tokens0, masked0)
    out = loop.decode(a.h, logits_fn, cfg.steps, stream=a.stream)
    b = G.GpuJot(G.params_of(cfg), tokens0, masked0)
    n = 0
    while b.active_count() > 0 and n < cfg.steps:
        n += 1
        logits_fn(n, J.jot_active_list(b.h), b.active_count())
        b.step(logits, transfer_frac=loop.linear_schedule(n, cfg.steps))
    assert out["steps"] == n and out["still_masked"] == b.active_count() == 0
    np.testing.assert_array_equal(a.tokens(), b.tokens())
    np.testing.assert_array_equal(a.commit_log(), b.commit_log())
    a.close()
    b.close()


@pytest.mark.parametrize("cid,small", [(2, dict(steps=24, L=64 + 64)), (4, dict(B=3, L=128 + 64, steps=64))])
def test_overlapped_loop_decodes_the_same_canvas(loop, cid, small):
    """decode_overlapped enqueues the next forward pass before it polls the loop test; the canvas,
    the finalization log and the number of steps are those of the blocking loop."""
    import gpu_harness as G
    import paper_2602_11133_amd as J
    from gen.device import DeviceGenerator
    from gen.trajectory import Trajectory
    cfg = CONFIGS[cid].replace(**small)
    traj = Trajectory(cfg)
    dgen = DeviceGenerator(cfg, traj.target, traj.rival)
    tokens0, masked0 = traj.initial_canvas()
    logits = dgen.alloc_logits(poison=True)
    # a "denoiser" that needs nothing from the host: it writes the rows of every generation position
    gen_pos = torch.from_numpy(np.flatnonzero(traj.gen).astype(np.int32)).cuda()

    def forward_fn(step):
        dgen.set_planted(*traj.planted(step))
        dgen.fill(logits, step, gen_pos.data_ptr(), gen_pos.numel())
        return logits.data_ptr(), cfg.L * cfg.V, cfg.V

    def logits_fn(step, active_dev, n_active):
        return forward_fn(step)

    kw = {}
    if cfg.block_size > 0:
        nt = torch.ones(cfg.B, dtype=torch.int32, device="cuda")
        kw = dict(schedule=None, n_transfer_dev=nt.data_ptr())
    a = G.GpuJot(G.params_of(cfg), tokens0, masked0)
    out_a = loop.decode(a.h, logits_fn, 2 * cfg.steps, stream=a.stream, **kw)
    b = G.GpuJot(G.params_of(cfg), tokens0, masked0)
    out_b = loop.decode_overlapped(b.h, forward_fn, 2 * cfg.steps, stream=b.stream, **kw)
    assert out_b["steps"] == out_a["steps"] and out_b["still_masked"] == out_a["still_masked"] == 0
    assert out_b["examined_per_step"] == out_a["examined_per_step"] and out_b["speculative_forwards"] == 1
    np.testing.assert_array_equal(a.tokens(), b.tokens())
    np.testing.assert_array_equal(a.commit_log(), b.commit_log())
    assert J.jot_step_index(b.h) == out_b["steps"]
    a.close()
    b.close()
