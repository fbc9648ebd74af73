"""Algorithm 1 as a loop around the library: logits from the caller's denoiser, then one
finalization pass per step (early exit of Eq. 6 OR-ed with the decoder's transfer schedule),
until nothing is masked or the step budget is spent.

Host control flow only -- every per-position operation runs in the library's kernels.  The
denoiser is the caller's: `logits_fn(step, active_list_dev, n_active)` must return
(device pointer, stride_b, stride_l) of the [B, L, V] logits of this step; only the rows of the
listed positions have to be valid.

Run as a script it decodes one of the synthetic workloads twice -- with the fixed schedule alone
(the early exit switched off by thresholds out of reach) and with the early exit on top -- and
prints the number of denoising steps each needs: the step reduction of Section 6 on synthetic
trajectories, not a reproduction of the paper's tables.
"""
from __future__ import annotations

import argparse
import json
import time

from . import binding as J


def linear_schedule(step: int, total_steps: int) -> float:
    """Fraction of the still-masked positions a uniform schedule reveals at this step, so that it
    ends on step `total_steps` at the latest (Section 3.2: the schedule decides how many of the
    masked positions are revealed)."""
    return 1.0 / max(1, total_steps - step + 1)


def decode(state: int, logits_fn, max_steps: int, *, schedule=linear_schedule, n_transfer_dev: int = 0,
           uniforms_fn=None, stream: int = 0) -> dict:
    """Runs the loop on an initialised state.  `schedule(step, max_steps)` -> fraction in [0, 1]
    of each row's examined positions to reveal (None: none); `n_transfer_dev`: device pointer of a
    [B] int32 array of positions to reveal per row and step on top of that (0: none) -- the form a
    block-wise decoder uses, block_size / steps_per_block.  With neither, only the early exit
    finalizes.  `uniforms_fn(step)` -> device pointer of the step's [B, L] uniform numbers for
    sampled tokens (None: argmax).  Returns the number of steps used and the examined count per
    step."""
    examined = []
    steps = 0
    n_active = J.jot_active_count(state)
    while n_active > 0 and steps < max_steps:
        step = steps + 1
        ptr, stride_b, stride_l = logits_fn(step, J.jot_active_list(state), n_active)
        opt = J.JotStepOptions()
        opt.transfer_frac = float(schedule(step, max_steps)) if schedule else 0.0
        opt.n_transfer_dev = n_transfer_dev or None
        if uniforms_fn is not None:
            opt.uniforms_dev = uniforms_fn(step)
        J.jot_step_ex(state, ptr, stride_b, stride_l, opt, stream)
        examined.append(n_active)
        n_active = J.jot_active_count(state)           # Algorithm 1's loop test
        steps = step
    return {"steps": steps, "examined_per_step": examined, "still_masked": n_active}


def decode_overlapped(state: int, forward_fn, max_steps: int, *, schedule=linear_schedule, n_transfer_dev: int = 0,
                      stream: int = 0) -> dict:
    """The same loop with the host's loop test taken off the critical path.  `forward_fn(step)`
    ENQUEUES the denoiser for `step` on `stream` -- it reads the canvas on the device
    (jot_tokens / jot_masked) and needs nothing from the host -- and returns (device pointer,
    stride_b, stride_l) of the logits it will have written.  After enqueueing the finalization
    pass of step n the loop enqueues the forward pass of step n + 1 straight away and only then
    looks, without blocking (jot_active_count_poll), whether step n left anything masked: the GPU
    never waits for the host between steps.  If nothing was left, that last forward pass was
    speculative work the GPU did for nothing; the canvas is the same as decode()'s."""
    examined = []
    n_active = J.jot_active_count(state)
    steps = 0
    if n_active == 0 or max_steps < 1:
        return {"steps": 0, "examined_per_step": examined, "still_masked": n_active, "speculative_forwards": 0}
    ptr, stride_b, stride_l = forward_fn(1)
    wasted = 0
    while True:
        step = steps + 1
        opt = J.JotStepOptions()
        opt.transfer_frac = float(schedule(step, max_steps)) if schedule else 0.0
        opt.n_transfer_dev = n_transfer_dev or None
        J.jot_step_ex(state, ptr, stride_b, stride_l, opt, stream)
        examined.append(n_active)
        steps = step
        if step == max_steps:
            n_active = J.jot_active_count(state)
            break
        ptr, stride_b, stride_l = forward_fn(step + 1)       # before the host knows whether it is needed
        deadline = time.perf_counter() + 5.0
        while True:
            n_active, done = J.jot_active_count_poll(state)
            if done >= step:
                break
            if time.perf_counter() > deadline:               # e.g. a state whose steps the host cannot count
                n_active = J.jot_active_count(state)
                break
        if n_active == 0:                                    # Algorithm 1's loop test, one forward pass late
            wasted = 1
            break
    return {"steps": steps, "examined_per_step": examined, "still_masked": n_active, "speculative_forwards": wasted}


def _synthetic_run(cfg, early_exit: bool, budget: int | None = None, overlapped: bool | None = None) -> dict:
    """One decode of a synthetic workload on cuda:0 (imports the generators of this repository).
    `overlapped`: None = decode() with a stand-in denoiser that writes the rows of the examined
    positions only; False / True = decode() / decode_overlapped() with one that writes the rows of
    every generation position and so needs nothing from the host (the same work in both).
    `budget`: the decoder's step budget T; the workload's own `steps` is the span over which its
    planted tokens converge, so a budget above it models a decoder configured with more steps
    than the sequence needs."""
    import numpy as np
    import torch
    from gen.device import DeviceGenerator
    from gen.trajectory import Trajectory

    if not early_exit:                                   # thresholds no confidence can reach
        cfg = cfg.replace(tau_max=3.0e38, tau_min=3.0e38)
    traj = Trajectory(cfg)
    dgen = DeviceGenerator(cfg, traj.target, traj.rival)
    tokens0, masked0 = traj.initial_canvas()
    p = J.JotParams(B=cfg.B, L=cfg.L, V=cfg.V, dtype=cfg.dtype, conf_mode=cfg.conf_mode, tau_max=cfg.tau_max,
                    tau_min=cfg.tau_min, gamma=cfg.gamma, D=cfg.D, eps=cfg.eps, gen_start=cfg.gen_start,
                    block_size=cfg.block_size)
    nbytes = J.jot_workspace_bytes(p)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    tok = torch.from_numpy(np.ascontiguousarray(tokens0, np.int32)).cuda()
    msk = torch.from_numpy(np.ascontiguousarray(masked0, np.uint8)).cuda()
    stream = torch.cuda.current_stream().cuda_stream
    h = J.jot_init_state(p, ws.data_ptr(), nbytes, tok.data_ptr(), msk.data_ptr(), stream)
    logits = dgen.alloc_logits(poison=False)

    def logits_fn(step, active_dev, n_active):
        T, R = traj.planted(step)
        dgen.set_planted(T, R)
        dgen.fill(logits, step, active_dev, n_active)
        return logits.data_ptr(), cfg.L * cfg.V, cfg.V

    budget = budget or cfg.steps
    kw = {}
    if cfg.block_size > 0:            # block-wise decoder: block_size / steps_per_block positions per row and step
        n_blocks = -(-cfg.n_gen // cfg.block_size)
        per_step = -(-cfg.block_size // max(1, budget // n_blocks))
        nt = torch.full((cfg.B,), per_step, dtype=torch.int32, device="cuda:0")
        kw = dict(schedule=None, n_transfer_dev=nt.data_ptr())
    gen_list = torch.from_numpy(np.flatnonzero(traj.gen).astype(np.int32)).cuda()

    def forward_fn(step):
        T, R = traj.planted(step)
        dgen.set_planted(T, R)
        dgen.fill(logits, step, gen_list.data_ptr(), gen_list.numel())
        return logits.data_ptr(), cfg.L * cfg.V, cfg.V

    t0 = time.perf_counter()
    if overlapped:
        out = decode_overlapped(h, forward_fn, budget, stream=stream, **kw)
    elif overlapped is not None:
        out = decode(h, lambda step, active_dev, n_active: forward_fn(step), budget, stream=stream, **kw)
    else:
        out = decode(h, logits_fn, budget, stream=stream, **kw)
    torch.cuda.synchronize()
    out["seconds_including_the_input_generator"] = time.perf_counter() - t0
    final = J.device_to_host(J.jot_tokens(h), cfg.B * cfg.L, np.int32)
    gen_pos = traj.gen
    out["tokens_equal_to_planted_targets"] = float(np.mean(final[gen_pos] == traj.target[gen_pos]))
    J.jot_release(h)
    return out


def main() -> None:
    from gen.configs import CONFIGS
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--config", type=int, default=2, help="synthetic workload 2-5")
    ap.add_argument("--steps", type=int, default=None,
                    help="steps over which the workload's planted tokens converge (default: the workload's)")
    ap.add_argument("--budget", type=int, default=None, help="the decoder's step budget T (default: twice --steps)")
    ap.add_argument("--batch", type=int, default=None, help="override the batch size")
    ap.add_argument("--overlapped", action="store_true",
                    help="also time the loop that enqueues the next forward pass before it tests the last step")
    args = ap.parse_args()
    cfg = CONFIGS[args.config]
    if args.steps:
        cfg = cfg.replace(steps=args.steps)
    if args.batch:
        cfg = cfg.replace(B=args.batch)
    budget = args.budget or 2 * cfg.steps
    fixed = _synthetic_run(cfg, early_exit=False, budget=budget)
    early = _synthetic_run(cfg, early_exit=True, budget=budget)
    extra = {}
    if args.overlapped:
        again = _synthetic_run(cfg, early_exit=True, budget=budget, overlapped=False)   # both timed on warm code paths
        over = _synthetic_run(cfg, early_exit=True, budget=budget, overlapped=True)
        extra = {"us_per_step_blocking_loop": 1e6 * again["seconds_including_the_input_generator"] / again["steps"],
                 "us_per_step_overlapped_loop": 1e6 * over["seconds_including_the_input_generator"] / over["steps"],
                 "steps_overlapped_loop": over["steps"]}
    print(json.dumps({
        **extra,
        "workload": cfg.name, "B": cfg.B, "generated_positions": cfg.n_gen, "V": cfg.V, "convergence_span": cfg.steps, "step_budget": budget,
        "steps_schedule_only": fixed["steps"], "steps_with_early_exit": early["steps"],
        "step_reduction": fixed["steps"] / max(1, early["steps"]),
        "target_tokens_schedule_only": fixed["tokens_equal_to_planted_targets"],
        "target_tokens_with_early_exit": early["tokens_equal_to_planted_targets"],
        "data": "synthetic trajectories"}))


if __name__ == "__main__":
    main()
