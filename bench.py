#!/usr/bin/env python3
"""Throughput of the JoT finalization pass on one MI355X.

A "step" is one jot_step() -- vocabulary reduction of every examined position, confidence,
spatial threshold, decision, commit and compaction -- followed by the jot_active_count() a decode
loop needs for its termination test.  The workload is the largest synthetic configuration
(B=64, 1024 generated positions after a 256-token prompt, V=152064, fp32 logits, the paper's
ratio signal with tau_max=90, tau_min=1, gamma=0.5, D=8), decoded from its first step; the
logits of the timed steps are generated on the device beforehand and are resident in HBM.

Prints one JSON line.  `value` = sum over the K timed steps of (examined positions x V) / wall time.
`step1` is the first of them alone (the largest examined set), `whole_loop` the same decode carried
on to its end (every step timed the same way; its logits are generated between the timed segments).
`roofline` is for the vocabulary-reduction kernel (the only kernel that touches the logits):
bytes = examined positions x V x element size, duration from HIP events around that kernel.
`cpu_baseline` is the double-precision CPU oracle timed on this machine on a sample of the same
step-1 rows.  Workloads whose step reads no more than 512 MB are timed with the caches evicted
before every step (a 1 GiB fill), so that their GB/s are HBM figures too.
"""
import argparse
import ctypes
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
FLUSH_BELOW_BYTES = 512 << 20   # steps that read less than this are timed with evicted caches
FLUSH_BYTES = 1 << 30

# HBM traffic of the vocabulary reduction from rocprofv3 counters, as a ratio to the algorithmic
# bytes (examined positions x V x element size) of the same launches: (FETCH_SIZE x 2.000 +
# WRITE_SIZE x 1.000) KiB, factors from a plain 1 GiB copy kernel in the same runs; see
# profiles/vocab_reduce_cfg5_hbm_traffic.md and profiles/vocab_reduce_bf16_hbm_traffic.md.  Valid
# for the kernel sources with these hashes and for these workloads and logit types; otherwise
# bench.py reports null.
MEASURED_TRAFFIC = {
    "hbm_bytes_per_algorithmic_byte": {(5, "f32"): 1.00060, (5, "bf16"): 1.00088, (3, "bf16"): 1.00085,
                                       (4, "bf16"): 1.00137, (2, "bf16"): 1.00311},
    "sha256": {"jot_vocab_reduce.h": "ec222316785395e737ad2d6907c8b24e1746203b62f883bb672246bb4554231d",
               "jot_device.h": "d4fb409aab4572866a739d578d94a361c1d9edb11176acebcc835d57ae63b89c"},
}


def measured_traffic_ratio(config: int, dtype: str):
    ratio = MEASURED_TRAFFIC["hbm_bytes_per_algorithmic_byte"].get((config, dtype))
    if ratio is None:
        return None
    for name, want in MEASURED_TRAFFIC["sha256"].items():
        path = os.path.join(ROOT, "paper_2602_11133_amd", "csrc", name)
        with open(path, "rb") as f:
            if hashlib.sha256(f.read()).hexdigest() != want:
                return None
    return float(ratio)


def host_threads() -> int:
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def load_probe():
    from paper_2602_11133_amd import build as jb
    if not os.path.exists(jb.PROBE_LIB):
        raise RuntimeError(f"{jb.PROBE_LIB} is missing: run __graft_entry__.build() first")
    lib = ctypes.CDLL(jb.PROBE_LIB)
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    lib.jot_probe_copy.argtypes, lib.jot_probe_copy.restype = [vp, vp, i64, vp], ctypes.c_int
    lib.jot_probe_read.argtypes, lib.jot_probe_read.restype = [vp, i64, vp, vp], ctypes.c_int
    lib.jot_probe_read_rows.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, i64, i64, i64, ctypes.c_int32, vp, vp]
    lib.jot_probe_read_rows.restype = ctypes.c_int
    return lib


def probe_copy_only(torch, reps: int):
    """Plain copy of 1 GiB, `reps` times: calibration target for FETCH_SIZE / WRITE_SIZE."""
    lib = load_probe()
    n = 1 << 30
    src = torch.zeros(n, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    st = torch.cuda.current_stream().cuda_stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        assert lib.jot_probe_copy(src.data_ptr(), dst.data_ptr(), n, st) == 0
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    print(json.dumps({"probe": "copy", "bytes_read_per_launch": n, "bytes_written_per_launch": n,
                      "launches": reps, "GBps_read_plus_write": 2 * n * reps / dt / 1e9}))


def read_probe(torch, buf, reps=3) -> float:
    """Best-of-reps GB/s of a plain read-only grid-stride kernel over one logits buffer (a
    reference point for the reduction, not a ceiling: the reduction itself may stream faster)."""
    lib = load_probe()
    nbytes = buf.numel() * buf.element_size() // 32768 * 32768
    out = torch.zeros(1, dtype=torch.int32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    best = 0.0
    for _ in range(reps + 1):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        assert lib.jot_probe_read(buf.data_ptr(), nbytes, out.data_ptr(), st) == 0
        e1.record()
        torch.cuda.synchronize()
        best = max(best, nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    return best


def read_probe_rows(torch, buf, cfg, reps=3) -> float:
    """Best-of-reps GB/s of a read-only kernel that streams the generated positions' rows of one
    logits buffer row by row, in the launch shape of the fp32 reduction (one workgroup per CU)."""
    lib = load_probe()
    row = cfg.V * cfg.elem_bytes
    if row % 16:
        return float("nan")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    out = torch.zeros(1, dtype=torch.int32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    nbytes = cfg.B * cfg.n_gen * row
    best = 0.0
    for _ in range(reps + 1):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        assert lib.jot_probe_read_rows(buf.data_ptr() + cfg.gen_start * row, cfg.B, cfg.n_gen, cfg.L * row, row, row,
                                       cus, out.data_ptr(), st) == 0
        e1.record()
        torch.cuda.synchronize()
        best = max(best, nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    return best


def cpu_baseline(cfg, traj, sample_rows: int):
    """The oracle's evaluation of step 1 on the first `sample_rows` batch rows, all host threads."""
    from gen.host import HostGenerator
    from oracle import jot_oracle as O
    threads = host_threads()
    rows_b = list(range(min(sample_rows, cfg.B)))
    tokens, masked = traj.initial_canvas()

    def oracle_params(c):
        return O.OracleParams(B=c.B, L=c.L, V=c.V, dtype=c.dtype, conf_mode=c.conf_mode, tau_max=c.tau_max,
                              tau_min=c.tau_min, gamma=c.gamma, D=c.D, eps=c.eps, gen_start=c.gen_start,
                              block_size=c.block_size)

    sub = cfg.replace(B=len(rows_b))
    st = O.OracleState.init(oracle_params(sub), tokens[rows_b], masked[rows_b], threads=threads)
    act = st.active_list()
    T, R = traj.planted(1)
    rows = HostGenerator(cfg, traj.target, traj.rival, threads).rows(1, act, T, R)   # untimed
    t0 = time.perf_counter()
    rec = st.evaluate(rows)
    dt = time.perf_counter() - t0
    assert rec.active.size == act.size
    # the same oracle on one thread, on the first batch row only
    one = O.OracleState.init(oracle_params(cfg.replace(B=1)), tokens[:1], masked[:1], threads=1)
    n1 = one.active_list().size
    t0 = time.perf_counter()
    one.evaluate(rows[:n1])
    dt1 = time.perf_counter() - t0
    return {"value": act.size * cfg.V / dt, "unit": "positions·vocab/s", "cores": threads, "kind": "oracle",
            "sample": f"step 1, batch rows 0-{len(rows_b) - 1} ({act.size} positions x V={cfg.V}), "
                      f"{dt:.2f} s wall on {threads} threads", "seconds": dt,
            "single_thread_value": n1 * cfg.V / dt1,
            "single_thread_sample": f"step 1, batch row 0 ({n1} positions), {dt1:.2f} s on 1 thread"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, help="workload 1-5 (default: the largest)")
    ap.add_argument("--cpu-sample-rows", type=int, default=16, help="batch rows timed on the CPU oracle")
    ap.add_argument("--dtype", choices=["f32", "bf16"], default=None,
                    help="override the logit type of the workload (changes the workload: for tuning)")
    ap.add_argument("--schedule", choices=["none", "linear"], default="none",
                    help="also apply a transfer schedule each step: 'linear' reveals "
                         "remaining/steps_left of every row's examined positions (jot_step_scheduled)")
    ap.add_argument("--sample", action="store_true",
                    help="sampling-based finalization (jot_step_sampled with uniform numbers drawn beforehand)")
    ap.add_argument("--graph", action="store_true",
                    help="capture each step's launches into a HIP graph once and replay them in the timed loop")
    ap.add_argument("--kl", type=float, default=None, metavar="TAU_KL",
                    help="also apply the KL stability rule with this threshold (the reduction then streams the "
                         "previous step's logits too; steps must fit the resident buffers)")
    ap.add_argument("--no-loop", action="store_true", help="do not carry the decode on to its end after the timed steps")
    ap.add_argument("--no-flush", action="store_true", help="never evict the caches before a timed step")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-probe", action="store_true")
    ap.add_argument("--probe-copy", type=int, default=0, metavar="N",
                    help="only run the plain 1 GiB copy kernel N times (counter calibration) and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: one GPU only (the pass would shard over batch rows with no exchange; "
              "no multi-GPU figure is produced). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the finalization pass has no CPU path", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.probe_copy:
        probe_copy_only(torch, args.probe_copy)
        return

    import paper_2602_11133_amd as J
    from paper_2602_11133_amd.session import JotSession
    from gen.configs import CONFIGS, F32
    from gen.device import DeviceGenerator
    from gen.trajectory import Trajectory

    cfg = CONFIGS[args.config]
    if args.dtype is not None:
        cfg = cfg.replace(dtype=0 if args.dtype == "f32" else 1, name=cfg.name + "_as_" + args.dtype)
    dtype_name = "f32" if cfg.dtype == F32 else "bf16"
    K, W = args.steps, args.warmup
    traj = Trajectory(cfg)
    dgen = DeviceGenerator(cfg, traj.target, traj.rival)
    tokens0, masked0 = traj.initial_canvas()
    params = J.JotParams(B=cfg.B, L=cfg.L, V=cfg.V, dtype=cfg.dtype, conf_mode=cfg.conf_mode, tau_max=cfg.tau_max,
                         tau_min=cfg.tau_min, gamma=cfg.gamma, D=cfg.D, eps=cfg.eps, gen_start=cfg.gen_start,
                         block_size=cfg.block_size)
    esz = cfg.elem_bytes
    buf_bytes = cfg.B * cfg.L * cfg.V * esz
    step1_bytes = int(masked0.sum() if cfg.block_size == 0 else cfg.B * min(cfg.block_size, cfg.n_gen)) * cfg.V * esz
    flush = (not args.no_flush) and step1_bytes <= FLUSH_BELOW_BYTES
    flush_buf = torch.empty(FLUSH_BYTES, dtype=torch.uint8, device="cuda") if flush else None
    free, _total = torch.cuda.mem_get_info()
    # segments no longer than the library's ring of kernel timings (JOT_PROFILE_RING steps)
    resident = int(max(1, min(max(K, 16), 64, (free * 0.85) // buf_bytes)))
    bufs = [dgen.alloc_logits(poison=False) for _ in range(resident)]
    stream = torch.cuda.current_stream().cuda_stream
    torch.manual_seed(cfg.seed)
    uniforms = [torch.rand((cfg.B, cfg.L), dtype=torch.float32, device="cuda") for _ in range(resident)] \
        if args.sample else None

    def fill_segment(g, first_step, count):
        """(untimed) logits of steps first_step .. first_step+count-1 for every position that is
        still examined when the segment starts (a superset of what each step will read)."""
        n_act = g.active_count()
        for k in range(count):
            T, R = traj.planted(first_step + k)
            dgen.set_planted(T, R)
            dgen.fill(bufs[k], first_step + k, J.jot_active_list(g.h), n_act)
        torch.cuda.synchronize()

    if args.kl is not None and (max(K, W) > resident or resident < 2):
        raise SystemExit("--kl needs every step's logits resident, and at least two steps: change --steps / --warmup")

    def enqueue_step(g, k, step_no, st):
        frac = 1.0 / max(1, cfg.steps - step_no + 1) if args.schedule == "linear" else 0.0
        if args.kl is not None:
            opt = J.JotStepOptions()
            opt.transfer_frac = frac
            if args.sample:
                opt.uniforms_dev = uniforms[k].data_ptr()
            opt.enable_kl = 1
            # step 1 has no history, its previous-step operand is never used for a decision: hand it a
            # buffer other than its own, so that the two streams do not share cache lines
            opt.prev_logits_dev = bufs[k - 1 if k > 0 else resident - 1].data_ptr()
            opt.kl_threshold, opt.kl_min_prob = args.kl, 0.0
            J.jot_step_ex(g.h, bufs[k].data_ptr(), cfg.L * cfg.V, cfg.V, opt, st)
        elif args.sample:
            J.jot_step_sampled(g.h, bufs[k].data_ptr(), cfg.L * cfg.V, cfg.V, 0, frac, uniforms[k].data_ptr(), st)
        elif args.schedule == "linear":
            J.jot_step_scheduled(g.h, bufs[k].data_ptr(), cfg.L * cfg.V, cfg.V, 0, frac, st)
        else:
            J.jot_step(g.h, bufs[k].data_ptr(), cfg.L * cfg.V, cfg.V, st)

    def capture_graphs(g):
        """One graph per resident logits buffer (the buffer address is part of the launch)."""
        graphs = []
        side = torch.cuda.Stream()
        for k in range(resident):
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=side):
                enqueue_step(g, k, 1, torch.cuda.current_stream().cuda_stream)
            graphs.append(gr)
        torch.cuda.synchronize()
        return graphs

    def decode(g, first_step, n_steps, timed, graphs=None):
        """Runs steps first_step .. first_step+n_steps-1 (or until nothing is left) in segments of
        `resident`; returns (seconds, [A_n], [reduce ms], [seconds per step])."""
        total, examined, kms, per_step = 0.0, [], [], []
        done = 0
        while done < n_steps:
            seg = min(resident, n_steps - done)
            fill_segment(g, first_step + done, seg)
            a_prev = g.active_count()
            if a_prev == 0:
                break
            ran = 0
            torch.cuda.synchronize()
            t_seg = time.perf_counter()
            for k in range(seg):
                if flush:
                    flush_buf.zero_()
                    torch.cuda.synchronize()
                t0 = time.perf_counter()
                if graphs:
                    graphs[k].replay()
                else:
                    enqueue_step(g, k, first_step + done + k, stream)
                a_next = J.jot_active_count(g.h)        # the decode loop's termination test
                per_step.append(time.perf_counter() - t0)
                examined.append(a_prev)
                a_prev = a_next
                ran += 1
                if a_next == 0:
                    break
            torch.cuda.synchronize()
            # without eviction the K steps are timed as one bracket, synchronised on both sides
            total += sum(per_step[-ran:]) if flush else time.perf_counter() - t_seg
            if timed and not graphs:
                kms += [J.jot_profile_read(g.h, first_step + done + k) for k in range(ran)]
            done += ran
            if a_prev == 0:
                break
        return total, examined, kms, per_step

    # warm-up on a state of its own, then a fresh state for the timed steps
    if W > 0:
        gw = JotSession(params, tokens0, masked0)
        decode(gw, 1, W, timed=False)
        gw.close()
    g = JotSession(params, tokens0, masked0)
    J.jot_profile_enable(g.h, True)
    graphs = capture_graphs(g) if args.graph else None
    seconds, examined, kms, per_step = decode(g, 1, K, timed=True, graphs=graphs)
    assert len(examined) == K, "the decode ended before the timed steps did: use fewer --steps"

    kl_factor = 2.0 if args.kl is not None else 1.0      # the same rows of the previous step's logits as well
    elems = float(sum(examined)) * cfg.V
    value = elems / seconds
    k_bytes = elems * esz * kl_factor / K           # algorithmic bytes per launch (average)
    if not kms:                                     # --graph: no events inside the graph; whole-step time instead
        kms = [seconds / K * 1e3] * K
    k_sec = sum(kms) * 1e-3 / K                     # average launch duration
    achieved = k_bytes / k_sec / 1e9
    plain = args.schedule == "none" and not args.sample and not args.graph and args.kl is None
    ratio = measured_traffic_ratio(args.config, dtype_name) if plain else None

    def rate_record(n_examined, sec, kernel_ms):
        b = float(n_examined) * cfg.V * esz * kl_factor
        return {"examined_positions": int(n_examined), "ms": sec * 1e3, "positions_vocab_per_s": n_examined * cfg.V / sec,
                "GBps_active_logits": b / sec / 1e9, "vocab_reduce_ms": kernel_ms,
                "vocab_reduce_GBps": (b / (kernel_ms * 1e-3) / 1e9) if kernel_ms else None}

    step1 = rate_record(examined[0], per_step[0], kms[0])

    whole = None
    if not args.no_loop and not args.graph and args.kl is None:
        # carry the same decode on to its end (or to the configured number of steps)
        sec2, ex2, kms2, _ = decode(g, K + 1, max(0, cfg.steps - K), timed=True)
        all_ex, all_sec, all_kms = examined + ex2, seconds + sec2, kms + kms2
        b = float(sum(all_ex)) * cfg.V * esz
        whole = {"steps": len(all_ex), "examined_positions_total": int(sum(all_ex)), "ms_per_step": all_sec / len(all_ex) * 1e3,
                 "positions_vocab_per_s": sum(all_ex) * cfg.V / all_sec, "GBps_active_logits": b / all_sec / 1e9,
                 "pct_of_hbm_peak": 100.0 * b / all_sec / 1e9 / HBM_PEAK_GBPS,
                 "vocab_reduce_GBps": b / (sum(all_kms) * 1e-3) / 1e9,
                 "still_active_after": int(g.active_count()),
                 "examined_every_32_steps": [int(a) for a in all_ex[::32]]}
    anomalies = J.jot_anomaly_count(g.h)
    remaining = g.active_count()
    g.close()

    out = {
        "metric": "active positions·vocab/s per jot_step",
        "value": value, "unit": "positions·vocab/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": seconds / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype_name, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B}, L={cfg.L} ({cfg.gen_start} prompt + {cfg.n_gen} generated), "
                               f"V={cfg.V}, decode steps 1..{K}", "examined_positions_per_step": examined,
                   "conf_mode": cfg.conf_mode, "tau_max": cfg.tau_max, "tau_min": cfg.tau_min,
                   "gamma": cfg.gamma, "D": cfg.D, "block_size": cfg.block_size, "schedule": args.schedule,
                   "sampled_tokens": bool(args.sample), "hip_graph": bool(args.graph), "kl_threshold": args.kl,
                   "resident_logit_buffers": resident, "caches_evicted_before_each_step": bool(flush),
                   "still_active_after": remaining, "anomalies": anomalies},
        "hbm_GBps_active_logits": k_bytes * K / seconds / 1e9,
        "pct_of_hbm_peak": 100.0 * k_bytes * K / seconds / 1e9 / HBM_PEAK_GBPS,
        "step1": step1,
        "whole_loop": whole,
        "roofline": {"bound": "hbm",
                     "kernel": "jot_vocab_reduce_kernel<KL>" if args.kl is not None else "jot_vocab_reduce_kernel",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": ratio * k_bytes if ratio is not None else None,
                     "traffic_per_algorithmic_byte": ratio,
                     "bytes_per_launch": k_bytes, "avg_launch_ms": k_sec * 1e3, "launch_ms": kms},
    }
    if not args.no_probe:
        out["read_only_probe_GBps"] = read_probe(torch, bufs[0])
        out["read_only_probe_same_launch_shape_GBps"] = read_probe_rows(torch, bufs[0], cfg)
    del bufs
    torch.cuda.empty_cache()
    if not args.no_cpu:
        cb = cpu_baseline(cfg, traj, args.cpu_sample_rows)
        cb["gpu_over_cpu"] = value / cb["value"]
        out["cpu_baseline"] = cb
    print(json.dumps(out))


if __name__ == "__main__":
    main()
