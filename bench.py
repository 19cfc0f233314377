#!/usr/bin/env python3
"""Benchmark of the batched Go environment step on one MI355X.

One "step" is one pass of the whole hot path over the batch: draw a uniform random legal action for every
game, apply it (legality gate, placement, capture, ko, history, termination + area score, auto-reset), and
emit the next legal mask [B][362], observation [B][19][19][17], rewards and terminated flags.  The default
workload is the headline configuration: 19x19, 16384 games, seed 3, auto-reset.

What is timed.  Every run first plays an UNTIMED pre-roll of `preroll` plies (workloads.py; 600 for the headline
configuration) through the rollout kernel, whatever --warmup says, so that the timed plies lie in the dense,
desynchronised regime of the workload and not on empty boards; then --warmup launches of the timed path; then
exactly --steps launches between two events (config.timed_ply_window names them).  The same plies are then
repeated with the outputs rotating over several slices (more bytes than the 256 MB memory-side cache holds), and a
plain 16-byte-store fill of the same output bytes is timed both ways as the practical ceiling.

Prints ONE JSON line.  Inputs are synthetic by construction: the paper's own benchmark is random play from the
empty board (Sec. 4.1).  `--ceilings` prints the reference measurements (fill, emit-only kernel, copy, launch gap,
slice sweep) instead; `--config k` selects another configuration of workloads.py.
"""
import argparse
import json
import math
import os
import re
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published
MEMORY_SIDE_CACHE = 256 << 20


def algorithmic_bytes_per_ply(N, with_obs):
    """Bytes one ply must move whatever the implementation: action in, packed positions in/out, scalars,
    legal mask and observation out.  19x19 with observation: 7272 B."""
    P = N * N
    packed = (P + 7) // 8                      # one colour of one position, bit-packed
    total = 4                                  # action
    total += (7 * 2 * packed) if with_obs else 2 * packed   # positions read (7 older ones feed the observation)
    total += 24                                # per-game scalars read + written
    total += 2 * packed                        # new position written
    total += P + 1                             # legal mask bytes
    total += P * 17 if with_obs else 0         # observation bytes
    total += 9                                 # rewards[2] + terminated
    return total


def read_traffic(path):
    """HBM bytes per launch of the dominant kernel, taken from the committed rocprofv3 counter summary."""
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def hex_bytes_per_ply(with_obs):
    """The same accounting for Hex 11x11: action, packed position in/out, scalars, 122 mask bytes, 484 observation
    bytes, rewards + terminated.  707 B with the observation."""
    return algorithmic_bytes_per_ply_generic(11, 4 if with_obs else 0, history_reads=1)


def algorithmic_bytes_per_ply_generic(N, planes, history_reads):
    P = N * N
    packed = (P + 7) // 8
    return 4 + history_reads * 2 * packed + 24 + 2 * packed + (P + 1) + P * planes + 9


def rotation_slices(out_bytes):
    """Output slices so that one rotation writes well beyond the memory-side cache (>= 800 MB), 2..8."""
    return int(min(8, max(2, math.ceil((800 << 20) / max(1, out_bytes)))))


def default_steps(cfg):
    """Timed plies when --steps is not given: the configuration's own count with auto-reset; a quarter of the game
    length without (the timed window must end before the games do)."""
    return cfg.steps if cfg.auto_reset else max(20, cfg.steps // 4)


def timed(fn, n):
    """ms per call of n back-to-back calls of fn(i), between two events on the current stream."""
    import torch

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(n):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / max(1, n)


def device_copy_gbs(nbytes):
    """A plain device copy (read + write counted) of as many bytes as one step writes; also the kernel of known size
    that calibrates the HBM counters."""
    import torch

    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(5): dst.copy_(src)
    ms = timed(lambda i: dst.copy_(src), 50)
    return 2 * nbytes / (ms * 1e-3) / 1e9


def fill_ceiling(nbytes, slices, reps=200):
    """Plain fill of `nbytes` with 16-byte stores, back-to-back launches: into one buffer (lines stay in the memory-side
    cache) and rotating over `slices` buffers (every line has to reach DRAM)."""
    import torch

    import paper_2303_17503_amd as pg

    n16 = nbytes // 16 * 16
    bufs = [torch.empty(n16, dtype=torch.uint8, device="cuda") for _ in range(slices)]
    for b in bufs: pg.fill_probe(b, 1)
    ms_in = timed(lambda i: pg.fill_probe(bufs[0], i), reps)
    ms_rot = timed(lambda i: pg.fill_probe(bufs[i % slices], i), reps)
    return {"bytes": n16, "slices": slices, "in_place_ms": ms_in, "in_place_gbs": n16 / (ms_in * 1e-3) / 1e9,
            "rotating_ms": ms_rot, "rotating_gbs": n16 / (ms_rot * 1e-3) / 1e9}


def launch_gap_us(reps=2000):
    """Time per launch of back-to-back empty kernels on one stream (enqueued by a C loop, so the host's per-call
    cost in Python does not enter)."""
    import paper_2303_17503_amd as pg

    pg.empty_probe(50)
    return timed(lambda i: pg.empty_probe(reps), 1) * 1e3 / reps


def cpu_baseline(cfg, pre, plies, n_threads, envs_per_thread, superko=False, min_seconds=1.0):
    """The CPU oracle as it stands on a fixed sample of the same workload, independent of --steps: the first
    n_threads*envs_per_thread environments of the configuration, pre-rolled (untimed) to the ply window the GPU times,
    then `plies` timed plies; the sample is repeated from scratch until it has run for min_seconds.  Sharded over host
    threads (the C calls release the GIL).  Returns (one-thread rate, all-threads rate, repetitions)."""
    import numpy as np

    import oracle
    import workloads

    oracle.lib()
    hx = None
    if cfg.game == "hex":
        from oracle import hex as hx
        hx.lib()
    spent = [0.0] * n_threads

    def work(i):
        ids = np.arange(i * envs_per_thread, (i + 1) * envs_per_thread, dtype=np.int32)
        start = workloads.start_times(cfg, ids) if cfg.game == "go" else None
        if cfg.game == "hex":
            o = hx.HexOracle(envs_per_thread, cfg.board_size, seed=cfg.seed, auto_reset=cfg.auto_reset, env_ids=ids)
            step = lambda t: o.step(o.random_actions(cfg.seed, t))
        else:
            o = oracle.GoOracle(envs_per_thread, cfg.board_size, seed=cfg.seed, komi_x2=cfg.komi_x2, auto_reset=cfg.auto_reset, env_ids=ids,
                                superko=superko)
            step = lambda t: o.step(o.random_actions(cfg.seed, t, start))
        for t in range(pre):
            step(t)
        t0 = time.perf_counter()
        for t in range(pre, pre + plies):
            step(t)
        spent[i] = time.perf_counter() - t0

    def run(k):
        """rate of k threads: env-plies of the timed windows / the slowest thread's timed seconds, repeated to min_seconds"""
        total, secs, reps = 0, 0.0, 0
        while secs < min_seconds and reps < 50:
            th = [threading.Thread(target=work, args=(i,)) for i in range(k)]
            for x in th: x.start()
            for x in th: x.join()
            total += k * envs_per_thread * plies
            secs += max(spent[:k])
            reps += 1
        return total / secs, reps

    single, r1 = run(1)
    multi, rk = run(n_threads) if n_threads > 1 else (single, r1)
    return single, multi, (r1, rk)


def bound_statement(kern_us, floor_us, fill_us, waves_per_simd):
    """Which limit binds, by a stated rule on quantities measured in this run (the counters are in profiles/)."""
    rule = ("latency if kernel <= 1.5 x the ply of ONE wavefront (launch gap + load -> rules -> emit -> store of a single "
            "wavefront); else hbm if a plain fill of the same output bytes takes >= 0.6 of the kernel; else valu issue")
    if kern_us <= 1.5 * floor_us:
        b = "launch gap + serial latency of one wavefront"
    elif fill_us / kern_us >= 0.6:
        b = "hbm (output stores)"
    else:
        b = "valu issue"
    return {"bound_by": b, "rule": rule, "one_wavefront_ply_us": floor_us, "fill_of_outputs_us": fill_us, "wavefronts_per_simd": waves_per_simd}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed launches (default: the configuration's plies; 2000 for the headline)")
    ap.add_argument("--warmup", type=int, default=20, help="untimed launches of the timed path right before the timed region (the pre-roll "
                                                           "that moves the games into their steady regime is separate and always played)")
    ap.add_argument("--game", choices=["go", "hex"], default="go", help="go: the headline workload; hex: the second workload (Hex 11x11)")
    ap.add_argument("--config", type=int, default=None, help="index into workloads.CONFIGS (default 3 = headline) or, with --game hex, "
                                                             "into workloads.HEX_CONFIGS (default 2)")
    ap.add_argument("--mode", choices=["fused", "separate", "rollout"], default="fused",
                    help="fused: one launch per ply, the step kernel also draws the next action (headline); separate: sampler kernel + "
                         "step kernel per ply; rollout: --rollout-len plies per launch with the state kept in registers")
    ap.add_argument("--rollout-len", type=int, default=50, help="plies per launch in rollout mode")
    ap.add_argument("--rollout-slices", type=int, default=1, help="trajectory slices the rollout writes to (1 = overwrite one set of buffers)")
    ap.add_argument("--superko", type=int, default=0, choices=[0, 1, 2], help="Go only: positional superko, 2 = honoured by the legal mask (the rule "
                                                                              "proper), 1 = enforced when the move is played (not the headline metric)")
    ap.add_argument("--line-padded", action="store_true", help="Go only: mask and observation pitches rounded up to 128-byte lines (not the "
                    "paper's dense tensors, hence not the headline: the layout for outputs that have to reach DRAM)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-obs", action="store_true", help="do not emit the observation (not the headline metric)")
    ap.add_argument("--ceilings", action="store_true", help="print the reference measurements of this configuration instead of the benchmark line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (games are independent; more GPUs would shard the batch "
              "with no communication); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.game == "hex":
        cfg = workloads.HEX_CONFIGS[2 if args.config is None else args.config]
    else:
        cfg = workloads.CONFIGS[3 if args.config is None else args.config]
    if args.steps is None:
        args.steps = default_steps(cfg)
    pre = cfg.warmup_max + cfg.preroll
    if not cfg.auto_reset and pre + args.warmup + 2 * args.steps > cfg.steps:
        print(f"bench.py: {cfg.name} has no auto-reset and ends after {cfg.steps} plies; pre-roll {pre} + warm-up {args.warmup} + "
              f"2 x {args.steps} timed plies (in place, then rotating) do not fit", file=sys.stderr)
        sys.exit(2)
    if args.ceilings:
        return ceilings(args, cfg)
    if args.game == "hex":
        return bench_hex(args, cfg)
    return bench_go(args, cfg)


def go_pitches(N, line_padded):
    """(mask pitch, observation pitch) in bytes: dense, or rounded up to 128-byte lines."""
    P = N * N
    return ((P + 1 + 127) // 128 * 128, (P * 17 + 127) // 128 * 128) if line_padded else (P + 1, P * 17)


def go_rollout_buffers(torch, S, B, pitches, with_obs):
    return dict(actions=torch.empty((S, B), dtype=torch.int32, device="cuda"),
                rewards=torch.empty((S, B, 2), dtype=torch.float32, device="cuda"),
                terminated=torch.empty((S, B), dtype=torch.uint8, device="cuda"),
                mask=torch.empty((S, B, pitches[0]), dtype=torch.uint8, device="cuda"),
                obs=torch.empty((S, B, pitches[1]), dtype=torch.uint8, device="cuda") if with_obs else None)


class GoStepper:
    """The one-launch-per-ply path on a GoEnv: pre-roll through the rollout kernel, then step_sample (fused) or
    step + random_actions (separate) with launch index t; acts[t & 1] holds the actions of launch t."""

    def __init__(self, cfg, B, with_obs, fused=True, superko=False, line_padded=False):
        import torch

        import paper_2303_17503_amd as pg
        import workloads

        self.torch, self.cfg, self.B, self.fused = torch, cfg, B, fused
        N = cfg.board_size
        self.env = pg.GoEnv(B, N, seed=cfg.seed, komi_x2=cfg.komi_x2, auto_reset=cfg.auto_reset, line_padded=line_padded)
        if superko:
            self.env.enable_superko(int(superko))
        ids = None if B == cfg.batch else list(range(B))
        start = workloads.start_times(cfg, ids)
        self.start = None if start is None else torch.as_tensor(start, device="cuda")
        self.mask = self.env.new_mask()
        self.obs = self.env.new_obs() if with_obs else None
        self.rew = torch.zeros((B, 2), dtype=torch.float32, device="cuda")
        self.term = torch.zeros(B, dtype=torch.uint8, device="cuda")
        self.env.bind_outputs(self.mask, self.obs, self.rew, self.term)
        self.acts = [torch.empty(B, dtype=torch.int32, device="cuda") for _ in range(2)]
        self.t = 0
        self.rollout_ok = True    # the pre-roll goes through the rollout kernel

    def preroll(self, plies):
        if plies and not self.rollout_ok:
            self.env.random_actions(self.cfg.seed, self.t, self.start, out=self.acts[self.t & 1])
            self.run(plies)
            return
        if plies:
            self.env.rollout(plies, self.cfg.seed, self.t, start_t=self.start)
            self.t += plies
        self.env.random_actions(self.cfg.seed, self.t, self.start, out=self.acts[self.t & 1])

    def step_once(self):
        t, seed = self.t, self.cfg.seed
        if self.fused:
            self.env.step_sample(self.acts[t & 1], seed, t + 1, self.start, out=self.acts[(t + 1) & 1])
        else:
            self.env.step(self.acts[t & 1])
            self.env.random_actions(seed, t + 1, self.start, out=self.acts[(t + 1) & 1])
        self.t = t + 1

    def run(self, n):
        for _ in range(n):
            self.step_once()

    def run_rotating(self, n, masks, obss):
        S = len(masks)
        for i in range(n):
            self.env.set_output_buffers(masks[i % S], None if obss is None else obss[i % S], self.rew, self.term)
            self.step_once()
        self.env.set_output_buffers(self.mask, self.obs, self.rew, self.term)


def bench_go(args, cfg):
    import torch

    import paper_2303_17503_amd as pg

    B, N, seed = cfg.batch, cfg.board_size, cfg.seed
    K, Wm = args.steps, args.warmup
    with_obs = not args.no_obs
    P = N * N
    pre = cfg.warmup_max + cfg.preroll     # plies before the timed path starts: configuration 4's own warm-up, then the pre-roll
    pitches = go_pitches(N, args.line_padded)
    out_bytes = B * (pitches[0] + (pitches[1] if with_obs else 0))
    S_rot = rotation_slices(out_bytes)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    dram = None
    seg_ms = []

    if args.mode == "rollout":
        S, Lr = args.rollout_slices, args.rollout_len
        assert K % Lr == 0, "--steps must be a multiple of --rollout-len"
        env = pg.GoEnv(B, N, seed=seed, komi_x2=cfg.komi_x2, auto_reset=cfg.auto_reset, line_padded=args.line_padded)
        if args.superko:
            env.enable_superko(int(args.superko))
        import workloads
        start = workloads.start_times(cfg)
        start_dev = None if start is None else torch.as_tensor(start, device="cuda")
        bufs = go_rollout_buffers(torch, S, B, pitches, with_obs)
        env.rollout(pre + Wm, seed, 0, start_t=start_dev, slices=S, **bufs)
        ev0.record(); ev1.record()                # torch creates the HIP events at their first record: not inside the timed region
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for i in range(K // Lr):
            env.rollout(Lr, seed, pre + Wm + i * Lr, start_t=start_dev, slices=S, **bufs)
        ev1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        kern_ms = ev0.elapsed_time(ev1) / K       # per ply: the launch covers rollout_len plies
        kname = "go_rollout_kernel<%d>" % N
        if S == 1:
            bufs_r = go_rollout_buffers(torch, S_rot, B, pitches, with_obs)
            ms = timed(lambda i: env.rollout(Lr, seed, pre + Wm + K + i * Lr, start_t=start_dev, slices=S_rot, **bufs_r), max(1, K // Lr)) / Lr
            dram = {"slices": S_rot, "kernel_ms": ms}
            del bufs_r
    else:
        st = GoStepper(cfg, B, with_obs, fused=(args.mode == "fused"), superko=args.superko, line_padded=args.line_padded)
        st.preroll(pre)
        st.run(Wm)
        first = st.t
        # the timed region, cut into five segments by events on the same stream (median and best segment are reported too)
        # (only when there are enough launches that the four extra event records between them do not matter)
        nseg = 5 if K >= 100 else 1
        cuts = [K * i // nseg for i in range(nseg + 1)]
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(nseg - 1)]
        for e in [ev0, ev1] + marks:              # torch creates the HIP events at their first record: not inside the timed region
            e.record()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for i in range(nseg):
            st.run(cuts[i + 1] - cuts[i])
            if i < nseg - 1: marks[i].record()
        ev1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        evs = [ev0] + marks + [ev1]
        seg_ms = [evs[i].elapsed_time(evs[i + 1]) / max(1, cuts[i + 1] - cuts[i]) for i in range(5)] if nseg == 5 else []
        kern_ms = ev0.elapsed_time(ev1) / K   # fused: K launches of the one kernel back to back on the stream the events are on
        if args.mode == "separate":           # the step kernel alone, an event pair around each launch
            n_ev = min(K, 500)
            pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ev)]
            for a, b in pairs:
                t = st.t
                a.record(); st.env.step(st.acts[t & 1]); b.record()
                st.env.random_actions(seed, t + 1, st.start, out=st.acts[(t + 1) & 1])
                st.t = t + 1
            torch.cuda.synchronize()
            kern_ms = sum(a.elapsed_time(b) for a, b in pairs) / n_ev
        kname = "go_step_superko_kernel<%d>" % N if args.superko else "go_step_kernel<%d,%s>" % (N, "true" if args.mode == "fused" else "false")
        # the same path, the next K plies, with mask and observation rotating over S_rot slices
        masks = [st.env.new_mask() for _ in range(S_rot)]
        obss = [st.env.new_obs() for _ in range(S_rot)] if with_obs else None
        st.run_rotating(min(K, 2 * S_rot), masks, obss)
        torch.cuda.synchronize()
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        r0.record(); st.run_rotating(K, masks, obss); r1.record()
        torch.cuda.synchronize()
        dram = {"slices": S_rot, "kernel_ms": r0.elapsed_time(r1) / K, "timed_ply_window": [st.t - K, st.t]}
        del masks, obss

    bytes_ply = algorithmic_bytes_per_ply(N, with_obs)
    achieved = bytes_ply * B / (kern_ms * 1e-3) / 1e9
    fill = fill_ceiling(out_bytes, S_rot)
    gap_us = launch_gap_us()
    copy_gbs = device_copy_gbs(out_bytes)
    pmc_file = os.path.join("profiles", f"{'go_rollout_kernel' if args.mode == 'rollout' else 'go_step_kernel'}_{cfg.name}.txt")
    traffic = read_traffic(os.path.join(ROOT, pmc_file)) if with_obs and args.mode != "separate" and not args.superko and not args.line_padded else None
    if dram is not None:
        a = bytes_ply * B / (dram["kernel_ms"] * 1e-3) / 1e9
        dram.update({"achieved": a, "frac": a / HBM_PEAK_GBS, "frac_of_fill": fill["rotating_ms"] / dram["kernel_ms"],
                     "output_bytes_per_rotation": out_bytes * dram["slices"],
                     "note": "the same kernel and plies with mask + observation written to a different slice every ply, so every output line "
                             "reaches DRAM (a trajectory recorder sees this rate)"})
    window = [pre + Wm, pre + Wm + K]
    out = {
        "metric": "Go env steps/sec on 1 MI355X (19x19, batch 16384, random legal play); HBM GB/s % peak",
        "value": B * K / wall,
        "unit": "env steps/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": Wm,
        "ms_per_step": wall / K * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": cfg.name, "board_size": N, "batch": B, "seed": seed, "auto_reset": cfg.auto_reset,
                   "observation": with_obs, "mode": args.mode, "superko": int(args.superko), "komi": cfg.komi_x2 / 2,
                   "layout": f"line-padded (mask pitch {pitches[0]}, observation pitch {pitches[1]}; pad bytes written as zeros)" if args.line_padded
                             else "dense (the paper's tensor shapes)",
                   "pre_roll_plies": pre, "timed_ply_window": window,
                   "window_note": f"launch indices since init; plies 0..{pre - 1} are an untimed pre-roll through pgxgo_rollout (boards dense, games out "
                                  f"of step), then {Wm} untimed launches of the timed path",
                   **({"rollout_len": args.rollout_len, "rollout_slices": args.rollout_slices} if args.mode == "rollout" else {})},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic,
                     "traffic_source": (pmc_file + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, committed; not re-measured in this run)") if traffic else None,
                     "kernel": kname, "kernel_ms": kern_ms, "algorithmic_bytes_per_ply": bytes_ply,
                     "memory": "in place: every ply overwrites the same output buffers, whose lines stay in the 256 MB memory-side cache "
                               "(cache-assisted write rate); `dram` is the same measurement with outputs that reach DRAM",
                     "frac_of_fill": fill["in_place_ms"] / kern_ms,
                     "dram": dram, "fill": fill, "launch_gap_us": gap_us,
                     "whole_step_gbs": bytes_ply * B * K / wall / 1e9, "device_copy_gbs": copy_gbs},
    }
    if traffic:
        # the fill's time scaled from the output bytes to the bytes the counters saw this kernel move (state included)
        out["roofline"]["frac_of_fill_at_traffic"] = fill["in_place_ms"] * traffic / out_bytes / kern_ms
    if seg_ms:
        out["roofline"]["kernel_ms_segments"] = seg_ms
        out["roofline"]["kernel_ms_median"] = sorted(seg_ms)[2]
        out["roofline"]["kernel_ms_best"] = min(seg_ms)
    if args.mode != "rollout":
        # the ply of ONE wavefront of the same kernel (W boards), launch gap included: the latency floor of a launch
        W = pg.lib().pgxgo_boards_per_wavefront(N)
        tiny = GoStepper(cfg, W, with_obs, fused=(args.mode == "fused"), line_padded=args.line_padded)
        tiny.env.set_boards_per_wavefront(W)
        tiny.preroll(min(pre, 60)); tiny.run(20)
        floor_us = timed(lambda i: tiny.step_once(), 200) * 1e3
        wb = st.env.set_boards_per_wavefront(0)
        out["roofline"]["binding"] = bound_statement(kern_ms * 1e3, floor_us, fill["in_place_ms"] * 1e3, math.ceil(B / wb) / 1024.0)
    if args.mode == "fused" and not args.superko and not args.line_padded and K >= args.rollout_len:
        # for information: the same workload and ply window through the rollout kernel (rollout_len plies per launch, state in registers)
        Lr = args.rollout_len
        Kr = K // Lr * Lr
        env2 = pg.GoEnv(B, N, seed=seed, komi_x2=cfg.komi_x2, auto_reset=cfg.auto_reset)
        bufs = dict(actions=torch.empty((1, B), dtype=torch.int32, device="cuda"), rewards=st.rew.view(1, B, 2), terminated=st.term.view(1, B),
                    mask=st.mask.view(1, B, -1), obs=None if st.obs is None else st.obs.view(1, B, -1))
        env2.rollout(pre + Wm, seed, 0, start_t=st.start, **bufs)
        torch.cuda.synchronize()
        tr0 = time.perf_counter()
        ms_r = timed(lambda i: env2.rollout(Lr, seed, pre + Wm + i * Lr, start_t=st.start, **bufs), Kr // Lr) / Lr
        wall_r = time.perf_counter() - tr0
        a_r = bytes_ply * B / (ms_r * 1e-3) / 1e9
        out["rollout"] = {"value": B * Kr / wall_r, "unit": "env steps/s", "steps": Kr, "rollout_len": Lr, "kernel": "go_rollout_kernel<%d>" % N,
                          "kernel_ms_per_ply": ms_r, "achieved": a_r, "frac": a_r / HBM_PEAK_GBS, "frac_of_fill": fill["in_place_ms"] / ms_r,
                          "timed_ply_window": [pre + Wm, pre + Wm + Kr],
                          "note": "pgxgo_rollout: the same plies and outputs (in place) with rollout_len plies per launch; not the headline value"}
    if not args.no_cpu_baseline:
        n_threads = max(1, min(16, os.cpu_count() or 1))
        per = max(1, min(64 if N == 19 else 256, B // n_threads))    # enough work per call that the C code, not the interpreter, is timed
        cpu_plies = 1500 if cfg.auto_reset else K
        single, multi, reps = cpu_baseline(cfg, pre + Wm, cpu_plies, n_threads, per, superko=args.superko)
        out["cpu_baseline"] = {"value": multi, "unit": "env steps/s", "cores": n_threads, "kind": "oracle",
                               "sample": f"first {n_threads * per} environments of {cfg.name} (same seed and sampler), {per} per host thread, each "
                                         f"pre-rolled untimed through plies 0..{pre + Wm - 1} and then timed over plies {pre + Wm}..{pre + Wm + cpu_plies - 1} "
                                         f"(the GPU window's regime; independent of --steps), repeated from scratch {reps[1]}x ({reps[0]}x for the "
                                         f"one-thread figure on the first {per} environments) to run for >= 1 s",
                               "single_core_value": single}
    print(json.dumps(out))


def bench_hex(args, cfg):
    """The same protocol for Hex 11x11: one launch per ply (step + next random action), mask and observation every ply."""
    import torch

    import paper_2303_17503_amd as pg

    assert args.mode in ("fused", "rollout"), "--game hex has the fused and rollout modes"
    B, seed, K, Wm = cfg.batch, cfg.seed, args.steps, args.warmup
    with_obs = not args.no_obs
    pre = cfg.preroll
    env = pg.HexEnv(B, seed=seed, auto_reset=cfg.auto_reset)
    mask = env.new_mask()
    obs = env.new_obs() if with_obs else None
    rew = torch.zeros((B, 2), dtype=torch.float32, device="cuda")
    term = torch.zeros(B, dtype=torch.uint8, device="cuda")
    env.bind_outputs(mask, obs, rew, term)
    out_bytes = B * (122 + (484 if with_obs else 0))
    S_rot = rotation_slices(out_bytes)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    env.rollout(pre, seed, 0)      # untimed pre-roll, no outputs
    dram = None
    if args.mode == "rollout":
        Lr = args.rollout_len
        assert K % Lr == 0, "--steps must be a multiple of --rollout-len"
        bufs = dict(actions=torch.empty((1, B), dtype=torch.int32, device="cuda"), rewards=rew.view(1, B, 2), terminated=term.view(1, B),
                    mask=mask.view(1, B, 122), obs=None if obs is None else obs.view(1, B, 484))
        if Wm:
            env.rollout(Wm, seed, pre, **bufs)
        ev0.record(); ev1.record()                # created at their first record: not inside the timed region
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for i in range(K // Lr):
            env.rollout(Lr, seed, pre + Wm + i * Lr, **bufs)
        ev1.record()
        torch.cuda.synchronize()
        kname = "hex_rollout_kernel"
    else:
        acts = [torch.empty(B, dtype=torch.int32, device="cuda") for _ in range(2)]
        env.random_actions(seed, pre, out=acts[pre & 1])
        for t in range(pre, pre + Wm):
            env.step_sample(acts[t & 1], seed, t + 1, out=acts[(t + 1) & 1])
        ev0.record(); ev1.record()                # created at their first record: not inside the timed region
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for t in range(pre + Wm, pre + Wm + K):
            env.step_sample(acts[t & 1], seed, t + 1, out=acts[(t + 1) & 1])
        ev1.record()
        torch.cuda.synchronize()
        kname = "hex_step_kernel<true>"
    wall = time.perf_counter() - t0
    kern_ms = ev0.elapsed_time(ev1) / K       # per ply (a rollout launch covers rollout_len plies)
    if args.mode == "fused":
        masks = [env.new_mask() for _ in range(S_rot)]
        obss = [env.new_obs() for _ in range(S_rot)] if with_obs else None
        tbase = pre + Wm + K

        def rot(i):
            t = tbase + i
            env.set_output_buffers(masks[i % S_rot], None if obss is None else obss[i % S_rot], rew, term)
            env.step_sample(acts[t & 1], seed, t + 1, out=acts[(t + 1) & 1])

        dram = {"slices": S_rot, "kernel_ms": timed(rot, K), "timed_ply_window": [tbase, tbase + K]}
        env.set_output_buffers(mask, obs, rew, term)
        del masks, obss
    fill = fill_ceiling(out_bytes, S_rot)
    gap_us = launch_gap_us()
    copy_gbs = device_copy_gbs(out_bytes)
    bytes_ply = hex_bytes_per_ply(with_obs)
    achieved = bytes_ply * B / (kern_ms * 1e-3) / 1e9
    if dram is not None:
        a = bytes_ply * B / (dram["kernel_ms"] * 1e-3) / 1e9
        dram.update({"achieved": a, "frac": a / HBM_PEAK_GBS, "frac_of_fill": fill["rotating_ms"] / dram["kernel_ms"]})
    pmc_file = os.path.join("profiles", f"{'hex_step_lane_kernel' if B >= 196608 else 'hex_step_kernel'}_{cfg.name}.txt")
    traffic = read_traffic(os.path.join(ROOT, pmc_file)) if with_obs and args.mode == "fused" else None
    out = {
        "metric": "Hex env steps/sec on 1 MI355X (11x11, random legal play); HBM GB/s % peak",
        "value": B * K / wall, "unit": "env steps/s", "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": wall / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32", "data": "synthetic",
        "config": {"workload": cfg.name, "board_size": 11, "batch": B, "seed": seed, "auto_reset": cfg.auto_reset, "observation": with_obs,
                   "mode": args.mode, "pre_roll_plies": pre, "timed_ply_window": [pre + Wm, pre + Wm + K],
                   **({"rollout_len": args.rollout_len} if args.mode == "rollout" else {})},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": (pmc_file + " (committed rocprofv3 --pmc runs; not re-measured in this run)") if traffic else None,
                     "kernel": kname, "kernel_ms": kern_ms, "algorithmic_bytes_per_ply": bytes_ply,
                     "memory": "in place (outputs overwritten every ply); `dram` = outputs rotating beyond the 256 MB memory-side cache",
                     "frac_of_fill": fill["in_place_ms"] / kern_ms, "dram": dram, "fill": fill, "launch_gap_us": gap_us,
                     "whole_step_gbs": bytes_ply * B * K / wall / 1e9, "device_copy_gbs": copy_gbs},
    }
    if traffic:   # the fill's time scaled from the output bytes to the bytes the counters saw this kernel move
        out["roofline"]["frac_of_fill_at_traffic"] = fill["in_place_ms"] * traffic / out_bytes / kern_ms
    if args.mode == "fused":
        tiny = pg.HexEnv(5, seed=seed, auto_reset=cfg.auto_reset)
        tm, to = tiny.new_mask(), tiny.new_obs() if with_obs else None
        tiny.bind_outputs(tm, to, None, None)
        ta = [torch.empty(5, dtype=torch.int32, device="cuda") for _ in range(2)]
        tiny.random_actions(seed, 0, out=ta[0])
        floor_us = timed(lambda t: tiny.step_sample(ta[t & 1], seed, t + 1, out=ta[(t + 1) & 1]), 200) * 1e3
        out["roofline"]["binding"] = bound_statement(kern_ms * 1e3, floor_us, fill["in_place_ms"] * 1e3, math.ceil(B / 5) / 1024.0)
    if not args.no_cpu_baseline:
        n_threads = max(1, min(16, os.cpu_count() or 1))
        per = max(1, min(1024, B // n_threads))                      # enough work per call that the C code, not the interpreter, is timed
        cpu_plies = 1500 if cfg.auto_reset else K
        single, multi, reps = cpu_baseline(cfg, pre + Wm, cpu_plies, n_threads, per)
        out["cpu_baseline"] = {"value": multi, "unit": "env steps/s", "cores": n_threads, "kind": "oracle",
                               "sample": f"first {n_threads * per} environments of {cfg.name} (same seed and sampler), {per} per host thread, pre-rolled "
                                         f"untimed through plies 0..{pre + Wm - 1}, timed over the next {cpu_plies} plies, repeated {reps[1]}x "
                                         f"({reps[0]}x for the one-thread figure) to run for >= 1 s", "single_core_value": single}
    print(json.dumps(out))


def ceilings(args, cfg):
    """Reference measurements on the buffers and sizes of the configuration, all from this file and the library:
    plain fill (in place / rotating), the emit-only kernel (state -> mask + observation), device copy, the gap between
    empty launches, the step path in place / rotating, and the rollout kernel over 1, 2, 4, 8, 16 output slices."""
    import torch

    import paper_2303_17503_amd as pg

    assert args.game == "go", "--ceilings covers the Go configurations"
    B, N, seed = cfg.batch, cfg.board_size, cfg.seed
    P = N * N
    with_obs = not args.no_obs
    pre = cfg.warmup_max + cfg.preroll
    pitches = go_pitches(N, args.line_padded)
    out_bytes = B * (pitches[0] + (pitches[1] if with_obs else 0))
    S_rot = rotation_slices(out_bytes)
    K = min(args.steps, 500)
    res = {"workload": cfg.name, "observation": with_obs, "layout": "line-padded" if args.line_padded else "dense", "output_bytes_per_ply": out_bytes, "pre_roll_plies": pre, "plies_timed": K,
           "launch_gap_us": launch_gap_us(), "fill": fill_ceiling(out_bytes, S_rot), "device_copy_gbs": device_copy_gbs(out_bytes)}
    st = GoStepper(cfg, B, with_obs, line_padded=args.line_padded)
    st.preroll(pre); st.run(20)
    res["emit_only_ms"] = timed(lambda i: st.env.emit(st.mask, st.obs), 200)
    res["step_fused_in_place_ms"] = timed(lambda i: st.step_once(), K)
    masks = [st.env.new_mask() for _ in range(S_rot)]
    obss = [st.env.new_obs() for _ in range(S_rot)] if with_obs else None
    st.run_rotating(2 * S_rot, masks, obss)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize(); e0.record(); st.run_rotating(K, masks, obss); e1.record(); torch.cuda.synchronize()
    res["step_fused_rotating_ms"] = e0.elapsed_time(e1) / K
    res["rotating_slices"] = S_rot
    del masks, obss
    Lr = args.rollout_len
    res["rollout_ms_per_ply_by_slices"] = {}
    for S in (1, 2, 4, 8, 16):
        if S * out_bytes > (12 << 30):
            break
        env = pg.GoEnv(B, N, seed=seed, komi_x2=cfg.komi_x2, auto_reset=cfg.auto_reset, line_padded=args.line_padded)
        bufs = go_rollout_buffers(torch, S, B, pitches, with_obs)
        env.rollout(pre + 20, seed, 0, start_t=st.start, slices=S, **bufs)
        res["rollout_ms_per_ply_by_slices"][str(S)] = timed(lambda i: env.rollout(Lr, seed, pre + 20 + i * Lr, start_t=st.start, slices=S, **bufs),
                                                            max(1, K // Lr)) / Lr
        del bufs, env
    # what the store path itself does to a plain fill of the same bytes: kind of store x alignment of a wavefront's 1 KB to 128-byte
    # lines (base shifted by 16 bytes) x one buffer / rotating buffers
    raw = [torch.empty(out_bytes // 16 * 16 + 256, dtype=torch.uint8, device="cuda") for _ in range(S_rot)]
    res["fill_by_store_kind_ms"] = {}
    for kind, kname in ((0, "ordinary"), (1, "non_temporal"), (2, "through_l2")):
        for off in (0, 16):
            v = [r[off: off + out_bytes // 16 * 16] for r in raw]
            for x in v: pg.fill_probe(x, 1, kind)
            res["fill_by_store_kind_ms"][f"{kname}_{'aligned' if off == 0 else 'shifted16'}"] = {
                "in_place": timed(lambda i: pg.fill_probe(v[0], i, kind), 200), "rotating": timed(lambda i: pg.fill_probe(v[i % S_rot], i, kind), 200)}
    del raw
    # the search-facing calls: B entries out of a pool of 2B games in the same regime, sources and destinations scattered over the pool
    pool = pg.GoEnv(2 * B, N, seed=seed, komi_x2=cfg.komi_x2, auto_reset=True, line_padded=args.line_padded)
    pool.rollout(pre + 20, seed, 0, slices=1)
    g = torch.Generator().manual_seed(seed)
    perm = torch.randperm(2 * B, generator=g).to(torch.int32).cuda()
    src, dst = perm[:B].contiguous(), perm[B:].contiguous()
    acts = pool.random_actions(seed, pre + 20)[src.long()].contiguous()
    m, o = st.mask, st.obs
    rew, term = torch.empty(B, 2, dtype=torch.float32, device="cuda"), torch.empty(B, dtype=torch.uint8, device="cuda")
    res["slots"] = {"pool": 2 * B, "entries": B,
                    "step_slots_ms": timed(lambda i: pool.step_slots(src, acts, dst, mask=m, obs=o, rewards=rew, terminated=term), 200),
                    "step_slots_mask_only_ms": timed(lambda i: pool.step_slots(src, acts, dst, mask=m, rewards=rew, terminated=term), 200),
                    "copy_slots_ms": timed(lambda i: pool.copy_slots(src, dst), 200)}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
