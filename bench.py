#!/usr/bin/env python3
"""Benchmark of the batched Go environment step on one MI355X.

One "step" is one pass of the whole hot path over the batch: draw a uniform random legal action for every
game, apply it (legality gate, placement, capture, ko, history, termination + area score, auto-reset), and
emit the next legal mask [B][362], observation [B][19][19][17], rewards and terminated flags.  The default
workload is the headline configuration: 19x19, 16384 games, seed 3, auto-reset, 2000 plies per game.

Prints ONE JSON line.  Inputs are synthetic by construction: the
paper's own benchmark is random play from the empty board (Sec. 4.1).
"""
import argparse
import json
import os
import re
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published


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


def device_copy_gbs(nbytes):
    """A plain device copy of as many bytes as one step writes: a practical ceiling, and the kernel of known size that
    calibrates the HBM counters."""
    import torch

    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(5): dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(50): dst.copy_(src)
    e1.record(); torch.cuda.synchronize()
    return 2 * nbytes * 50 / (e0.elapsed_time(e1) * 1e-3) / 1e9


def cpu_baseline(cfg, steps, n_threads, envs_per_thread, superko=False):
    """The CPU oracle as it stands on the same workload: the first n_threads*envs_per_thread environments
    of the configuration, all `steps` plies, sharded over host threads (the C calls release the GIL)."""
    import numpy as np

    import oracle

    oracle.lib()
    if cfg.game == "hex":
        from oracle import hex as hx
        hx.lib()
    done = [0] * n_threads

    def work(i):
        ids = np.arange(i * envs_per_thread, (i + 1) * envs_per_thread, dtype=np.int32)
        if cfg.game == "hex":
            from oracle import hex as hx
            o = hx.HexOracle(envs_per_thread, cfg.board_size, seed=cfg.seed, auto_reset=cfg.auto_reset, env_ids=ids)
        else:
            o = oracle.GoOracle(envs_per_thread, cfg.board_size, seed=cfg.seed, komi_x2=cfg.komi_x2, auto_reset=cfg.auto_reset, env_ids=ids,
                            superko=superko)
        for t in range(steps):
            o.step(o.random_actions(cfg.seed, t))
        done[i] = envs_per_thread * steps

    def run(k):
        th = [threading.Thread(target=work, args=(i,)) for i in range(k)]
        t0 = time.perf_counter()
        for x in th: x.start()
        for x in th: x.join()
        return sum(done[:k]) / (time.perf_counter() - t0)

    single = run(1)
    multi = run(n_threads) if n_threads > 1 else single
    return single, multi


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--game", choices=["go", "hex"], default="go", help="go: the headline workload; hex: the second workload (Hex 11x11)")
    ap.add_argument("--config", type=int, default=None, help="index into workloads.CONFIGS (default 3 = headline) or, with --game hex, "
                                                             "into workloads.HEX_CONFIGS (default 2)")
    ap.add_argument("--mode", choices=["fused", "separate", "rollout"], default="fused",
                    help="fused: one launch per ply, the step kernel also draws the next action (headline); separate: sampler kernel + "
                         "step kernel per ply; rollout: --rollout-len plies per launch with the state kept in registers")
    ap.add_argument("--rollout-len", type=int, default=50, help="plies per launch in rollout mode")
    ap.add_argument("--rollout-slices", type=int, default=1, help="trajectory slices the rollout writes to (1 = overwrite one set of buffers)")
    ap.add_argument("--superko", action="store_true", help="Go only: switch the positional-superko rule on (not the headline metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-obs", action="store_true", help="do not emit the observation (not the headline metric)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (games are independent; more GPUs would shard the batch "
              "with no communication); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2303_17503_amd as pg
    from paper_2303_17503_amd import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.game == "hex":
        return bench_hex(args, workloads.HEX_CONFIGS[2 if args.config is None else args.config])
    cfg = workloads.CONFIGS[3 if args.config is None else args.config]
    B, N, seed = cfg.batch, cfg.board_size, cfg.seed
    K, Wm = args.steps, args.warmup
    with_obs = not args.no_obs

    env = pg.GoEnv(B, N, seed=seed, komi_x2=cfg.komi_x2, auto_reset=cfg.auto_reset)
    if args.superko:
        assert args.mode != "rollout", "the rollout kernel does not carry the superko tables"
        env.enable_superko()
    start = workloads.start_times(cfg)
    start_dev = None if start is None else torch.as_tensor(start, device="cuda")
    pre = cfg.warmup_max          # config 4: the plies that build the mid-game positions are not part of the measurement
    P = N * N
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    if args.mode == "rollout":
        S, Lr = args.rollout_slices, args.rollout_len
        assert K % Lr == 0 and (pre + Wm) >= 0, "--steps must be a multiple of --rollout-len"
        bufs = dict(actions=torch.empty((S, B), dtype=torch.int32, device="cuda"),
                    rewards=torch.empty((S, B, 2), dtype=torch.float32, device="cuda"),
                    terminated=torch.empty((S, B), dtype=torch.uint8, device="cuda"),
                    mask=torch.empty((S, B, P + 1), dtype=torch.uint8, device="cuda"),
                    obs=torch.empty((S, B, P * 17), dtype=torch.uint8, device="cuda") if with_obs else None)
        if pre + Wm:
            env.rollout(pre + Wm, seed, 0, start_t=start_dev, slices=S, **bufs)
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
    else:
        mask = env.new_mask()
        obs = env.new_obs() if with_obs else None
        rew = torch.zeros((B, 2), dtype=torch.float32, device="cuda")
        term = torch.zeros(B, dtype=torch.uint8, device="cuda")
        env.bind_outputs(mask, obs, rew, term)
        acts = [torch.empty(B, dtype=torch.int32, device="cuda") for _ in range(2)]

        def run_steps(t0, n, events=None):
            """n passes of the hot path for launches t0..t0+n-1; acts[t & 1] holds the actions of launch t."""
            for i in range(n):
                t = t0 + i
                if args.mode == "fused":
                    env.step_sample(acts[t & 1], seed, t + 1, start_dev, out=acts[(t + 1) & 1])
                else:
                    if events is not None: events[i][0].record()
                    env.step(acts[t & 1])
                    if events is not None: events[i][1].record()
                    env.random_actions(seed, t + 1, start_dev, out=acts[(t + 1) & 1])

        env.random_actions(seed, 0, start_dev, out=acts[0])
        run_steps(0, pre + Wm)
        torch.cuda.synchronize()
        # the timed region, cut into five segments by events on the same stream (median and best segment are reported too)
        cuts = [K * i // 5 for i in range(6)]
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        t0 = time.perf_counter()
        ev0.record()
        for i in range(5):
            run_steps(pre + Wm + cuts[i], cuts[i + 1] - cuts[i])
            if i < 4: marks[i].record()
        ev1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        evs = [ev0] + marks + [ev1]
        seg_ms = [evs[i].elapsed_time(evs[i + 1]) / max(1, cuts[i + 1] - cuts[i]) for i in range(5)] if K >= 5 else []
        if args.mode == "fused":
            # the timed region is K launches of the one kernel, back to back on the stream the events are on
            kern_ms = ev0.elapsed_time(ev1) / K
        else:
            n_ev = min(K, 500)
            events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ev)]
            run_steps(pre + Wm + K, n_ev, events)
            torch.cuda.synchronize()
            kern_ms = sum(a.elapsed_time(b) for a, b in events) / n_ev
        kname = "go_step_superko_kernel<%d>" % N if args.superko else "go_step_kernel<%d,%s>" % (N, "true" if args.mode == "fused" else "false")

    copy_gbs = device_copy_gbs(B * (N * N * 17 + N * N + 1))

    bytes_ply = algorithmic_bytes_per_ply(N, with_obs)
    achieved = bytes_ply * B / (kern_ms * 1e-3) / 1e9
    traffic = read_traffic(os.path.join(ROOT, "profiles", f"go_step_kernel_{cfg.name}_pmc.txt")) if with_obs and args.mode == "fused" and not args.superko else None
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
                   "observation": with_obs, "mode": args.mode, "superko": bool(args.superko), "komi": cfg.komi_x2 / 2, "pre_warmup_plies_max": cfg.warmup_max,
                   **({"rollout_len": args.rollout_len, "rollout_slices": args.rollout_slices} if args.mode == "rollout" else {})},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "kernel": kname, "kernel_ms": kern_ms, "algorithmic_bytes_per_ply": bytes_ply,
                     "whole_step_gbs": bytes_ply * B * K / wall / 1e9, "device_copy_gbs": copy_gbs},
    }
    if args.mode == "fused" and not args.superko and K >= args.rollout_len:
        # for information: the same workload through the rollout kernel (rollout_len plies per launch, state in registers)
        Lr = args.rollout_len
        Kr = K // Lr * Lr
        env2 = pg.GoEnv(B, N, seed=seed, komi_x2=cfg.komi_x2, auto_reset=cfg.auto_reset)
        bufs = dict(actions=torch.empty((1, B), dtype=torch.int32, device="cuda"), rewards=rew.view(1, B, 2), terminated=term.view(1, B),
                    mask=mask.view(1, B, -1), obs=None if obs is None else obs.view(1, B, -1))
        if pre + Wm:
            env2.rollout(pre + Wm, seed, 0, start_t=start_dev, **bufs)
        torch.cuda.synchronize()
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        tr0 = time.perf_counter()
        r0.record()
        for i in range(Kr // Lr):
            env2.rollout(Lr, seed, pre + Wm + i * Lr, start_t=start_dev, **bufs)
        r1.record()
        torch.cuda.synchronize()
        wall_r = time.perf_counter() - tr0
        ms_r = r0.elapsed_time(r1) / Kr
        out["rollout"] = {"value": B * Kr / wall_r, "unit": "env steps/s", "steps": Kr, "rollout_len": Lr, "kernel": "go_rollout_kernel<%d>" % N,
                          "kernel_ms_per_ply": ms_r, "achieved": bytes_ply * B / (ms_r * 1e-3) / 1e9, "frac": bytes_ply * B / (ms_r * 1e-3) / 1e9 / HBM_PEAK_GBS,
                          "note": "pgxgo_rollout: the same plies and outputs with rollout_len plies per launch; not the headline value"}
    if args.mode == "fused" and seg_ms:
        out["roofline"]["kernel_ms_segments"] = seg_ms
        out["roofline"]["kernel_ms_median"] = sorted(seg_ms)[2]
        out["roofline"]["kernel_ms_best"] = min(seg_ms)
    if not args.no_cpu_baseline:
        n_threads = max(1, min(16, os.cpu_count() or 1))
        envs_per_thread = 16
        cpu_steps = min(K, 2000)
        single, multi = cpu_baseline(cfg, cpu_steps, n_threads, envs_per_thread, superko=args.superko)
        out["cpu_baseline"] = {"value": multi, "unit": "env steps/s", "cores": n_threads, "kind": "oracle",
                               "sample": f"first {n_threads * envs_per_thread} environments of {cfg.name} (same seed and sampler), "
                                         f"{cpu_steps} plies each, {envs_per_thread} per host thread; warm-up of config 4 not replayed",
                               "single_core_value": single}
    print(json.dumps(out))


def bench_hex(args, cfg):
    """The same protocol for Hex 11x11: one launch per ply (step + next random action), mask and observation every ply."""
    import torch

    import paper_2303_17503_amd as pg

    assert args.mode in ("fused", "rollout"), "--game hex has the fused and rollout modes"
    B, seed, K, Wm = cfg.batch, cfg.seed, args.steps, args.warmup
    with_obs = not args.no_obs
    env = pg.HexEnv(B, seed=seed, auto_reset=cfg.auto_reset)
    mask = env.new_mask()
    obs = env.new_obs() if with_obs else None
    rew = torch.zeros((B, 2), dtype=torch.float32, device="cuda")
    term = torch.zeros(B, dtype=torch.uint8, device="cuda")
    env.bind_outputs(mask, obs, rew, term)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.mode == "rollout":
        Lr = args.rollout_len
        assert K % Lr == 0, "--steps must be a multiple of --rollout-len"
        bufs = dict(actions=torch.empty((1, B), dtype=torch.int32, device="cuda"), rewards=rew.view(1, B, 2), terminated=term.view(1, B),
                    mask=mask.view(1, B, 122), obs=None if obs is None else obs.view(1, B, 484))
        if Wm:
            env.rollout(Wm, seed, 0, **bufs)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for i in range(K // Lr):
            env.rollout(Lr, seed, Wm + i * Lr, **bufs)
        ev1.record()
        torch.cuda.synchronize()
        kname = "hex_rollout_kernel"
    else:
        acts = [torch.empty(B, dtype=torch.int32, device="cuda") for _ in range(2)]
        env.random_actions(seed, 0, out=acts[0])
        for t in range(Wm):
            env.step_sample(acts[t & 1], seed, t + 1, out=acts[(t + 1) & 1])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for t in range(Wm, Wm + K):
            env.step_sample(acts[t & 1], seed, t + 1, out=acts[(t + 1) & 1])
        ev1.record()
        torch.cuda.synchronize()
        kname = "hex_step_kernel<true>"
    wall = time.perf_counter() - t0
    kern_ms = ev0.elapsed_time(ev1) / K       # per ply (a rollout launch covers rollout_len plies)
    copy_gbs = device_copy_gbs(B * (484 + 122))
    bytes_ply = hex_bytes_per_ply(with_obs)
    achieved = bytes_ply * B / (kern_ms * 1e-3) / 1e9
    traffic = read_traffic(os.path.join(ROOT, "profiles", f"hex_step_kernel_{cfg.name}_pmc.txt")) if with_obs and args.mode == "fused" else None
    out = {
        "metric": "Hex env steps/sec on 1 MI355X (11x11, random legal play); HBM GB/s % peak",
        "value": B * K / wall, "unit": "env steps/s", "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": wall / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32", "data": "synthetic",
        "config": {"workload": cfg.name, "board_size": 11, "batch": B, "seed": seed, "auto_reset": cfg.auto_reset, "observation": with_obs,
                   "mode": args.mode, **({"rollout_len": args.rollout_len} if args.mode == "rollout" else {})},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "kernel": kname, "kernel_ms": kern_ms, "algorithmic_bytes_per_ply": bytes_ply,
                     "whole_step_gbs": bytes_ply * B * K / wall / 1e9, "device_copy_gbs": copy_gbs},
    }
    if not args.no_cpu_baseline:
        n_threads = max(1, min(16, os.cpu_count() or 1))
        cpu_steps = min(K, 2000)
        single, multi = cpu_baseline(cfg, cpu_steps, n_threads, 64)
        out["cpu_baseline"] = {"value": multi, "unit": "env steps/s", "cores": n_threads, "kind": "oracle",
                               "sample": f"first {n_threads * 64} environments of {cfg.name} (same seed and sampler), {cpu_steps} plies each, "
                                         "64 per host thread", "single_core_value": single}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
