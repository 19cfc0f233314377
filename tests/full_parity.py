#!/usr/bin/env python3
"""Exhaustive parity run: EVERY environment and EVERY ply of a benchmark configuration, HIP path against CPU oracle.

The batch is cut into contiguous shards, one oracle per shard, stepped
by a pool of host threads (the oracle's C calls and numpy's comparisons release the GIL).  After every ply the drawn
actions, legal masks, observations, rewards and terminated flags of the whole batch are copied to the host and
compared bit for bit; every `--state-every` plies the exported state is compared too.

  python tests/full_parity.py --config 3            # Go 19x19 x 16384, 2000 plies (a few minutes)
  python tests/full_parity.py --game hex --config 2

tests/test_gpu_full_parity.py runs it for every configuration; prints one progress line per 100 plies.
"""
import argparse
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


class Args:
    def __init__(self, game="go", config=3, plies=0, threads=16, state_every=100, superko=False, rollout=0, seed=None, mapping=0, line_padded=False):
        self.game, self.config, self.plies, self.threads, self.state_every = game, config, plies, threads, state_every
        self.superko, self.rollout, self.seed, self.mapping, self.line_padded = superko, rollout, seed, mapping, line_padded


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--game", choices=["go", "hex"], default="go")
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--plies", type=int, default=0, help="0 = warm-up + the configuration's measured plies")
    ap.add_argument("--threads", type=int, default=16)
    ap.add_argument("--state-every", type=int, default=100)
    ap.add_argument("--superko", type=int, default=0, help="Go only: both sides with the positional-superko rule on (1: enforced at play time, "
                                                            "2: honoured by the legal mask)")
    ap.add_argument("--rollout", type=int, default=0, help="L > 0: use the rollout kernel, L plies per launch, every ply recorded in its own slice")
    ap.add_argument("--seed", type=int, default=None, help="another seed than the configuration's (more trajectories of the same shape)")
    ap.add_argument("--mapping", type=int, default=0, help="Hex only: 1 = a board row per lane, 2 = a board per lane, 0 = the library's choice")
    ap.add_argument("--line-padded", action="store_true", help="Go only: output pitches rounded up to 128-byte lines (pad bytes must come out as zeros)")
    a = ap.parse_args()
    try:
        run(Args(a.game, a.config, a.plies, a.threads, a.state_every, a.superko, a.rollout, a.seed, a.mapping, a.line_padded))
    except AssertionError as e:
        print(e, flush=True)
        sys.exit(1)


def run(args):
    """Returns the number of game-plies compared; raises AssertionError at the first mismatch."""
    import torch

    import oracle
    import paper_2303_17503_amd as pg
    from oracle import hex as hx
    import workloads

    assert torch.cuda.is_available(), "needs a GPU"
    go = args.game == "go"
    cfg = (workloads.CONFIGS if go else workloads.HEX_CONFIGS)[args.config]
    B, N = cfg.batch, cfg.board_size
    seed = cfg.seed if args.seed is None else args.seed
    P = N * N
    planes = 17 if go else 4
    T = args.plies or (cfg.warmup_max + cfg.steps)
    start = workloads.start_times(cfg) if go else None
    st_dev = None if start is None else torch.as_tensor(start, device="cuda")

    assert go or not args.line_padded, "the line-padded layout is a Go option"
    env = pg.GoEnv(B, N, seed=seed, komi_x2=cfg.komi_x2, auto_reset=cfg.auto_reset, line_padded=args.line_padded) if go else \
        pg.HexEnv(B, seed=seed, auto_reset=cfg.auto_reset)
    if args.mapping:
        assert not go, "the mapping is a Hex launch-shape choice"
        assert env.set_mapping(args.mapping) == args.mapping
    if args.superko:
        assert go, "the superko rule is a Go option"
        env.enable_superko(int(args.superko))
    mask, obs = env.new_mask(), env.new_obs()
    if args.line_padded:
        mask.fill_(7); obs.fill_(7)     # the pad bytes belong to the records and have to come out as zeros
    rew = torch.zeros((B, 2), dtype=torch.float32, device="cuda")
    term = torch.zeros(B, dtype=torch.uint8, device="cuda")
    env.bind_outputs(mask, obs, rew, term)

    K = max(1, min(args.threads, B))
    cuts = [B * i // K for i in range(K + 1)]
    shards = [(cuts[i], cuts[i + 1]) for i in range(K) if cuts[i + 1] > cuts[i]]

    def make(lo, hi):
        ids = np.arange(lo, hi, dtype=np.int32)
        if go:
            return oracle.GoOracle(hi - lo, N, seed=seed, komi_x2=cfg.komi_x2, auto_reset=cfg.auto_reset, env_ids=ids, superko=int(args.superko))
        return hx.HexOracle(hi - lo, N, seed=seed, auto_reset=cfg.auto_reset, env_ids=ids)

    oracle.lib(); hx.lib()
    pool = ThreadPoolExecutor(len(shards))
    orcs = list(pool.map(lambda s: make(*s), shards))

    # pinned host mirrors of the outputs
    h_act = torch.empty(B, dtype=torch.int32, pin_memory=True)
    h_mask = torch.empty(mask.shape, dtype=torch.uint8, pin_memory=True)
    h_obs = torch.empty(obs.shape, dtype=torch.uint8, pin_memory=True)
    h_rew = torch.empty((B, 2), dtype=torch.float32, pin_memory=True)
    h_term = torch.empty(B, dtype=torch.uint8, pin_memory=True)
    n_act, n_mask, n_obs, n_rew, n_term = (x.numpy() for x in (h_act, h_mask, h_obs, h_rew, h_term))
    state_fields = ("board", "history", "ko", "to_play", "steps", "passes", "terminated", "black_player", "episode") if go else \
                   ("board", "to_play", "steps", "terminated", "black_player", "episode")

    def check(k, t, g_state):
        lo, hi = shards[k]
        o = orcs[k]
        a = o.random_actions(seed, t, None if start is None else start[lo:hi])
        if not (n_act[lo:hi] == a).all(): return f"drawn action, shard {k}"
        o.step(a)
        live = a >= 0
        if not (n_mask[lo:hi, :P + 1] == o.legal_mask()).all(): return f"mask, shard {k}"
        if not (n_obs[lo:hi, :P * planes].reshape(hi - lo, N, N, planes) == o.observe()).all(): return f"observation, shard {k}"
        if args.line_padded and (n_mask[lo:hi, P + 1:][live].any() or n_obs[lo:hi, P * planes:][live].any()): return f"pad bytes, shard {k}"
        if not (n_rew[lo:hi][live] == o.rewards()[live]).all(): return f"rewards, shard {k}"
        if not (n_term[lo:hi][live] == o.terminated()[live]).all(): return f"terminated, shard {k}"
        if g_state is not None:
            c = o.export_state()
            for name in state_fields:
                if not (g_state[name][lo:hi].astype(np.int64) == getattr(c, name).astype(np.int64)).all(): return f"state field {name}, shard {k}"
            if not (g_state["illegal"][lo:hi].astype(np.int64) == o.illegal_count().astype(np.int64)).all(): return f"illegal counter, shard {k}"
        return None

    t0 = time.time()
    n_plies = 0

    def compare(t, with_state):
        nonlocal n_plies
        g_state = {k: v.cpu().numpy() for k, v in env.export_state().items()} if with_state else None
        torch.cuda.synchronize()
        n_plies += int((n_act >= 0).sum())
        bad = [r for r in pool.map(lambda k: check(k, t, g_state), range(len(shards))) if r]
        assert not bad, f"MISMATCH at ply {t}: {bad[0]}"
        if t % 100 == 99 or t == T - 1:
            print(f"[{time.time() - t0:6.0f} s] ply {t + 1}/{T}: all {B} environments agree", flush=True)

    if args.rollout:
        L = args.rollout
        tr = dict(actions=torch.empty((L, B), dtype=torch.int32, device="cuda"), rewards=torch.empty((L, B, 2), dtype=torch.float32, device="cuda"),
                  terminated=torch.empty((L, B), dtype=torch.uint8, device="cuda"), mask=torch.empty((L,) + tuple(mask.shape), dtype=torch.uint8, device="cuda"),
                  obs=torch.empty((L,) + tuple(obs.shape), dtype=torch.uint8, device="cuda"))
        for t in range(0, T, L):
            n = min(L, T - t)
            env.rollout(n, seed, t, start_t=st_dev, slices=L, **tr)       # ply t+i of this launch lands in slice i
            for i in range(n):
                h_act.copy_(tr["actions"][i]); h_mask.copy_(tr["mask"][i]); h_obs.copy_(tr["obs"][i])
                h_rew.copy_(tr["rewards"][i]); h_term.copy_(tr["terminated"][i])
                compare(t + i, with_state=(i == n - 1))                     # the state on the device is the one after the launch
    else:
        acts = [torch.empty(B, dtype=torch.int32, device="cuda") for _ in range(2)]
        env.random_actions(seed, 0, st_dev, out=acts[0])
        for t in range(T):
            h_act.copy_(acts[t & 1])
            env.step_sample(acts[t & 1], seed, t + 1, st_dev, out=acts[(t + 1) & 1])
            h_mask.copy_(mask); h_obs.copy_(obs); h_rew.copy_(rew); h_term.copy_(term)
            compare(t, with_state=(t % args.state_every == 0 or t == T - 1))
    print(f"FULL PARITY OK: {cfg.name}{(' with superko (mode %d)' % int(args.superko)) if args.superko else ''}{' through the rollout kernel' if args.rollout else ''}{' with line-padded pitches' if args.line_padded else ''}, {B} environments x {T} launches = {n_plies} game-plies, every drawn action, mask, observation, "
          f"reward and terminated flag compared; state every {args.state_every} plies; {len(shards)} oracle shards; {time.time() - t0:.0f} s", flush=True)
    pool.shutdown()
    return n_plies


if __name__ == "__main__":
    main()
