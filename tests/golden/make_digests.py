"""Writes tests/golden/trajectory_digests.txt from the CPU oracle alone (regression pins, not correctness pins).

For each benchmark configuration (Go, then Hex): environments 0..7 of the configuration (same seed, sampler and warm-up
schedule), the first min(steps, 300) measured plies after the warm-up; the digest is blake2b-64 over, per ply,
the boards, legal masks, observations, rewards and terminated flags.  Run: python tests/golden/make_digests.py
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from oracle import hex as hex_oracle  # noqa: E402
import workloads  # noqa: E402  (configuration table only; a top-level module outside the product package)

ENVS = 8


def digest_config(cfg):
    ids = np.arange(ENVS, dtype=np.int32)
    o = oracle.GoOracle(ENVS, cfg.board_size, seed=cfg.seed, komi_x2=cfg.komi_x2, auto_reset=cfg.auto_reset, env_ids=ids)
    start = workloads.start_times(cfg, ids)
    h = hashlib.blake2b(digest_size=8)
    T = cfg.warmup_max + min(cfg.steps, 300)
    for t in range(T):
        o.step(o.random_actions(cfg.seed, t, start))
        if t >= cfg.warmup_max:
            for arr in (o.export_state().board, o.legal_mask(), o.observe(), o.rewards(), o.terminated()):
                h.update(np.ascontiguousarray(arr).tobytes())
    return h.hexdigest()


def digest_hex_config(cfg):
    """The same for a Hex workload: environments 0..7, the first min(steps, 300) plies."""
    ids = np.arange(ENVS, dtype=np.int32)
    o = hex_oracle.HexOracle(ENVS, cfg.board_size, seed=cfg.seed, auto_reset=cfg.auto_reset, env_ids=ids)
    h = hashlib.blake2b(digest_size=8)
    for t in range(min(cfg.steps, 300)):
        o.step(o.random_actions(cfg.seed, t))
        for arr in (o.export_state().board, o.legal_mask(), o.observe(), o.rewards(), o.terminated()):
            h.update(np.ascontiguousarray(arr).tobytes())
    return h.hexdigest()


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "trajectory_digests.txt")
    with open(out, "w") as f:
        f.write("# blake2b-64 digests of oracle trajectories (tests/golden/make_digests.py); config name, digest\n")
        for cfg in workloads.CONFIGS:
            f.write(f"{cfg.name} {digest_config(cfg)}\n")
        for cfg in workloads.HEX_CONFIGS:
            f.write(f"{cfg.name} {digest_hex_config(cfg)}\n")
    print(open(out).read())


if __name__ == "__main__":
    main()
