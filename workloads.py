"""Seeded synthetic workloads (the five benchmark configurations) shared by tests, bench and smoke.

This module holds no rule arithmetic.  The only numbers it draws are the per-environment warm-up
lengths of configuration 4, produced with the counter-based hash written out in numpy and handed to
both the HIP path and the CPU oracle as a plain input array.

The paper's benchmark (Sec. 4.1) is itself synthetic: a uniform random legal policy with auto-reset,
so these configurations reproduce its structure directly; no dataset stands behind them.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    board_size: int
    batch: int
    seed: int
    auto_reset: bool
    steps: int            # measured plies per environment
    warmup_max: int = 0   # config 4: each environment first plays k ~ U[0, warmup_max] plies
    emit_obs: bool = True
    komi_x2: int = 15
    game: str = "go"
    preroll: int = 0      # benchmark only: untimed plies played before the timed window, so that it lies in the workload's steady regime


CONFIGS = [
    Config("go9_b256_fullgame", 9, 256, 0, False, 162, preroll=30),
    Config("go9_b4096_autoreset", 9, 4096, 1, True, 1000, preroll=300),
    Config("go19_b1024_fullgame", 19, 1024, 2, False, 722, preroll=200),
    Config("go19_b16384_autoreset_obs", 19, 16384, 3, True, 2000, preroll=600),
    Config("go19_b65536_midgame", 19, 65536, 4, True, 500, warmup_max=300),   # its warm-up is its pre-roll
]

# Hex 11x11 (the second workload): random legal play from the empty board as in Sec. 4.1; a game lasts at most 122 plies
HEX_CONFIGS = [
    Config("hex11_b1024_fullgame", 11, 1024, 5, False, 122, game="hex", preroll=15),
    Config("hex11_b16384_autoreset", 11, 16384, 6, True, 1000, game="hex", preroll=200),
    Config("hex11_b262144_autoreset", 11, 262144, 7, True, 500, game="hex", preroll=200),
]

_M = np.uint64(0xFFFFFFFF)


def _mix(x):
    x = x.astype(np.uint64)
    x ^= x >> np.uint64(16); x = (x * np.uint64(0x7FEB352D)) & _M
    x ^= x >> np.uint64(15); x = (x * np.uint64(0x846CA68B)) & _M
    x ^= x >> np.uint64(16)
    return x


def counter_hash(seed, tag, env, t):
    """uint32 hash of (seed, tag, env, t); env may be an array."""
    env = np.asarray(env, dtype=np.uint64)
    s = np.uint64((seed + 0x9E3779B9 * (tag + 1)) & 0xFFFFFFFF)
    return _mix(_mix(_mix(np.full_like(env, s)) ^ env) ^ np.uint64(t & 0xFFFFFFFF)).astype(np.uint32)


def start_times(cfg: Config, env_ids=None):
    """int32[batch] launch index at which each environment starts to move (None when there is no warm-up).

    Environment e plays k_e = hash(seed, 2, e, 0) mod (warmup_max+1) warm-up plies: it is skipped
    (action -1) while t < warmup_max - k_e, so that all environments finish warming up at t = warmup_max."""
    if cfg.warmup_max == 0:
        return None
    ids = np.arange(cfg.batch) if env_ids is None else np.asarray(env_ids)
    k = counter_hash(cfg.seed, 2, ids, 0) % np.uint32(cfg.warmup_max + 1)
    return (cfg.warmup_max - k.astype(np.int64)).astype(np.int32)
