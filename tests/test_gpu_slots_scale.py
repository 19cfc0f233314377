"""The search-facing slot API at search scale (paper Sec. 5: tree search calls `step` from copies of stored states,
32 simulations per move): pools of >= 8192 state slots, >= 4096 entries per call over many blocks with a ragged last
block, random src -> dst expansions with in-place entries, legal / illegal / out-of-range / copy (-1) actions and a
few out-of-pool slot indices.  After EVERY call every entry's mask, observation, rewards and terminated flag and the
exported state of the WHOLE pool are compared with the CPU oracle (one oracle per shard of entries on host threads)."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
import paper_2303_17503_amd as pg
from gpu_common import to_np

pytestmark = pytest.mark.gpu

FIELDS = ("board", "history", "ko", "to_play", "steps", "passes", "terminated", "black_player", "episode")
THREADS = 16


def dev(a):
    return torch.as_tensor(np.ascontiguousarray(a), device="cuda")


def take(state, idx, P):
    sub = oracle.State(len(idx), P)
    for name in FIELDS:
        getattr(sub, name)[...] = getattr(state, name)[idx]
    return sub


@pytest.mark.parametrize("N,pool,calls,auto_reset", [(19, 8192, 50, True), (9, 12000, 60, False), (9, 8200, 50, True)])
def test_slot_api_at_search_scale(N, pool, calls, auto_reset):
    rng = np.random.default_rng(1000 + N + pool)
    seed, P = 77, N * N
    W = pg.lib().pgxgo_boards_per_wavefront(N)
    env = pg.GoEnv(pool, N, seed=seed, auto_reset=auto_reset)
    # every slot gets a different amount of history: slot e plays min(t, ...) random plies, staggered by start times
    warm = 90 if N == 19 else 50
    start = (rng.integers(0, warm, pool)).astype(np.int32)
    env.rollout(warm, seed, 0, start_t=dev(start))
    pool_state = oracle.State(pool, P)
    g = env.export_state()
    for name in FIELDS:
        getattr(pool_state, name)[...] = to_np(g[name]).astype(getattr(pool_state, name).dtype)
    illegal = to_np(g["illegal"]).astype(np.int64)
    ex = ThreadPoolExecutor(THREADS)
    oracle.lib()
    n_entries = n_illegal = n_copy = n_inplace = n_ended = 0

    for it in range(calls):
        n = int(rng.integers(4096, min(pool - 1500, 6200)))
        if n % (4 * W) == 0:
            n += 1                                            # a ragged last wavefront and block
        perm = rng.permutation(pool)
        dst = perm[:n].astype(np.int32)                       # pairwise distinct destinations
        src = rng.choice(perm[n:], n).astype(np.int32)        # sources that are nobody's destination ...
        same = rng.random(n) < 0.3
        src = np.where(same, dst, src).astype(np.int32)       # ... or the entry's own destination (in-place step)
        bad = rng.choice(n, 3, replace=False)                 # three entries with a slot index outside the pool
        src_call, dst_call = src.copy(), dst.copy()
        src_call[bad[0]] = pool + 7; dst_call[bad[1]] = -1; src_call[bad[2]] = -5
        good = np.ones(n, bool); good[bad] = False

        cuts = [n * k // THREADS for k in range(THREADS + 1)]

        def prepare(k):
            lo, hi = cuts[k], cuts[k + 1]
            o = oracle.GoOracle(hi - lo, N, seed=seed, auto_reset=auto_reset, env_ids=dst[lo:hi])
            o.import_state(take(pool_state, src[lo:hi], P))
            return o

        orcs = list(ex.map(prepare, range(THREADS)))
        m = np.concatenate([o.legal_mask() for o in orcs])
        pick = (rng.random(m.shape) * m).argmax(axis=1).astype(np.int32)     # a uniformly random legal action
        kind = rng.integers(0, 12, n)
        act = np.where(kind == 0, rng.integers(0, P, n), pick)               # any point: often illegal
        act = np.where(kind == 1, -1, act)                                   # plain copy
        act = np.where(kind == 2, rng.choice([P + 1, P + 50, -2, -100, 1 << 20], n), act).astype(np.int32)   # out of range: illegal
        term_before = np.concatenate([o.export_state().terminated for o in orcs])

        def advance(k):
            lo, hi = cuts[k], cuts[k + 1]
            orcs[k].step(act[lo:hi])
            return orcs[k].legal_mask(), orcs[k].observe(), orcs[k].rewards(), orcs[k].terminated(), orcs[k].export_state(), orcs[k].illegal_count()

        res = list(ex.map(advance, range(THREADS)))
        mask = torch.full((n, P + 1), 9, dtype=torch.uint8, device="cuda")
        obs = torch.full((n, P * 17), 9, dtype=torch.uint8, device="cuda")
        rew = torch.full((n, 2), 9.0, dtype=torch.float32, device="cuda")
        term = torch.full((n,), 9, dtype=torch.uint8, device="cuda")
        env.step_slots(dev(src_call), dev(act), dev(dst_call), mask=mask, obs=obs, rewards=rew, terminated=term)
        g_mask, g_obs, g_rew, g_term = to_np(mask), to_np(obs).reshape(n, N, N, 17), to_np(rew), to_np(term)
        c_mask = np.concatenate([r[0] for r in res]); c_obs = np.concatenate([r[1] for r in res])
        c_rew = np.concatenate([r[2] for r in res]); c_term = np.concatenate([r[3] for r in res])
        assert (g_mask[good] == c_mask[good]).all(), f"mask, call {it}"
        assert (g_obs[good] == c_obs[good]).all(), f"observation, call {it}"
        copied = act == -1
        live = good & ~copied
        assert g_rew[live].tobytes() == c_rew[live].tobytes(), f"rewards, call {it}"
        assert (g_rew[good & copied] == 0).all(), f"rewards of copied entries, call {it}"
        assert (g_term[live] == c_term[live]).all(), f"terminated, call {it}"
        assert (g_term[good & copied] == term_before[good & copied]).all(), f"terminated of copied entries, call {it}"
        assert (g_term[bad] == 255).all() and (g_mask[bad] == 0).all() and (g_obs[bad] == 0).all(), f"out-of-pool entries, call {it}"
        # write the stepped entries back into the host copy of the pool and compare the whole pool
        for k in range(THREADS):
            lo, hi = cuts[k], cuts[k + 1]
            sel = good[lo:hi]
            after = res[k][4]
            for name in FIELDS:
                getattr(pool_state, name)[dst[lo:hi][sel]] = getattr(after, name)[sel]
            illegal[dst[lo:hi][sel]] = illegal[src[lo:hi][sel]] + res[k][5][sel]
        g = env.export_state()
        for name in FIELDS:
            assert (to_np(g[name]).astype(np.int64) == getattr(pool_state, name).astype(np.int64)).all(), f"pool state field {name}, call {it}"
        assert (to_np(g["illegal"]).astype(np.int64) == illegal).all(), f"illegal counters, call {it}"
        n_entries += int(good.sum()); n_copy += int((good & copied).sum()); n_inplace += int((good & same).sum())
        n_illegal += int(sum(r[5][good[cuts[k]:cuts[k + 1]]].sum() for k, r in enumerate(res)))
        n_ended += int(c_term[live].sum())

    # copy_slots over many blocks
    n = 5001
    perm = rng.permutation(pool)
    dst, src = perm[:n].astype(np.int32), rng.choice(perm[n:], n).astype(np.int32)
    env.copy_slots(dev(src), dev(dst))
    for name in FIELDS:
        getattr(pool_state, name)[dst] = getattr(pool_state, name)[src]
    illegal[dst] = illegal[src]
    g = env.export_state()
    for name in FIELDS:
        assert (to_np(g[name]).astype(np.int64) == getattr(pool_state, name).astype(np.int64)).all(), f"pool state field {name} after copy_slots"
    assert (to_np(g["illegal"]).astype(np.int64) == illegal).all()
    assert n_entries >= calls * 4090 and n_illegal > calls * 50 and n_copy > calls * 100 and n_inplace > calls * 500 and n_ended > calls * 50
    ex.shutdown()
