"""Pins of the counter-based hash and of the k-th-legal-action sampler."""
import numpy as np

import oracle

M = 0xFFFFFFFF


def mix32_py(x):
    x ^= x >> 16; x = (x * 0x7FEB352D) & M
    x ^= x >> 15; x = (x * 0x846CA68B) & M
    x ^= x >> 16
    return x


def hash_py(seed, tag, env, t):
    return mix32_py(mix32_py(mix32_py((seed + 0x9E3779B9 * (tag + 1)) & M) ^ env) ^ t)


def test_hash_matches_independent_python_expression():
    rng = np.random.default_rng(0)
    cases = [(0, 0, 0, 0), (0, 1, 0, 0), (3, 0, 16383, 1999), (M, 2, M, M), (4, 2, 65535, 0)]
    cases += [tuple(int(v) for v in rng.integers(0, 2**32, 4)) for _ in range(200)]
    for c in cases:
        assert oracle.hash4(*c) == hash_py(*c), c
    # the mixer is a bijection built from xorshifts and odd multipliers: spot-check that it spreads bits
    vals = {oracle.hash4(0, 0, e, 0) for e in range(4096)}
    assert len(vals) == 4096
    assert 0.45 < np.mean([oracle.hash4(1, 1, e, 0) & 1 for e in range(4096)]) < 0.55


def test_sampler_picks_kth_legal_action_and_skips():
    B, N = 32, 9
    o = oracle.GoOracle(B, N, seed=9, auto_reset=True)
    for t in range(150):
        m = o.legal_mask()
        start = np.where(np.arange(B) % 4 == 0, 40, 0).astype(np.int32)
        a = o.random_actions(77, t, start_t=start)
        for b in range(B):
            if t < start[b]:
                assert a[b] == -1
                continue
            legal = np.flatnonzero(m[b])
            assert a[b] == legal[hash_py(77, 0, b, t) % len(legal)]
        o.step(a)
    s = o.export_state()
    assert (s.steps[::4] + 40 * (s.episode[::4] == 0) <= 150).all()


def test_env_ids_give_the_same_trajectories_as_the_full_batch():
    N, T = 9, 120
    full = oracle.GoOracle(40, N, seed=4, auto_reset=True)
    ids = np.array([3, 17, 39], np.int32)
    part = oracle.GoOracle(3, N, seed=4, auto_reset=True, env_ids=ids)
    for t in range(T):
        af, ap = full.random_actions(4, t), part.random_actions(4, t)
        assert (af[ids] == ap).all()
        full.step(af); part.step(ap)
    assert (full.export_state().board[ids] == part.export_state().board).all()
    assert (full.observe()[ids] == part.observe()).all()
    assert (full.export_state().black_player[ids] == part.export_state().black_player).all()
