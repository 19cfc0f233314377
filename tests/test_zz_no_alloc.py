"""pgxgo_init_static, the entry point that allocates nothing (for callers under HIP graph capture or with a ban on
allocation): its games must behave exactly like those of pgxgo_init with a caller-owned buffer.  Two calls in a row on
the same GPU share the library's static state buffer, the second with a smaller input; each is compared ply by ply
(drawn actions, legal mask, observation, rewards, terminated flags, exported state) with a handle made by pgxgo_init,
and with the CPU oracle.  Sizes beyond the buffer are refused with PGXGO_ELIMIT."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import paper_2303_17503_amd as pg

pytestmark = pytest.mark.gpu

FIELDS = ("board", "history", "ko", "to_play", "steps", "passes", "terminated", "black_player", "episode", "illegal")


def to_np(t):
    return t.detach().cpu().numpy()


def bound(env):
    mask, obs = env.new_mask(), env.new_obs()
    rew = torch.zeros((env.B, 2), dtype=torch.float32, device="cuda")
    term = torch.zeros(env.B, dtype=torch.uint8, device="cuda")
    env.bind_outputs(mask, obs, rew, term)
    return mask, obs, rew, term


def run_pair(B, N, seed, plies):
    """The same games through a static handle and through an ordinary one; returns the number of compared plies."""
    a = pg.GoEnv(B, N, seed=seed, auto_reset=True, static_state=True)
    b = pg.GoEnv(B, N, seed=seed, auto_reset=True)
    orc = oracle.GoOracle(B, N, seed=seed, auto_reset=True)
    assert a._state is None and b._state is not None
    oa, ob = bound(a), bound(b)
    for x, y in zip(oa, ob):
        assert to_np(x).tobytes() == to_np(y).tobytes()
    act_a, act_b = a.random_actions(seed, 0), b.random_actions(seed, 0)
    for t in range(plies):
        act_c = orc.random_actions(seed, t)
        assert (to_np(act_a) == to_np(act_b)).all() and (to_np(act_a) == act_c).all(), f"actions t={t}"
        if t % 2:                                   # both stepping paths
            act_a, act_b = a.step_sample(act_a, seed, t + 1), b.step_sample(act_b, seed, t + 1)
        else:
            a.step(act_a); b.step(act_b)
            act_a, act_b = a.random_actions(seed, t + 1), b.random_actions(seed, t + 1)
        orc.step(act_c)
        for name, x, y in zip(("mask", "obs", "rewards", "terminated"), oa, ob):
            assert to_np(x).tobytes() == to_np(y).tobytes(), f"{name} t={t}"
        assert (to_np(oa[0]) == orc.legal_mask()).all() and (to_np(oa[1]).reshape(B, N, N, 17) == orc.observe()).all(), f"oracle t={t}"
        assert to_np(oa[2]).tobytes() == orc.rewards().tobytes() and (to_np(oa[3]) == orc.terminated()).all(), f"oracle t={t}"
        if t % 25 == 0 or t == plies - 1:
            sa, sb = a.export_state(), b.export_state()
            for f in FIELDS:
                assert to_np(sa[f]).tobytes() == to_np(sb[f]).tobytes(), f"state field {f} t={t}"
    # the rollout kernel and the getters on the static handle as well
    a.rollout(30, seed, plies); b.rollout(30, seed, plies)
    assert to_np(a.legal_mask()).tobytes() == to_np(b.legal_mask()).tobytes() and to_np(a.observe()).tobytes() == to_np(b.observe()).tobytes()
    sa, sb = a.export_state(), b.export_state()
    for f in FIELDS:
        assert to_np(sa[f]).tobytes() == to_np(sb[f]).tobytes(), f"state field {f} after the rollout"
    return plies


def test_static_state_two_calls_in_a_row_the_second_smaller():
    assert run_pair(600, 19, seed=5, plies=160) == 160       # fills 0.65 MB of the static buffer
    assert run_pair(83, 19, seed=6, plies=120) == 120        # smaller input on the same buffer: nothing of the first call shows
    assert run_pair(1000, 9, seed=7, plies=200) == 200       # another board size, another layout of the same bytes
    assert run_pair(5, 9, seed=8, plies=60) == 60


def test_sizes_beyond_the_static_buffer_are_refused():
    L = pg.lib()
    h = C.c_void_p()
    limit = 8 << 20
    assert L.pgxgo_state_bytes(7000, 19) <= limit < L.pgxgo_state_bytes(9000, 19)
    assert L.pgxgo_init_static(C.byref(h), 9000, 19, 0, None) == -4 and not h.value
    assert L.pgxgo_strerror(-4) == b"size beyond the limit of the library's static buffer"
    assert L.pgxgo_init_static(C.byref(h), 0, 19, 0, None) == -1 and L.pgxgo_init_static(C.byref(h), 10, 13, 0, None) == -1
    assert L.pgxgo_init_static(None, 10, 19, 0, None) == -1
    assert L.pgxgo_init_static(C.byref(h), 7000, 19, 0, None) == 0 and h.value     # the largest sizes still fit
    assert L.pgxgo_sync(h) == 0 and L.pgxgo_destroy(h) == 0
