"""The step entry points only enqueue kernels, so a caller may capture them in a HIP graph.  Each replay is checked
against the CPU oracle, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import oracle
import paper_2303_17503_amd as pg
from oracle import hex as hx

pytestmark = pytest.mark.gpu


def to_np(t):
    return t.detach().cpu().numpy()


def run(make_env, make_oracle, obs_shape, B, seed, replays=6):
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        env = make_env()
        orc = make_oracle()
        mask, obs = env.new_mask(), env.new_obs()
        rew = torch.zeros((B, 2), dtype=torch.float32, device="cuda")
        term = torch.zeros(B, dtype=torch.uint8, device="cuda")
        env.bind_outputs(mask, obs, rew, term)
        acts = [torch.empty(B, dtype=torch.int32, device="cuda") for _ in range(2)]
        env.random_actions(seed, 0, out=acts[0])
        a_c = orc.random_actions(seed, 0)
        s.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):           # two plies; the sampler counters 1 and 2 are baked into the graph
            env.step_sample(acts[0], seed, 1, out=acts[1])
            env.step_sample(acts[1], seed, 2, out=acts[0])
        s.synchronize()
        for rep in range(replays):
            g.replay()
            cur = env.current_player()                # eager work of the same handle between the replays
            s.synchronize()
            orc.step(a_c)
            a1 = orc.random_actions(seed, 1)
            assert (to_np(acts[1]) == a1).all(), f"replay {rep}: first drawn action"
            orc.step(a1)
            a_c = orc.random_actions(seed, 2)
            assert (to_np(acts[0]) == a_c).all(), f"replay {rep}: second drawn action"
            assert (to_np(mask) == orc.legal_mask()).all(), f"replay {rep}: mask"
            assert (to_np(obs).reshape(obs_shape) == orc.observe()).all(), f"replay {rep}: observation"
            assert (to_np(rew) == orc.rewards()).all() and (to_np(term) == orc.terminated()).all(), f"replay {rep}: rewards"
            assert (to_np(cur) == orc.current_player()).all(), f"replay {rep}: current player"
        # and eager stepping still works after the replays
        nxt = env.step_sample(acts[0], seed, 3)
        orc.step(a_c)
        assert (to_np(nxt) == orc.random_actions(seed, 3)).all() and (to_np(mask) == orc.legal_mask()).all()


def test_go_step_in_a_graph():
    B, N, seed = 200, 9, 21
    run(lambda: pg.GoEnv(B, N, seed=seed, auto_reset=True), lambda: oracle.GoOracle(B, N, seed=seed, auto_reset=True), (B, N, N, 17), B, seed)


def test_go19_step_in_a_graph():
    B, N, seed = 100, 19, 22
    run(lambda: pg.GoEnv(B, N, seed=seed, auto_reset=True), lambda: oracle.GoOracle(B, N, seed=seed, auto_reset=True), (B, N, N, 17), B, seed, replays=4)


def test_hex_step_in_a_graph():
    B, seed = 333, 23
    run(lambda: pg.HexEnv(B, seed=seed, auto_reset=True), lambda: hx.HexOracle(B, 11, seed=seed, auto_reset=True), (B, 11, 11, 4), B, seed, replays=8)


def test_two_handles_on_two_streams():
    """Handles share nothing: two batches stepped concurrently on their own streams both follow the oracle."""
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    B1, B2, seed = 300, 500, 31
    with torch.cuda.stream(s1):
        e1 = pg.GoEnv(B1, 19, seed=seed, auto_reset=True)
        m1, o1 = e1.new_mask(), e1.new_obs()
        e1.bind_outputs(m1, o1, None, None)
        a1 = e1.random_actions(seed, 0)
    with torch.cuda.stream(s2):
        e2 = pg.HexEnv(B2, seed=seed, auto_reset=True)
        m2, o2 = e2.new_mask(), e2.new_obs()
        e2.bind_outputs(m2, o2, None, None)
        a2 = e2.random_actions(seed, 0)
    c1 = oracle.GoOracle(B1, 19, seed=seed, auto_reset=True)
    c2 = hx.HexOracle(B2, 11, seed=seed, auto_reset=True)
    T = 150
    for t in range(T):                       # no synchronisation inside the loop: the two launch chains overlap freely
        with torch.cuda.stream(s1):
            a1 = e1.step_sample(a1, seed, t + 1)
        with torch.cuda.stream(s2):
            a2 = e2.step_sample(a2, seed, t + 1)
    for t in range(T):
        c1.step(c1.random_actions(seed, t))
        c2.step(c2.random_actions(seed, t))
    s1.synchronize(); s2.synchronize()
    assert (to_np(m1) == c1.legal_mask()).all() and (to_np(o1).reshape(B1, 19, 19, 17) == c1.observe()).all()
    assert (to_np(a1) == c1.random_actions(seed, T)).all()
    assert (to_np(m2) == c2.legal_mask()).all() and (to_np(o2).reshape(B2, 11, 11, 4) == c2.observe()).all()
    assert (to_np(a2) == c2.random_actions(seed, T)).all()
