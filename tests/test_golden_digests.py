"""Regression pins: the oracle still produces the stored trajectory digests, and (GPU) the HIP path produces them too."""
import hashlib
import importlib.util
import os

import numpy as np
import pytest

import workloads

HERE = os.path.dirname(os.path.abspath(__file__))
spec = importlib.util.spec_from_file_location("make_digests", os.path.join(HERE, "golden", "make_digests.py"))
make_digests = importlib.util.module_from_spec(spec)
spec.loader.exec_module(make_digests)


def stored():
    out = {}
    for line in open(os.path.join(HERE, "golden", "trajectory_digests.txt")):
        if not line.startswith("#") and line.strip():
            k, v = line.split()
            out[k] = v
    return out


@pytest.mark.parametrize("ci", range(5))
def test_oracle_reproduces_stored_digests(ci):
    cfg = workloads.CONFIGS[ci]
    assert make_digests.digest_config(cfg) == stored()[cfg.name]


@pytest.mark.gpu
@pytest.mark.parametrize("ci", range(5))
def test_gpu_reproduces_stored_digests(ci):
    """The same digest from the HIP path: the full batch runs on the GPU (so that environments 0..7 sit in their
    real wavefronts), their outputs are hashed on the host."""
    import torch

    import paper_2303_17503_amd as pg
    cfg = workloads.CONFIGS[ci]
    B, N, P = cfg.batch, cfg.board_size, cfg.board_size ** 2
    E = make_digests.ENVS
    env = pg.GoEnv(B, N, seed=cfg.seed, komi_x2=cfg.komi_x2, auto_reset=cfg.auto_reset)
    mask, obs = env.new_mask(), env.new_obs()
    rew = torch.zeros((B, 2), dtype=torch.float32, device="cuda")
    term = torch.zeros(B, dtype=torch.uint8, device="cuda")
    env.bind_outputs(mask, obs, rew, term)
    start = workloads.start_times(cfg)
    st = None if start is None else torch.as_tensor(start, device="cuda")
    h = hashlib.blake2b(digest_size=8)
    T = cfg.warmup_max + min(cfg.steps, 300)
    a = env.random_actions(cfg.seed, 0, st)
    for t in range(T):
        a = env.step_sample(a, cfg.seed, t + 1, st)
        if t >= cfg.warmup_max:
            board = env.export_state()["board"][:E].cpu().numpy()
            for arr in (board, mask[:E, :P + 1].cpu().numpy(), obs[:E, :P * 17].cpu().numpy().reshape(E, N, N, 17),
                        rew[:E].cpu().numpy(), term[:E].cpu().numpy()):
                h.update(np.ascontiguousarray(arr).tobytes())
    assert h.hexdigest() == stored()[cfg.name]


@pytest.mark.parametrize("ci", range(3))
def test_hex_oracle_reproduces_stored_digests(ci):
    cfg = workloads.HEX_CONFIGS[ci]
    assert make_digests.digest_hex_config(cfg) == stored()[cfg.name]


@pytest.mark.gpu
@pytest.mark.parametrize("ci", range(3))
def test_gpu_reproduces_stored_hex_digests(ci):
    import torch

    import paper_2303_17503_amd as pg
    cfg = workloads.HEX_CONFIGS[ci]
    B, E = cfg.batch, make_digests.ENVS
    env = pg.HexEnv(B, seed=cfg.seed, auto_reset=cfg.auto_reset)
    mask, obs = env.new_mask(), env.new_obs()
    rew = torch.zeros((B, 2), dtype=torch.float32, device="cuda")
    term = torch.zeros(B, dtype=torch.uint8, device="cuda")
    env.bind_outputs(mask, obs, rew, term)
    h = hashlib.blake2b(digest_size=8)
    a = env.random_actions(cfg.seed, 0)
    for t in range(min(cfg.steps, 300)):
        a = env.step_sample(a, cfg.seed, t + 1)
        board = env.export_state()["board"][:E].cpu().numpy()
        for arr in (board, mask[:E].cpu().numpy(), obs[:E].cpu().numpy().reshape(E, 11, 11, 4), rew[:E].cpu().numpy(), term[:E].cpu().numpy()):
            h.update(np.ascontiguousarray(arr).tobytes())
    assert h.hexdigest() == stored()[cfg.name]
