"""Helpers of the GPU parity tests: run the HIP path and the CPU oracle side by side and compare bit-exactly."""
import numpy as np
import torch

import oracle
import paper_2303_17503_amd as pg


def to_np(t):
    return t.detach().cpu().numpy()


class Pair:
    """A GoEnv on the GPU and a GoOracle on the CPU over the same environments.

    ids: the oracle replays only these global environment indices (sampled comparison at large batch);
    None = every environment."""

    def __init__(self, batch, N, seed, auto_reset, ids=None, komi_x2=15, max_steps=0, obs_pitch=0, mask_pitch=0, bind=True, emit_obs=True,
                 superko=False):
        self.B, self.N, self.P = batch, N, N * N
        self.env = pg.GoEnv(batch, N, seed=seed, komi_x2=komi_x2, max_steps=max_steps, auto_reset=auto_reset, obs_pitch=obs_pitch, mask_pitch=mask_pitch)
        self.ids = None if ids is None else np.asarray(ids, np.int32)
        nb = batch if ids is None else len(ids)
        self.orc = oracle.GoOracle(nb, N, seed=seed, komi_x2=komi_x2, max_steps=max_steps, auto_reset=auto_reset, env_ids=self.ids, superko=superko)
        if superko:
            self.env.enable_superko(superko)     # True / 1: at play time; "mask" / 2: honoured by the legal mask
        self.sel = None if ids is None else torch.as_tensor(self.ids.astype(np.int64), device="cuda")
        self.bound = bind
        self.n_compared = 0      # environment-plies whose outputs were compared
        self.n_actions = 0
        if bind:
            self.mask = self.env.new_mask()
            self.obs = self.env.new_obs() if emit_obs else None
            self.rew = torch.zeros((batch, 2), dtype=torch.float32, device="cuda")
            self.term = torch.zeros(batch, dtype=torch.uint8, device="cuda")
            self.env.bind_outputs(self.mask, self.obs, self.rew, self.term)

    def pick(self, t):
        return to_np(t if self.sel is None else t.index_select(0, self.sel))

    def gpu_mask(self):
        m = self.mask if self.bound else self.env.legal_mask()
        return self.pick(m)[:, : self.P + 1]

    def gpu_obs(self):
        o = self.obs if (self.bound and self.obs is not None) else self.env.observe()
        return self.pick(o)[:, : self.P * 17].reshape(-1, self.N, self.N, 17)

    def gpu_rew(self):
        return self.pick(self.rew if self.bound else self.env.rewards())

    def gpu_term(self):
        return self.pick(self.term if self.bound else self.env.terminated())

    def step(self, a_gpu, a_cpu):
        self.env.step(a_gpu)
        self.orc.step(a_cpu)

    def compare(self, tag="", state=True, obs=True):
        o = self.orc
        self.n_compared += o.B
        assert (self.gpu_mask() == o.legal_mask()).all(), f"mask {tag}"
        if obs:
            assert (self.gpu_obs() == o.observe()).all(), f"obs {tag}"
        r_g, r_c = self.gpu_rew(), o.rewards()
        assert r_g.tobytes() == r_c.tobytes(), f"rewards {tag}"   # exact bytes: -0.0 must not pass for 0.0
        assert (self.gpu_term() == o.terminated()).all(), f"terminated {tag}"
        assert (self.pick(self.env.current_player()) == o.current_player()).all(), f"current_player {tag}"
        if state:
            g, c = self.env.export_state(), o.export_state()
            for name in ("board", "history", "ko", "to_play", "steps", "passes", "terminated", "black_player", "episode"):
                gv = self.pick(g[name])
                cv = getattr(c, name)
                assert (gv.astype(np.int64) == cv.astype(np.int64)).all(), f"{name} {tag}"
            assert (self.pick(g["illegal"]).astype(np.int64) == o.illegal_count().astype(np.int64)).all(), f"illegal {tag}"

    def rollout(self, seed, t0, t1, start_t=None, every=1, state_every=None, obs=True, fused=False):
        """Random legal play for launches t0..t1-1, actions sampled on each side from its own mask."""
        st_g = None if start_t is None else torch.as_tensor(start_t, device="cuda")
        st_c = None if start_t is None else (start_t if self.ids is None else start_t[self.ids])
        a_g = self.env.random_actions(seed, t0, st_g)
        for t in range(t0, t1):
            a_c = self.orc.random_actions(seed, t, st_c)
            assert (self.pick(a_g) == a_c).all(), f"actions t={t}"
            self.n_actions += int((a_c >= 0).sum())
            if fused and t + 1 < t1:
                nxt = self.env.step_sample(a_g, seed, t + 1, st_g)
                self.orc.step(a_c)
                a_g = nxt
            else:
                self.step(a_g, a_c)
                if t + 1 < t1:
                    a_g = self.env.random_actions(seed, t + 1, st_g)
            if (t - t0) % every == 0 or t == t1 - 1:
                full = state_every is not None and ((t - t0) % state_every == 0 or t == t1 - 1)
                self.compare(f"t={t}", state=full, obs=obs)
