"""GPU parity of the Hex kernels against the CPU Hex oracle, bit-exact, through the C ABI (include/pgxhex.h)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

N, P, A, OBS = 11, 121, 122, 484


def to_np(t):
    return t.detach().cpu().numpy()


class HexPair:
    """A HexEnv on the GPU and a HexOracle on the CPU over the same environments (ids: a sample of them)."""

    def __init__(self, batch, seed, auto_reset, ids=None, bind=True, mask=None, obs=None, mapping=0):
        import paper_2303_17503_amd as pg
        from oracle import hex as hx
        self.B = batch
        self.env = pg.HexEnv(batch, seed=seed, auto_reset=auto_reset)
        if mapping:
            assert self.env.set_mapping(mapping) == mapping       # 1: a board row per lane, 2: a board per lane
        self.ids = None if ids is None else np.asarray(ids, np.int32)
        self.orc = hx.HexOracle(batch if ids is None else len(ids), N, seed=seed, auto_reset=auto_reset, env_ids=self.ids)
        self.sel = None if ids is None else torch.as_tensor(self.ids.astype(np.int64), device="cuda")
        self.bound = bind
        self.n_compared = 0
        if bind:
            self.mask = self.env.new_mask() if mask is None else mask
            self.obs = self.env.new_obs() if obs is None else obs
            self.rew = torch.zeros((batch, 2), dtype=torch.float32, device="cuda")
            self.term = torch.zeros(batch, dtype=torch.uint8, device="cuda")
            self.env.bind_outputs(self.mask, self.obs, self.rew, self.term)

    def pick(self, t):
        return to_np(t if self.sel is None else t.index_select(0, self.sel))

    def compare(self, tag="", state=True, last_step=True):
        """last_step=False: skip the rewards / terminated values of the last step call (the rollout kernel reports them in its
        trajectory buffers only)."""
        e, o = self.env, self.orc
        self.n_compared += o.B
        mask = self.mask if self.bound else e.legal_mask()
        obs = self.obs if self.bound else e.observe()
        assert (self.pick(mask) == o.legal_mask()).all(), f"mask {tag}"
        assert (self.pick(obs).reshape(-1, N, N, 4) == o.observe()).all(), f"observation {tag}"
        if last_step:
            assert (self.pick(self.rew if self.bound else e.rewards()) == o.rewards()).all(), f"rewards {tag}"
            assert (self.pick(self.term if self.bound else e.terminated()) == o.terminated()).all(), f"terminated {tag}"
        assert (self.pick(e.current_player()) == o.current_player()).all(), f"current player {tag}"
        if state:
            g, c = e.export_state(), o.export_state()
            assert (self.pick(g["board"]) == c.board).all(), f"board {tag}"
            assert (self.pick(g["to_play"]) == c.to_play).all() and (self.pick(g["steps"]) == c.steps).all(), f"to_play/steps {tag}"
            assert (self.pick(g["terminated"]) == c.terminated).all() and (self.pick(g["black_player"]) == c.black_player).all(), f"flags {tag}"
            assert (self.pick(g["episode"]).astype(np.uint32) == c.episode).all(), f"episode {tag}"
            assert (self.pick(g["illegal"]).astype(np.uint32) == o.illegal_count()).all(), f"illegal {tag}"

    def step(self, a_cpu_full):
        """a_cpu_full: int32[B] actions of every environment."""
        a = np.ascontiguousarray(a_cpu_full, np.int32)
        self.env.step(torch.as_tensor(a, device="cuda"))
        self.orc.step(a if self.ids is None else a[self.ids])

    def rollout(self, seed, t0, t1, fused=False, state_every=1, start_t=None):
        """Random legal play for launches t0..t1-1; every drawn action and every output is compared."""
        e, o = self.env, self.orc
        st_dev = None if start_t is None else torch.as_tensor(start_t, device="cuda")
        st_cpu = None if start_t is None else (start_t if self.ids is None else start_t[self.ids])
        acts = [torch.empty(self.B, dtype=torch.int32, device="cuda") for _ in range(2)]
        e.random_actions(seed, t0, st_dev, out=acts[t0 & 1])
        for t in range(t0, t1):
            a_c = o.random_actions(seed, t, st_cpu)
            assert (self.pick(acts[t & 1]) == a_c).all(), f"drawn action t={t}"
            if fused:
                e.step_sample(acts[t & 1], seed, t + 1, st_dev, out=acts[(t + 1) & 1])
            else:
                e.step(acts[t & 1])
                e.random_actions(seed, t + 1, st_dev, out=acts[(t + 1) & 1])
            o.step(a_c)
            self.compare(f"t={t}", state=(t % state_every == 0) or t == t1 - 1)


def test_initial_state():
    for B in (1, 5, 13, 64):
        p = HexPair(B, seed=B, auto_reset=False)
        p.compare("init")
        m = to_np(p.mask)
        assert m[:, :P].all() and not m[:, P].any()


@pytest.mark.parametrize("B,seed", [(57, 1), (203, 2)])
def test_rollout_full_games(B, seed):
    p = HexPair(B, seed=seed, auto_reset=False)
    p.rollout(seed, 0, 125)
    assert to_np(p.term).all()              # no game outlasts 122 plies; finished games stay frozen
    assert p.n_compared == B * 125


@pytest.mark.parametrize("fused", [False, True])
def test_rollout_auto_reset(fused):
    B, seed = 333, 4
    p = HexPair(B, seed=seed, auto_reset=True)
    p.rollout(seed, 0, 450, fused=fused, state_every=7)
    assert to_np(p.env.export_state()["episode"]).min() >= 2


def test_rollout_with_staggered_starts():
    B, seed = 77, 9
    start = (np.arange(B) % 40).astype(np.int32)
    p = HexPair(B, seed=seed, auto_reset=True)
    p.rollout(seed, 0, 200, fused=True, start_t=start)


def test_start_times_negative_zero_and_positive():
    """start_t is compared as a signed number by every path: negative and zero entries never wait.  The same start array
    through random_actions + step, step_sample, and the rollout kernel (which must equal the loop of the first two)."""
    B, seed, T = 83, 12, 60
    start = np.array([-2147483648, -5, -1, 0, 1, 7, 30][: 7] * 12, np.int32)[:B]
    for fused in (False, True):
        p = HexPair(B, seed=seed, auto_reset=True)
        p.rollout(seed, 0, T, fused=fused, start_t=start)
        assert (to_np(p.env.export_state()["steps"])[start <= 0] > 0).all()
    q = HexPair(B, seed=seed, auto_reset=True, bind=False)
    tr = alloc_traj(T, B)
    q.env.rollout(T, seed, 0, start_t=torch.as_tensor(start, device="cuda"), slices=T, **tr)
    got = {k: to_np(v) for k, v in tr.items()}
    for t in range(T):
        a = q.orc.random_actions(seed, t, start)
        assert (got["actions"][t] == a).all() and ((a >= 0) == (t >= start)).all(), f"action t={t}"
        q.orc.step(a)
        assert (got["mask"][t] == q.orc.legal_mask()).all(), f"mask t={t}"
    q.compare("state after the launch", last_step=False)


@pytest.mark.parametrize("B", [1, 5, 63, 64, 65, 130, 333])
@pytest.mark.parametrize("fused", [False, True])
def test_board_per_lane_mapping(B, fused):
    """The step kernels with a whole board per lane (the mapping used from ~28 k games on), forced at small ragged batches:
    full wavefronts, partly filled ones, several blocks; random play with auto-reset and staggered starts, every ply compared."""
    seed = 40 + B
    start = ((np.arange(B) * 7) % 30 - 3).astype(np.int32)
    p = HexPair(B, seed=seed, auto_reset=True, mapping=2)
    p.rollout(seed, 0, 260, fused=fused, state_every=13, start_t=start)
    assert to_np(p.env.export_state()["episode"]).max() >= 1
    q = HexPair(B, seed=seed + 1, auto_reset=False, mapping=2)
    q.rollout(seed + 1, 0, 125, fused=fused, state_every=25)
    assert to_np(q.term).all()


def test_board_per_lane_swap_illegal_frozen_and_skip():
    B = 70
    p = HexPair(B, seed=3, auto_reset=False, mapping=2)
    first = (np.arange(B) * 5 + 2) % P
    p.step(first)
    p.compare("after the first stone")
    assert to_np(p.mask)[:, P].all()
    a = np.where(np.arange(B) % 2 == 0, P, (first + 1) % P)         # every other game swaps
    p.step(a)
    p.compare("after the swap")
    bd = to_np(p.env.export_state()["board"]).reshape(B, N, N)
    for b in range(0, B, 2):
        r, c = divmod(int(first[b]), N)
        assert bd[b, c, r] == -1 and np.abs(bd[b]).sum() == 1
    kinds = np.arange(B) % 7
    occupied = np.array([int(np.flatnonzero(bd[b].reshape(-1))[0]) for b in range(B)])
    a = np.select([kinds == 0, kinds == 1, kinds == 2, kinds == 3, kinds == 4, kinds == 5], [occupied, 121, -7, 5000, -1, 122], default=60)
    p.step(a)                                                       # occupied / swap off its turn / out of range x3 / skip / maybe legal
    p.compare("illegal mix")
    p.step(np.full(B, 61))                                          # finished games stay frozen
    p.compare("frozen")
    p.rollout(3, 4, 130)
    for mapping in (1, 2):                                          # switching the mapping mid-game changes nothing
        assert p.env.set_mapping(mapping) == mapping
        p.rollout(3, 130, 140)


def test_swap_rule():
    B = 23
    p = HexPair(B, seed=3, auto_reset=False)
    first = (np.arange(B) * 5 + 2) % P
    p.step(first)
    p.compare("after the first stone")
    assert to_np(p.mask)[:, P].all()                                 # the swap is on offer now
    a = np.where(np.arange(B) % 2 == 0, P, (first + 1) % P)         # every other game swaps
    p.step(a)
    p.compare("after the swap")
    bd = to_np(p.env.export_state()["board"]).reshape(B, N, N)
    for b in range(0, B, 2):
        r, c = divmod(int(first[b]), N)
        assert bd[b, c, r] == -1 and np.abs(bd[b]).sum() == 1
    assert not to_np(p.mask)[:, P].any()
    p.rollout(3, 2, 124)


def test_illegal_frozen_and_skip():
    B = 31
    p = HexPair(B, seed=5, auto_reset=False)
    p.step(np.full(B, 60))
    kinds = np.arange(B) % 6
    a = np.select([kinds == 0, kinds == 1, kinds == 2, kinds == 3, kinds == 4], [60, 122, -7, 5000, -1], default=61)
    p.step(a)                                                       # occupied / out of range x3 / skip / legal
    p.compare("illegal mix")
    t = to_np(p.term)
    assert (t[kinds <= 3] == 1).all() and (t[kinds >= 4] == 0).all()
    a2 = np.select([kinds == 4], [P], default=3)                    # the skipped games may still swap; others: frozen or a legal stone
    p.step(a2)
    p.compare("frozen / late swap")
    p.step(np.full(B, P))                                           # swap on the wrong turn everywhere it is still live
    p.compare("swap on the wrong turn")
    assert to_np(p.term).all()
    p.step(np.full(B, 0))
    p.compare("all frozen")
    assert (to_np(p.rew) == 0).all()


def test_illegal_with_auto_reset():
    B = 19
    p = HexPair(B, seed=6, auto_reset=True)
    p.step(np.full(B, 10))
    p.step(np.where(np.arange(B) % 3 == 0, 10, 11))
    p.compare("occupied cell with auto-reset")
    st = p.env.export_state()
    assert (to_np(st["episode"])[::3] == 1).all() and (to_np(st["illegal"])[::3] == 1).all()
    p.rollout(6, 2, 150)


def test_misaligned_output_bases():
    B = 29
    for off_m, off_o in ((1, 7), (15, 9), (4, 12)):
        raw_m = torch.zeros(B * A + 32, dtype=torch.uint8, device="cuda")
        raw_o = torch.zeros(B * OBS + 32, dtype=torch.uint8, device="cuda")
        raw_m.fill_(0xAB); raw_o.fill_(0xCD)
        mask = raw_m[off_m: off_m + B * A].view(B, A)
        obs = raw_o[off_o: off_o + B * OBS].view(B, OBS)
        p = HexPair(B, seed=off_m, auto_reset=True, mask=mask, obs=obs)
        p.rollout(off_m, 0, 60, fused=True, state_every=10)
        assert (to_np(raw_m[:off_m]) == 0xAB).all() and (to_np(raw_m[off_m + B * A:]) == 0xAB).all()   # nothing written outside
        assert (to_np(raw_o[:off_o]) == 0xCD).all() and (to_np(raw_o[off_o + B * OBS:]) == 0xCD).all()


def test_unbound_outputs_and_reset():
    B = 41
    p = HexPair(B, seed=8, auto_reset=False, bind=False)
    for t in range(40):
        a = p.orc.random_actions(8, t)
        p.step(a)
        if t % 8 == 0:
            p.compare(f"t={t}")
    p.env.reset(); p.orc.reset()
    p.compare("after reset")
    assert (to_np(p.env.export_state()["episode"]) == 1).all()


def test_import_export_continue():
    from oracle import hex as hx
    B, seed = 66, 10
    src = hx.HexOracle(B, N, seed=seed)
    for t in range(55):
        src.step(src.random_actions(seed, t))
    s = src.export_state()
    s.steps[:7] = 1; s.board[:7] = 0; s.board[np.arange(7), np.arange(7) * 13] = 1; s.to_play[:7] = -1; s.terminated[:7] = 0   # swap on offer
    p = HexPair(B, seed=seed, auto_reset=False)
    p.orc.import_state(s)
    p.env.import_state({"board": torch.as_tensor(s.board, device="cuda"), "to_play": torch.as_tensor(s.to_play, device="cuda"),
                        "steps": torch.as_tensor(s.steps, device="cuda"), "terminated": torch.as_tensor(s.terminated, device="cuda"),
                        "black_player": torch.as_tensor(s.black_player, device="cuda"),
                        "episode": torch.as_tensor(s.episode.astype(np.int32), device="cuda")})
    p.compare("after import")
    assert to_np(p.mask)[:7, P].all()
    p.rollout(seed, 55, 180)


def whole_batch_properties(env, mask, obs):
    """Facts that hold for every environment at any size, checked on the device tensors."""
    st = env.export_state()
    occ = (st["board"] != 0)
    assert bool(((mask[:, :P] == 1) == ~occ).all())                                  # legal cells = empty cells
    assert bool((mask[:, P] == (st["steps"] == 1)).all())                            # swap exactly on the second turn
    o = obs.view(-1, P, 4)
    assert bool(((o[:, :, 0] + o[:, :, 1]) == occ).all())
    assert bool((o[:, :, 2] == (st["to_play"] == 1)[:, None]).all())
    assert bool((o[:, :, 3] == (st["steps"] == 1)[:, None]).all())
    assert bool((o <= 1).all())


@pytest.mark.parametrize("k", [0, 1, 2])
def test_full_size_configurations(k):
    """The three Hex workloads at full batch, in the launch shape bench.py times (fused sampler); the oracle replays
    every environment (1024 games) or a seeded sample for every ply (test_gpu_full_parity.py replays all of them),
    and the whole-batch properties are checked here."""
    import workloads
    cfg = workloads.HEX_CONFIGS[k]
    rng = np.random.default_rng(100 + k)
    if k == 0:
        ids = None
    else:
        n = 220 if k == 1 else 120
        ids = None if n >= cfg.batch else np.unique(np.concatenate([[0, 1, 4, 5, cfg.batch - 1, cfg.batch - 2, cfg.batch - 5], rng.integers(0, cfg.batch, n)]))
    p = HexPair(cfg.batch, seed=cfg.seed, auto_reset=cfg.auto_reset, ids=ids)
    plies = cfg.steps if k < 2 else 400
    p.rollout(cfg.seed, 0, plies, fused=True, state_every=50)
    whole_batch_properties(p.env, p.mask, p.obs)
    assert p.n_compared == (cfg.batch if ids is None else len(ids)) * plies


@pytest.mark.parametrize("mapping", [1, 2])
def test_outputs_beyond_four_gibibytes(mapping):
    """8900003 games: the observation tensor is 4.31 GB, so the byte offsets of the last 26000 games do not fit 32 bits,
    and the batch is no multiple of a wavefront's games.  The oracle replays the first games, the games on both sides of
    the 4 GiB offset and the last ones, in both lane mappings."""
    B, seed, T = 8900003, 17, 24
    cross = (1 << 32) // OBS
    ids = np.concatenate([np.arange(0, 320), np.arange(cross - 160, cross + 160), np.arange(B - 320, B)])
    p = HexPair(B, seed=seed, auto_reset=True, ids=ids, mapping=mapping)
    assert p.obs.numel() > (1 << 32)
    p.rollout(seed, 0, T, fused=True, state_every=12)
    assert p.n_compared == len(ids) * T
    assert bool((p.mask.sum(dim=1) > 0).all())          # every game has a legal action
    del p
    torch.cuda.empty_cache()


def alloc_traj(S, B):
    return dict(actions=torch.empty((S, B), dtype=torch.int32, device="cuda"),
                rewards=torch.empty((S, B, 2), dtype=torch.float32, device="cuda"),
                terminated=torch.empty((S, B), dtype=torch.uint8, device="cuda"),
                mask=torch.empty((S, B, A), dtype=torch.uint8, device="cuda"),
                obs=torch.empty((S, B, OBS), dtype=torch.uint8, device="cuda"))


@pytest.mark.parametrize("mapping", [1, 2])
@pytest.mark.parametrize("B,auto_reset,stagger", [(131, True, False), (64, False, False), (77, True, True)])
def test_rollout_kernel_records_the_trajectory(B, auto_reset, stagger, mapping):
    """One launch of T plies against ply-by-ply oracle stepping: every slice of the recorded trajectory is compared
    (both mappings: a board row per lane, a board per lane)."""
    seed, T = 31, 140
    p = HexPair(B, seed=seed, auto_reset=auto_reset, bind=False, mapping=mapping)
    start = (np.arange(B) % 23).astype(np.int32) if stagger else None
    tr = alloc_traj(T, B)
    p.env.rollout(T, seed, 0, start_t=None if start is None else torch.as_tensor(start, device="cuda"), slices=T, **tr)
    got = {k: to_np(v) for k, v in tr.items()}
    for t in range(T):
        a = p.orc.random_actions(seed, t, start)
        assert (got["actions"][t] == a).all(), f"action t={t}"
        p.orc.step(a)
        live = a >= 0
        assert (got["mask"][t] == p.orc.legal_mask()).all(), f"mask t={t}"
        assert (got["obs"][t].reshape(B, N, N, 4) == p.orc.observe()).all(), f"observation t={t}"
        assert (got["rewards"][t][live] == p.orc.rewards()[live]).all() and (got["rewards"][t][~live] == 0).all(), f"rewards t={t}"
        assert (got["terminated"][t][live] == p.orc.terminated()[live]).all() and (got["terminated"][t][~live] == 0).all(), f"terminated t={t}"
    p.compare("state after the launch", last_step=False)


def test_rollout_kernel_single_slice_full_batch():
    """The launch shape of bench.py's rollout mode: every ply overwrites one set of buffers; sampled environments."""
    import workloads
    cfg = workloads.HEX_CONFIGS[1]
    ids = np.unique(np.concatenate([[0, 4, 5, cfg.batch - 1], np.random.default_rng(3).integers(0, cfg.batch, 150)]))
    p = HexPair(cfg.batch, seed=cfg.seed, auto_reset=True, ids=ids, bind=False)
    tr = alloc_traj(1, cfg.batch)
    t = 0
    for L_ in (50, 1, 37, 50):
        p.env.rollout(L_, cfg.seed, t, slices=1, **tr)
        for i in range(L_):
            a = p.orc.random_actions(cfg.seed, t + i)
            p.orc.step(a)
        t += L_
        assert (p.pick(tr["actions"][0]) == a).all()
        assert (p.pick(tr["mask"][0]) == p.orc.legal_mask()).all() and (p.pick(tr["obs"][0]).reshape(-1, N, N, 4) == p.orc.observe()).all()
        assert (p.pick(tr["rewards"][0]) == p.orc.rewards()).all() and (p.pick(tr["terminated"][0]) == p.orc.terminated()).all()
        p.compare(f"after {t} plies", last_step=False)


@pytest.mark.parametrize("B", [1, 2, 6])
def test_tiny_batches(B):
    p = HexPair(B, seed=80 + B, auto_reset=True)
    p.rollout(80 + B, 0, 300, fused=True, state_every=20)
    assert to_np(p.env.export_state()["episode"]).min() >= 1
    q = HexPair(B, seed=81, auto_reset=True, bind=False)
    tr = alloc_traj(1, B)
    q.env.rollout(130, 81, 0, slices=1, **tr)
    for t in range(130):
        a = q.orc.random_actions(81, t)
        q.orc.step(a)
    assert (to_np(tr["actions"][0]) == a).all() and (to_np(tr["mask"][0]) == q.orc.legal_mask()).all()
    q.compare("after the launch", last_step=False)
