"""GPU parity: the HIP path against the CPU oracle, bit-exact, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import positions as pos
import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2303_17503_amd as pg
    pg.lib()   # fails loudly if the HIP library is not built


def test_lane_shift_layout():
    import paper_2303_17503_amd as pg
    v = torch.arange(100, 164, dtype=torch.int32, device="cuda")
    below, above = pg.lane_shift_probe(v)
    torch.cuda.synchronize()
    assert below.cpu().tolist() == [0] + list(range(100, 163))
    assert above.cpu().tolist() == list(range(101, 164)) + [0]


def test_initial_state_and_getters():
    from gpu_common import Pair
    for N, B in ((9, 7), (19, 5), (19, 64)):
        p = Pair(B, N, seed=11, auto_reset=False, bind=False)
        p.compare("init unbound")
        p = Pair(B, N, seed=11, auto_reset=False, bind=True)
        p.compare("init bound")


def test_hand_built_scripts_on_gpu():
    """All hand-written rule scripts at once, one environment each; shorter scripts idle with the skip action."""
    from gpu_common import Pair
    names = sorted(pos.SCRIPTS)
    B, T = len(names), max(len(pos.SCRIPTS[n]["moves"]) for n in names)
    p = Pair(B, 9, seed=1, auto_reset=False)
    for t in range(T):
        a = np.array([pos.idx(pos.SCRIPTS[n]["moves"][t]) if t < len(pos.SCRIPTS[n]["moves"]) else -1 for n in names], np.int32)
        p.step(torch.as_tensor(a, device="cuda"), a)
        p.compare(f"script ply {t}")
    g = p.env.export_state()
    board, ko, tp = g["board"].cpu().numpy(), g["ko"].cpu().numpy(), g["to_play"].cpu().numpy()
    mask = p.gpu_mask()
    for i, n in enumerate(names):
        sc = pos.SCRIPTS[n]
        assert board[i].tolist() == sc["board"], n
        assert ko[i] == (-1 if sc["ko"] == -1 else sc["ko"][0] * 9 + sc["ko"][1]), n
        assert tp[i] == sc["to_play"], n
        for rc in sc.get("illegal_next", []):
            assert mask[i, rc[0] * 9 + rc[1]] == 0, (n, rc)
        for rc in sc.get("legal_next", []):
            assert mask[i, rc[0] * 9 + rc[1]] == 1, (n, rc)


@pytest.mark.parametrize("N,B,T,auto_reset", [(9, 256, 162, False), (9, 100, 400, True), (19, 64, 722, False), (19, 50, 900, True)])
def test_rollout_every_env_every_ply(N, B, T, auto_reset):
    """Sizes that span several wavefronts with a ragged last one (B not a multiple of boards per wavefront)."""
    from gpu_common import Pair
    p = Pair(B, N, seed=N + B, auto_reset=auto_reset)
    p.rollout(N + B, 0, T, every=1, state_every=25)
    assert p.n_compared == B * T and p.n_actions == B * T
    s = p.orc.export_state()
    assert s.episode.max() >= 1 if auto_reset else (s.terminated == 1).all()


@pytest.mark.parametrize("N", [9, 19])
def test_rollout_fused_sampler_and_unbound_getters(N):
    from gpu_common import Pair
    p = Pair(40, N, seed=5, auto_reset=True, bind=True)
    p.rollout(5, 0, 300, every=1, state_every=50, fused=True)
    q = Pair(10, N, seed=6, auto_reset=True, bind=False)
    q.rollout(6, 0, 120, every=3, state_every=30)


@pytest.mark.parametrize("obs_pitch,mask_pitch", [(6144, 368), (6137 + 3, 362 + 5)])
def test_padded_and_misaligned_pitches(obs_pitch, mask_pitch):
    from gpu_common import Pair
    p = Pair(20, 19, seed=8, auto_reset=True, obs_pitch=obs_pitch, mask_pitch=mask_pitch)
    p.obs.fill_(7); p.mask.fill_(7)
    p.env.bind_outputs(p.mask, p.obs, p.rew, p.term)
    p.rollout(8, 0, 150, every=1, state_every=50)
    # bytes between the environments' records are never touched
    assert (p.obs[:, 6137:] == 7).all() and (p.mask[:, 362:] == 7).all()


@pytest.mark.parametrize("N,B", [(19, 20), (19, 7), (9, 50), (9, 4)])
def test_line_padded_pitches(N, B):
    """Pitches rounded up to 128-byte lines: the pad bytes belong to the record and are written as zeros; step, the
    getters, the rollout kernel and the slot call in that layout, with ragged last wavefronts."""
    from gpu_common import Pair
    import paper_2303_17503_amd as pg
    P = N * N
    op, mp = (P * 17 + 127) // 128 * 128, (P + 1 + 127) // 128 * 128
    p = Pair(B, N, seed=8, auto_reset=True, obs_pitch=op, mask_pitch=mp)
    assert p.env.obs_pitch == op and p.env.mask_pitch == mp
    p.obs.fill_(7); p.mask.fill_(7)
    p.rollout(8, 0, 150, every=1, state_every=50)
    assert (p.obs[:, P * 17:] == 0).all() and (p.mask[:, P + 1:] == 0).all()
    assert (p.env.obs_view(p.obs).cpu().numpy() == p.orc.observe()).all()
    got_o, got_m = p.env.observe(), p.env.legal_mask()
    assert torch.equal(got_o, p.obs) and torch.equal(got_m, p.mask)
    # the same games through GoEnv(line_padded=True) and the rollout kernel, every ply in its own slice
    T = 40
    e = pg.GoEnv(B, N, seed=8, auto_reset=True, line_padded=True)
    assert (e.obs_pitch, e.mask_pitch) == (op, mp)
    obs = torch.full((T, B, op), 7, dtype=torch.uint8, device="cuda")
    mask = torch.full((T, B, mp), 7, dtype=torch.uint8, device="cuda")
    acts = torch.empty((T, B), dtype=torch.int32, device="cuda")
    e.rollout(T, 8, 0, slices=T, actions=acts, mask=mask, obs=obs)
    q = Pair(B, N, seed=8, auto_reset=True, bind=False)
    for t in range(T):
        a = q.orc.random_actions(8, t)
        assert (acts[t].cpu().numpy() == a).all()
        q.orc.step(a)
        assert (mask[t, :, :P + 1].cpu().numpy() == q.orc.legal_mask()).all(), t
        assert (obs[t, :, :P * 17].cpu().numpy().reshape(B, N, N, 17) == q.orc.observe()).all(), t
    assert (obs[:, :, P * 17:] == 0).all() and (mask[:, :, P + 1:] == 0).all()
    # slot call: every game stepped into itself with a random legal action
    idx = torch.arange(B, dtype=torch.int32, device="cuda")
    a = q.orc.random_actions(8, T)
    m2, o2 = e.new_mask().fill_(7), e.new_obs().fill_(7)
    e.step_slots(idx, torch.as_tensor(a, device="cuda"), idx, mask=m2, obs=o2)
    q.orc.step(a)
    assert (m2[:, :P + 1].cpu().numpy() == q.orc.legal_mask()).all()
    assert (e.obs_view(o2).cpu().numpy() == q.orc.observe()).all()
    assert (o2[:, P * 17:] == 0).all() and (m2[:, P + 1:] == 0).all()


def test_fill_probe_fills_exactly_its_range():
    """The measurement helper stores through the same 16-byte store the kernels use for whole lines."""
    import paper_2303_17503_amd as pg
    raw = torch.full((1 << 20,), 7, dtype=torch.uint8, device="cuda")
    for kind in (0, 1, 2):
        for off, n in ((0, 16), (16, 4096), (48, 100000 * 16), (0, (1 << 20) - 64)):
            raw.fill_(7)
            pg.fill_probe(raw[off: off + n], 0x01020304 + kind, kind=kind)
            torch.cuda.synchronize()
            got = raw.cpu().numpy()
            assert (got[:off] == 7).all() and (got[off + n:] == 7).all()
            assert (got[off: off + n].view(np.uint32) == 0x01020304 + kind).all()
    with pytest.raises(pg.PgxGoError):
        pg.fill_probe(raw[:64], 1, kind=3)


def test_misaligned_output_base_pointers():
    from gpu_common import Pair
    import paper_2303_17503_amd as pg
    B, N = 9, 9
    p = Pair(B, N, seed=3, auto_reset=True, bind=False)
    raw_o = torch.full((B * 1377 + 64,), 9, dtype=torch.uint8, device="cuda")
    raw_m = torch.full((B * 82 + 64,), 9, dtype=torch.uint8, device="cuda")
    for off in (1, 5, 16, 31):
        ob = raw_o[off: off + B * 1377].view(B, 1377)
        mk = raw_m[off: off + B * 82].view(B, 82)
        raw_o.fill_(9); raw_m.fill_(9)
        p.env.bind_outputs(mk, ob, None, None)
        a = p.env.random_actions(3, off)
        a_c = p.orc.random_actions(3, off)
        p.step(a, a_c)
        assert (ob.cpu().numpy().reshape(B, N, N, 17) == p.orc.observe()).all()
        assert (mk.cpu().numpy() == p.orc.legal_mask()).all()
        assert (raw_o[:off] == 9).all() and (raw_o[off + B * 1377:] == 9).all()
        assert (raw_m[:off] == 9).all() and (raw_m[off + B * 82:] == 9).all()
    p.env.bind_outputs(None, None, None, None)


def test_illegal_actions_frozen_games_and_skips():
    from gpu_common import Pair
    for auto_reset in (False, True):
        B, N = 30, 9
        p = Pair(B, N, seed=2, auto_reset=auto_reset)
        rng = np.random.default_rng(0)
        for t in range(60):
            a = p.orc.random_actions(2, t)
            kind = rng.integers(0, 12, B)
            a = np.where(kind == 0, rng.integers(0, 81, B), a)        # often an occupied or suicidal point
            a = np.where(kind == 1, -1, a)                            # skip
            a = np.where(kind == 2, 500, a)                           # out of range
            a = np.where(kind == 3, -5, a)
            a = a.astype(np.int32)
            p.step(torch.as_tensor(a, device="cuda"), a)
            p.compare(f"t={t}")
        assert p.orc.illegal_count().sum() > 0


def test_import_export_round_trip_and_continue():
    """Mid-game positions produced by the oracle are imported into the GPU state (which rebuilds its private
    chain data) and play continues in lock step."""
    from gpu_common import Pair
    for N, B in ((9, 33), (19, 10)):
        src = oracle.GoOracle(B, N, seed=77, auto_reset=False)
        for t in range(N * N):
            src.step(src.random_actions(77, t))
        st = src.export_state()
        p = Pair(B, N, seed=77, auto_reset=False)
        p.orc.import_state(st)
        dev = {k: torch.as_tensor(getattr(st, k), device="cuda") for k in st.__slots__}
        dev["episode"] = dev["episode"].to(torch.int32)
        p.env.import_state(dev)
        p.compare("after import")
        p.rollout(78, 1000, 1000 + N * N, every=1, state_every=20)


def test_reset_all():
    from gpu_common import Pair
    p = Pair(12, 9, seed=4, auto_reset=False)
    p.rollout(4, 0, 30, every=10)
    p.env.reset(); p.orc.reset()
    p.compare("after reset")
    p.rollout(4, 30, 60, every=10, state_every=10)


# ---- the five benchmark configurations at full size, in the launch configuration the benchmark times ----
def sampled_ids(batch, n, seed):
    rng = np.random.default_rng(seed)
    ids = np.unique(np.concatenate([[0, 1, 2, batch - 1, batch - 2], rng.choice(batch, n, replace=False)]))
    return ids.astype(np.int32)


@pytest.mark.parametrize("ci", [0, 1, 2, 3, 4])
def test_benchmark_configs_full_size(ci):
    """Full batch on the GPU; the oracle replays a seeded sample of environments for every ply (every environment of
    every configuration is replayed in test_gpu_full_parity.py), with the action accounting and the whole-batch
    properties checked here."""
    from gpu_common import Pair
    cfg = workloads.CONFIGS[ci]
    n_sample = {0: None, 1: 96, 2: 160, 3: 48, 4: 40}[ci]
    ids = None if n_sample is None else sampled_ids(cfg.batch, n_sample, ci)
    p = Pair(cfg.batch, cfg.board_size, seed=cfg.seed, auto_reset=cfg.auto_reset, ids=ids)
    start = workloads.start_times(cfg)
    T = cfg.warmup_max + cfg.steps
    p.rollout(cfg.seed, 0, T, start_t=start, every=1, state_every=100, fused=(ci >= 3))
    nb = p.orc.B
    assert p.n_compared == nb * T
    assert p.n_actions == (nb * T if start is None else int((T - start[ids]).sum()))
    print(f"config {ci}: {cfg.batch} envs on the GPU, {nb} replayed by the oracle, {T} launches, {p.n_actions} plies compared")
    # whole-batch properties that hold at any size
    g = p.env.export_state()
    P = cfg.board_size ** 2
    mask = p.mask[:, :P + 1]
    assert bool((mask[:, P] == 1).all())
    assert bool(((mask[:, :P] == 1) & (g["board"] != 0)).sum() == 0)
    obs = p.obs[:, : P * 17].view(cfg.batch, P, 17)
    assert bool(((obs[:, :, 0] + obs[:, :, 1]) == (g["board"] != 0)).all())
    assert bool((obs.max() <= 1))
    if not cfg.auto_reset:
        assert bool((g["terminated"] == 1).all())


def test_outputs_beyond_four_gibibytes():
    """720001 games of 19x19: the observation tensor is 4.42 GB, so the byte offsets of the last 20000 games do not fit
    32 bits; the batch is not a multiple of the boards of a wavefront or of a block.  The oracle replays the first games,
    the games on both sides of the 4 GiB offset and the last ones, every tenth ply of 150."""
    from gpu_common import Pair
    B, N, seed, T = 720001, 19, 11, 150
    cross = (1 << 32) // (N * N * 17)      # the game whose observation straddles the 4 GiB offset
    ids = np.concatenate([np.arange(0, 384), np.arange(cross - 192, cross + 192), np.arange(B - 384, B)]).astype(np.int32)
    p = Pair(B, N, seed=seed, auto_reset=True, ids=ids)
    assert p.obs.numel() > (1 << 32)
    p.rollout(seed, 0, T, every=10, state_every=50, fused=True)
    assert p.n_actions == len(ids) * T
    g = p.env.export_state()
    P = N * N
    assert bool((p.mask[:, P] == 1).all())
    assert bool(((p.mask[:, :P] == 1) & (g["board"] != 0)).sum() == 0)
    obs = p.obs.view(B, P, 17)
    assert bool(((obs[:, :, 0] + obs[:, :, 1]) == (g["board"] != 0)).all())
    stones = int((g["board"] != 0).sum())
    assert stones > 60 * B                 # boards have filled up (about 100 stones after 150 plies)
    del g, obs
    # the rollout kernel on the same games, two output slices (the second one starts 4.4 GB after the first)
    env, orc, sel = p.env, p.orc, p.sel
    acts = torch.empty((2, B), dtype=torch.int32, device="cuda")
    rew = torch.empty((2, B, 2), dtype=torch.float32, device="cuda")
    term = torch.empty((2, B), dtype=torch.uint8, device="cuda")
    mask = torch.empty((2, B, P + 1), dtype=torch.uint8, device="cuda")
    obs2 = torch.empty((2, B, P * 17), dtype=torch.uint8, device="cuda")
    env.rollout(6, seed, T, slices=2, actions=acts, rewards=rew, terminated=term, mask=mask, obs=obs2)
    for i in range(6):
        a = orc.random_actions(seed, T + i)
        orc.step(a)
        if i >= 4:                         # the last two plies are still in the slices (ply i -> slice i % 2)
            k = i & 1
            assert (acts[k].index_select(0, sel).cpu().numpy() == a).all(), i
            assert (mask[k].index_select(0, sel).cpu().numpy() == orc.legal_mask()).all(), i
            assert (obs2[k].index_select(0, sel).cpu().numpy().reshape(-1, N, N, 17) == orc.observe()).all(), i
            assert (rew[k].index_select(0, sel).cpu().numpy() == orc.rewards()).all(), i
            assert (term[k].index_select(0, sel).cpu().numpy() == orc.terminated()).all(), i
    del p, env, acts, rew, term, mask, obs2
    torch.cuda.empty_cache()


@pytest.mark.parametrize("N,B,T,slices,auto_reset", [(9, 100, 200, 200, True), (19, 50, 300, 300, True), (19, 64, 120, 1, False), (9, 13, 90, 7, True)])
def test_rollout_kernel_equals_stepwise_play(N, B, T, slices, auto_reset):
    """One launch of `T` plies (state kept in registers) against the oracle stepping ply by ply: every slice of
    the recorded trajectory and the final state."""
    import paper_2303_17503_amd as pg
    seed = N * 1000 + B
    env = pg.GoEnv(B, N, seed=seed, auto_reset=auto_reset)
    orc = oracle.GoOracle(B, N, seed=seed, auto_reset=auto_reset)
    start = (np.arange(B) % 5 * 3).astype(np.int32)
    S, P = slices, N * N
    acts = torch.full((S, B), -9, dtype=torch.int32, device="cuda")
    rew = torch.full((S, B, 2), 7.0, dtype=torch.float32, device="cuda")
    term = torch.full((S, B), 9, dtype=torch.uint8, device="cuda")
    mask = torch.full((S, B, P + 1), 9, dtype=torch.uint8, device="cuda")
    obs = torch.full((S, B, P * 17), 9, dtype=torch.uint8, device="cuda")
    # two launches back to back: the second continues from the stored state
    T1 = T // 3
    env.rollout(T1, seed, 0, start_t=torch.as_tensor(start, device="cuda"), slices=S, actions=acts, rewards=rew, terminated=term, mask=mask, obs=obs)
    first = [x.cpu().numpy().copy() for x in (acts, rew, term, mask, obs)]
    env.rollout(T - T1, seed, T1, start_t=torch.as_tensor(start, device="cuda"), slices=S, actions=acts, rewards=rew, terminated=term, mask=mask, obs=obs)
    second = [x.cpu().numpy() for x in (acts, rew, term, mask, obs)]
    for t in range(T):
        a = orc.random_actions(seed, t, start)
        orc.step(a)
        i = t % S if t < T1 else (t - T1) % S
        # a slice can be checked if no later ply of the same launch overwrote it
        src = first if t < T1 else second
        n_launch = T1 if t < T1 else T - T1
        base = 0 if t < T1 else T1
        if (t - base) + S < n_launch:
            continue
        g_a, g_r, g_t, g_m, g_o = (x[i] for x in src)
        assert (g_a == a).all(), f"actions t={t}"
        assert (g_m == orc.legal_mask()).all(), f"mask t={t}"
        assert (g_o.reshape(B, N, N, 17) == orc.observe()).all(), f"obs t={t}"
        waiting = a < 0
        assert (g_r[~waiting] == orc.rewards()[~waiting]).all() and (g_r[waiting] == 0).all(), f"rewards t={t}"
        assert (g_t[~waiting] == orc.terminated()[~waiting]).all() and (g_t[waiting] == 0).all(), f"terminated t={t}"
    g, c = env.export_state(), orc.export_state()
    for name in ("board", "history", "ko", "to_play", "steps", "passes", "terminated", "black_player", "episode"):
        assert (g[name].cpu().numpy().astype(np.int64) == getattr(c, name).astype(np.int64)).all(), name
    assert (env.legal_mask().cpu().numpy() == orc.legal_mask()).all()
    # and ordinary stepping continues from there
    a = env.random_actions(seed, T)
    assert (a.cpu().numpy() == orc.random_actions(seed, T)).all()


@pytest.mark.parametrize("N,B,komi_x2,max_steps", [(9, 1, 0, 40), (9, 7, 13, 0), (19, 2, -3, 100), (9, 65, 14, 161)])
def test_options_komi_and_ply_cap(N, B, komi_x2, max_steps):
    """Non-default komi (even: draws possible; negative) and ply caps, tiny and ragged batches."""
    from gpu_common import Pair
    p = Pair(B, N, seed=17, auto_reset=True, komi_x2=komi_x2, max_steps=max_steps)
    T = 3 * (max_steps or 2 * N * N) + 5
    p.rollout(17, 0, T, every=1, state_every=20)
    assert p.orc.export_state().episode.min() >= 2


def test_mask_only_and_obs_only_bindings():
    from gpu_common import Pair
    import paper_2303_17503_amd as pg
    B, N = 20, 9
    p = Pair(B, N, seed=9, auto_reset=True, bind=False)
    mask, obs = p.env.new_mask(), p.env.new_obs()
    for t in range(60):
        p.env.bind_outputs(mask if t % 2 == 0 else None, obs if t % 3 == 0 else None, None, None)
        a = p.env.random_actions(9, t)
        a_c = p.orc.random_actions(9, t)
        assert (a.cpu().numpy() == a_c).all()
        p.step(a, a_c)
        if t % 2 == 0:
            assert (mask.cpu().numpy() == p.orc.legal_mask()).all()
        if t % 3 == 0:
            assert (obs.cpu().numpy().reshape(B, N, N, 17) == p.orc.observe()).all()
        assert (p.env.rewards().cpu().numpy() == p.orc.rewards()).all()
        assert (p.env.terminated().cpu().numpy() == p.orc.terminated()).all()
    p.env.bind_outputs(None, None, None, None)


def test_import_with_ko_and_finished_games():
    """Positions with a live ko ban, and games already over, survive import: the ban is honoured and the
    finished games stay frozen."""
    from gpu_common import Pair
    N, B = 9, len(pos.SCRIPTS)
    src = oracle.GoOracle(B, N, seed=5)
    names = sorted(pos.SCRIPTS)
    T = max(len(pos.SCRIPTS[n]["moves"]) for n in names)
    for t in range(T):
        a = np.array([pos.idx(pos.SCRIPTS[n]["moves"][t]) if t < len(pos.SCRIPTS[n]["moves"]) else -1 for n in names], np.int32)
        src.step(a)
    st = src.export_state()
    assert (st.ko >= 0).sum() >= 3
    st.terminated[::4] = 1                     # every fourth game is declared over
    p = Pair(B, N, seed=5, auto_reset=False)
    p.orc.import_state(st)
    dev = {k: torch.as_tensor(getattr(st, k), device="cuda") for k in st.__slots__}
    dev["episode"] = dev["episode"].to(torch.int32)
    p.env.import_state(dev)
    p.compare("after import")
    p.rollout(6, 50, 90, every=1, state_every=10)
    after = p.env.export_state()
    assert (after["board"].cpu().numpy()[::4] == st.board[::4]).all()


def test_rollout_single_slice_with_staggered_start_at_full_batch():
    """The rollout kernel in the launch shape the benchmark uses (16384 games, one slice), checked on a seeded
    sample of environments at the end of every launch."""
    import paper_2303_17503_amd as pg
    B, N, seed, P = 16384, 19, 3, 361
    ids = np.array(sorted({0, 1, 2, 3, 5000, 5001, 16381, 16382, 16383} | set(np.random.default_rng(1).choice(B, 24, replace=False).tolist())), np.int32)
    env = pg.GoEnv(B, N, seed=seed, auto_reset=True)
    orc = oracle.GoOracle(len(ids), N, seed=seed, auto_reset=True, env_ids=ids)
    start = (np.arange(B) % 7).astype(np.int32)
    sel = torch.as_tensor(ids.astype(np.int64), device="cuda")
    acts = torch.empty((1, B), dtype=torch.int32, device="cuda")
    rew = torch.empty((1, B, 2), dtype=torch.float32, device="cuda")
    term = torch.empty((1, B), dtype=torch.uint8, device="cuda")
    mask = torch.empty((1, B, P + 1), dtype=torch.uint8, device="cuda")
    obs = torch.empty((1, B, P * 17), dtype=torch.uint8, device="cuda")
    t = 0
    for L in (1, 2, 50, 50, 97, 400):
        env.rollout(L, seed, t, start_t=torch.as_tensor(start, device="cuda"), slices=1, actions=acts, rewards=rew, terminated=term, mask=mask, obs=obs)
        for i in range(L):
            a = orc.random_actions(seed, t + i, start[ids])
            orc.step(a)
        t += L
        assert (acts[0].index_select(0, sel).cpu().numpy() == a).all()
        assert (mask[0].index_select(0, sel).cpu().numpy() == orc.legal_mask()).all(), t
        assert (obs[0].index_select(0, sel).cpu().numpy().reshape(-1, N, N, 17) == orc.observe()).all(), t
        assert (rew[0].index_select(0, sel).cpu().numpy() == orc.rewards()).all(), t
        assert (term[0].index_select(0, sel).cpu().numpy() == orc.terminated()).all(), t
    g = env.export_state()
    assert (g["board"].index_select(0, sel).cpu().numpy() == orc.export_state().board).all()
    assert int(g["episode"].max()) >= 1


@pytest.mark.parametrize("N,pool,auto_reset", [(9, 40, False), (19, 25, True)])
def test_slot_step_and_copy_for_tree_search(N, pool, auto_reset):
    """step_slots / copy_slots against the oracle: a pool of states, random (src -> dst) expansions with random
    legal or illegal actions, like a search expanding children from stored nodes."""
    import paper_2303_17503_amd as pg
    from gpu_common import to_np
    rng = np.random.default_rng(N)
    seed, P = 31, N * N
    env = pg.GoEnv(pool, N, seed=seed, auto_reset=auto_reset)
    orc = oracle.GoOracle(pool, N, seed=seed, auto_reset=auto_reset)
    for t in range(30):                      # some history in every slot
        a = orc.random_actions(seed, t)
        env.step(torch.as_tensor(a, device="cuda")); orc.step(a)
    fields = ("board", "history", "ko", "to_play", "steps", "passes", "terminated", "black_player", "episode")

    def check_pool(tag):
        g, c = env.export_state(), orc.export_state()
        for name in fields:
            assert (to_np(g[name]).astype(np.int64) == getattr(c, name).astype(np.int64)).all(), (tag, name)
        assert (to_np(env.legal_mask()) == orc.legal_mask()).all(), tag

    check_pool("start")
    for it in range(40):
        n = int(rng.integers(1, pool // 2))
        perm = rng.permutation(pool)
        dst = perm[:n].astype(np.int32)                       # distinct destinations
        free_src = perm[n:]                                   # sources that are nobody's destination ...
        src = rng.choice(free_src, n).astype(np.int32)
        same = rng.random(n) < 0.3                            # ... or the entry's own destination (in-place step)
        src = np.where(same, dst, src).astype(np.int32)
        st = orc.export_state()
        tmp = oracle.GoOracle(n, N, seed=seed, auto_reset=auto_reset, env_ids=dst)
        sub = oracle.State(n, P)
        for name in fields:
            getattr(sub, name)[...] = getattr(st, name)[src]
        tmp.import_state(sub)
        m = tmp.legal_mask()
        act = np.array([rng.choice(np.flatnonzero(m[i])) for i in range(n)], np.int32)
        kind = rng.integers(0, 10, n)
        act = np.where(kind == 0, rng.integers(0, P, n), act)  # maybe illegal
        act = np.where(kind == 1, -1, act).astype(np.int32)    # plain copy
        tmp.step(act)
        mask = torch.full((n, P + 1), 9, dtype=torch.uint8, device="cuda")
        obs = torch.full((n, P * 17), 9, dtype=torch.uint8, device="cuda")
        rew = torch.full((n, 2), 9.0, dtype=torch.float32, device="cuda")
        term = torch.full((n,), 9, dtype=torch.uint8, device="cuda")
        env.step_slots(torch.as_tensor(src, device="cuda"), torch.as_tensor(act, device="cuda"), torch.as_tensor(dst, device="cuda"),
                       mask=mask, obs=obs, rewards=rew, terminated=term)
        assert (to_np(mask) == tmp.legal_mask()).all(), it
        assert (to_np(obs).reshape(n, N, N, 17) == tmp.observe()).all(), it
        copied = act == -1
        assert (to_np(rew)[~copied] == tmp.rewards()[~copied]).all() and (to_np(rew)[copied] == 0).all(), it
        assert (to_np(term)[~copied] == tmp.terminated()[~copied]).all(), it
        assert (to_np(term)[copied] == sub.terminated[copied]).all(), it
        after = tmp.export_state()
        for name in fields:
            getattr(st, name)[dst] = getattr(after, name)
        orc.import_state(st)
        check_pool(f"iteration {it}")
    # copy_slots, and an out-of-range entry
    src = np.array([0, 1, 2], np.int32); dst = np.array([5, 6, 7], np.int32)
    env.copy_slots(torch.as_tensor(src, device="cuda"), torch.as_tensor(dst, device="cuda"))
    st = orc.export_state()
    for name in fields:
        getattr(st, name)[dst] = getattr(st, name)[src]
    orc.import_state(st)
    check_pool("copy")
    term = torch.zeros(2, dtype=torch.uint8, device="cuda")
    env.step_slots(torch.as_tensor(np.array([3, pool + 5], np.int32), device="cuda"), torch.as_tensor(np.array([-1, 0], np.int32), device="cuda"),
                   torch.as_tensor(np.array([3, 4], np.int32), device="cuda"), terminated=term)
    assert to_np(term)[1] == 255
    check_pool("bad slot ignored")


@pytest.mark.parametrize("N,B", [(19, 100), (9, 500)])
def test_switching_output_buffers_and_the_combined_getter(N, B):
    """pgxgo_set_output_buffers: a different slice every ply records the trajectory, no emission or copy at the switch;
    pgxgo_emit: mask and observation of the current state in one launch."""
    from gpu_common import Pair, to_np
    seed, S = 21, 5
    p = Pair(B, N, seed=seed, auto_reset=True)
    masks = [torch.full_like(p.mask, 7) for _ in range(S)]
    obss = [torch.full_like(p.obs, 7) for _ in range(S)]
    rews = [torch.full_like(p.rew, 7.0) for _ in range(S)]
    terms = [torch.full_like(p.term, 7) for _ in range(S)]
    p.env.set_output_buffers(masks[0], obss[0], rews[0], terms[0])
    assert (to_np(masks[0]) == 7).all() and (to_np(rews[0]) == 7).all()          # nothing was written at the switch
    a = p.env.random_actions(seed, 0)
    for t in range(40):
        i = t % S
        p.env.set_output_buffers(masks[i], obss[i], rews[i], terms[i])
        a_c = p.orc.random_actions(seed, t)
        assert (to_np(a) == a_c).all()
        a = p.env.step_sample(a, seed, t + 1)
        p.orc.step(a_c)
        assert (to_np(masks[i]) == p.orc.legal_mask()).all() and (to_np(obss[i]).reshape(B, N, N, 17) == p.orc.observe()).all(), t
        assert to_np(rews[i]).tobytes() == p.orc.rewards().tobytes() and (to_np(terms[i]) == p.orc.terminated()).all(), t
    m2, o2 = torch.full_like(p.mask, 9), torch.full_like(p.obs, 9)
    p.env.emit(m2, o2)
    assert (to_np(m2) == p.orc.legal_mask()).all() and (to_np(o2).reshape(B, N, N, 17) == p.orc.observe()).all()
    m3 = torch.full_like(p.mask, 9)
    p.env.emit(mask=m3)
    assert (to_np(m3) == p.orc.legal_mask()).all()
    p.env.set_output_buffers()                                                   # back to the internal rewards / terminated arrays
    a_c = p.orc.random_actions(seed, 40)
    p.env.step(torch.as_tensor(a_c, device="cuda")); p.orc.step(a_c)
    assert to_np(p.env.rewards()).tobytes() == p.orc.rewards().tobytes() and (to_np(p.env.terminated()) == p.orc.terminated()).all()
    assert (to_np(p.env.legal_mask()) == p.orc.legal_mask()).all()


@pytest.mark.parametrize("line_padded", [False, True])
def test_store_kinds_of_a_mid_size_batch(line_padded):
    """The kind of the output stores follows the bytes a launch writes and whether it overwrites the previous launch's
    buffers: 19x19 x 6001 games (39 MB per ply) in place, then rotating over three sets of buffers, then in place
    again; sampled games against the oracle every ply, the whole batch against the getters (which use ordinary stores)."""
    from gpu_common import to_np
    import paper_2303_17503_amd as pg
    N, B, seed = 19, 6001, 12
    P = N * N
    ids = np.unique(np.concatenate([np.arange(0, 12), np.arange(2990, 3010), np.arange(B - 9, B), np.random.default_rng(1).integers(0, B, 40)])).astype(np.int32)
    env = pg.GoEnv(B, N, seed=seed, auto_reset=True, line_padded=line_padded)
    orc = oracle.GoOracle(len(ids), N, seed=seed, auto_reset=True, env_ids=ids)
    sel = torch.as_tensor(ids.astype(np.int64), device="cuda")
    sets = [(env.new_mask().fill_(7), env.new_obs().fill_(7)) for _ in range(3)]
    rew, term = torch.zeros((B, 2), device="cuda"), torch.zeros(B, dtype=torch.uint8, device="cuda")
    env.bind_outputs(sets[0][0], sets[0][1], rew, term)
    a = env.random_actions(seed, 0)
    for t in range(45):
        k = 0 if (t < 15 or t >= 36) else t % 3          # in place, rotating, in place
        env.set_output_buffers(sets[k][0], sets[k][1], rew, term)
        a_c = orc.random_actions(seed, t)
        assert (to_np(a.index_select(0, sel)) == a_c).all(), t
        a = env.step_sample(a, seed, t + 1)
        orc.step(a_c)
        m, o = sets[k]
        assert (to_np(m.index_select(0, sel))[:, :P + 1] == orc.legal_mask()).all(), t
        assert (to_np(env.obs_view(o).index_select(0, sel)) == orc.observe()).all(), t
        assert to_np(rew.index_select(0, sel)).tobytes() == orc.rewards().tobytes(), t
        if t % 7 == 0 or t >= 40:
            assert torch.equal(env.legal_mask()[:, :P + 1], m[:, :P + 1]) and torch.equal(env.obs_view(env.observe()), env.obs_view(o)), t
            if line_padded:
                assert (m[:, P + 1:] == 0).all() and (o[:, P * 17:] == 0).all()


@pytest.mark.parametrize("N,wb", [(19, 1), (19, 2), (19, 3), (9, 1), (9, 2), (9, 3), (9, 4), (9, 5), (9, 6)])
def test_every_launch_shape(N, wb):
    """The number of boards a wavefront holds is a launch-shape choice: every value gives the oracle's results
    (ragged last wavefront, step with and without the fused sampler, the rollout kernel, the superko kernel)."""
    import paper_2303_17503_amd as pg
    from gpu_common import Pair, to_np
    B, seed = 6 * wb + (wb + 1) // 2 + 11, 40 + wb
    p = Pair(B, N, seed=seed, auto_reset=True)
    assert p.env.set_boards_per_wavefront(wb) == wb
    p.rollout(seed, 0, 60, fused=False, state_every=10)
    p.rollout(seed, 60, 140, fused=True, state_every=20)
    # rollout kernel: 35 plies in one launch, then compare the state
    p.env.rollout(35, seed, 140)
    for t in range(140, 175):
        p.orc.step(p.orc.random_actions(seed, t))
    g, c = p.env.export_state(), p.orc.export_state()
    assert (to_np(g["board"]) == c.board).all() and (to_np(g["history"]) == c.history).all() and (to_np(g["steps"]) == c.steps).all()
    for mode in (1, "mask"):
        q = Pair(B, N, seed=seed, auto_reset=True, superko=mode)
        q.env.set_boards_per_wavefront(wb)
        q.rollout(seed, 0, 90, fused=True, state_every=30)
        q.env.rollout(20, seed, 90)                            # the rollout kernel carries the key tables in every launch shape
        for t in range(90, 110):
            q.orc.step(q.orc.random_actions(seed, t))
        q.rollout(seed, 110, 130, fused=True, state_every=10)
    with pytest.raises(pg.PgxGoError):
        p.env.set_boards_per_wavefront(7)
    assert p.env.set_boards_per_wavefront(0) == 1            # automatic choice for a batch this small


@pytest.mark.parametrize("N,B", [(19, 1), (19, 2), (9, 1), (9, 7)])
def test_tiny_batches(N, B):
    """A single game (one partly filled wavefront, one block) through every stepping path."""
    from gpu_common import Pair, to_np
    p = Pair(B, N, seed=70 + B, auto_reset=True)
    p.rollout(70 + B, 0, 2 * N * N + 40, fused=True, state_every=25)
    assert to_np(p.env.export_state()["episode"]).min() >= 1
    for mode in (1, "mask"):
        q = Pair(B, N, seed=71, auto_reset=False, superko=mode)
        q.rollout(71, 0, 120, fused=False, state_every=30)
    r = Pair(B, N, seed=72, auto_reset=True, bind=False)
    r.env.rollout(90, 72, 0)
    for t in range(90):
        r.orc.step(r.orc.random_actions(72, t))
    g, c = r.env.export_state(), r.orc.export_state()
    assert (to_np(g["board"]) == c.board).all() and (to_np(g["history"]) == c.history).all() and (to_np(g["ko"]) == c.ko).all()


@pytest.mark.parametrize("ci,plies", [(3, 420), (4, 380)])
def test_whole_batch_properties_every_ply(ci, plies):
    """Facts that hold for every game at any size, checked on the device tensors of the full batch after every ply
    (the oracle replays only a sample of these batches): pass is legal, legal points are empty, an empty point next to
    an empty point is legal unless it is the ko point, observation planes against the exported history, the
    shift-and-swap of the planes from ply to ply, rewards and termination."""
    import paper_2303_17503_amd as pg
    cfg = workloads.CONFIGS[ci]
    B, N, seed = cfg.batch, cfg.board_size, cfg.seed
    P = N * N
    env = pg.GoEnv(B, N, seed=seed, komi_x2=cfg.komi_x2, auto_reset=True)
    mask, obs = env.new_mask(), env.new_obs()
    rew = torch.zeros((B, 2), dtype=torch.float32, device="cuda")
    term = torch.zeros(B, dtype=torch.uint8, device="cuda")
    env.bind_outputs(mask, obs, rew, term)
    start = workloads.start_times(cfg)
    st = None if start is None else torch.as_tensor(start, device="cuda")
    a = env.random_actions(seed, 0, st)
    prev = None
    n_term = 0
    for t in range(plies):
        a = env.step_sample(a, seed, t + 1, st)
        o = obs.view(B, N, N, 17)
        assert bool((mask[:, P] == 1).all()), f"pass legal t={t}"
        if t % 20 == 0 or t == plies - 1:
            g = env.export_state()
            bd = g["board"].view(B, N, N)
            emp = bd == 0
            m = mask[:, :P].view(B, N, N) == 1
            assert bool((m & ~emp).sum() == 0), f"legal points are empty t={t}"
            nb = torch.zeros_like(emp)
            nb[:, 1:, :] |= emp[:, :-1, :]; nb[:, :-1, :] |= emp[:, 1:, :]; nb[:, :, 1:] |= emp[:, :, :-1]; nb[:, :, :-1] |= emp[:, :, 1:]
            ko = torch.zeros((B, P + 1), dtype=torch.bool, device="cuda")
            ko[torch.arange(B, device="cuda"), torch.where(g["ko"] >= 0, g["ko"], P).long()] = True
            must = emp & nb & ~ko[:, :P].view(B, N, N)
            assert bool((must & ~m).sum() == 0), f"an empty point next to an empty point is legal t={t}"
            mover = g["to_play"].view(B, 1, 1, 1)
            hist = g["history"].view(B, 8, N, N).permute(0, 2, 3, 1)                      # [B][N][N][8]
            assert bool((o[..., 0:16:2] == (hist == mover)).all()) and bool((o[..., 1:16:2] == (hist == -mover)).all()), f"planes vs history t={t}"
            assert bool((o[..., 16] == (g["to_play"] == 1).view(B, 1, 1)).all()), f"colour plane t={t}"
            assert bool((hist[..., 0] == bd).all()), f"history[0] is the position t={t}"
        # rewards and termination of this ply
        fin = term == 1
        n_term += int(fin.sum())
        assert bool((rew.sum(1) == 0).all()) and bool((rew[fin].abs() == 1).all()) and bool((rew[~fin] == 0).all()), f"rewards t={t}"
        moved = (a >= -1) if st is None else (st <= t)          # games already past their start time took part in this ply
        if prev is not None:
            keep = ~fin & moved & prev_moved                     # no reset in between: the planes shift by one ply and swap sides
            assert bool((o[keep][..., 2:16:2] == prev[keep][..., 1:14:2]).all()) and bool((o[keep][..., 3:16:2] == prev[keep][..., 0:14:2]).all()), f"shift t={t}"
        prev = o.clone()
        prev_moved = moved if isinstance(moved, torch.Tensor) else torch.ones(B, dtype=torch.bool, device="cuda")
    assert n_term > 0 or ci == 4


def test_c_abi_with_default_options():
    """The boundary used directly (ctypes, no binding class): NULL options select komi 7.5, cap 2*N*N, no auto-reset,
    tight pitches and the default stream."""
    import ctypes as C
    import paper_2303_17503_amd as pg
    L = pg.lib()
    B, N = 5, 9
    nbytes = L.pgxgo_state_bytes(B, N)
    state = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    h = C.c_void_p()
    assert L.pgxgo_init(C.byref(h), B, N, 123, None, C.c_void_p(state.data_ptr()), nbytes) == 0
    try:
        mask = torch.empty((B, 82), dtype=torch.uint8, device="cuda")
        rew = torch.empty((B, 2), dtype=torch.float32, device="cuda")
        term = torch.empty(B, dtype=torch.uint8, device="cuda")
        cur = torch.empty(B, dtype=torch.uint8, device="cuda")
        acts = torch.full((B,), 81, dtype=torch.int32, device="cuda")           # everybody passes
        p = lambda t: C.c_void_p(t.data_ptr())
        assert L.pgxgo_legal_mask(h, p(mask)) == 0 and L.pgxgo_current_player(h, p(cur)) == 0
        assert L.pgxgo_sync(h) == 0
        assert bool((mask == 1).all())
        black = cur.clone()                                                        # Black moves first: the player to move now holds Black
        assert L.pgxgo_step(h, p(acts)) == 0 and L.pgxgo_step(h, p(acts)) == 0
        assert L.pgxgo_rewards(h, p(rew)) == 0 and L.pgxgo_terminated(h, p(term)) == 0 and L.pgxgo_sync(h) == 0
        assert bool((term == 1).all())                                             # two passes end the game; no auto-reset
        r = rew.cpu().numpy(); bp = black.cpu().numpy()
        for b in range(B):                                                         # empty board: White wins by the komi
            assert r[b, bp[b]] == -1 and r[b, 1 - bp[b]] == 1
        assert L.pgxgo_step(h, p(acts)) == 0 and L.pgxgo_rewards(h, p(rew)) == 0 and L.pgxgo_sync(h) == 0
        assert bool((rew == 0).all())                                              # frozen afterwards
    finally:
        assert L.pgxgo_destroy(h) == 0
