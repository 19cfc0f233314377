"""Pins of the CPU oracle against hand-built positions, the paper's printed shapes and closed forms."""
import os

import numpy as np
import pytest

import oracle
import positions as pos

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def facts():
    out = {}
    with open(os.path.join(GOLDEN, "paper_go_facts.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out[line[0]] = [int(x) for x in line[1:]]
    return out


def run_script(moves, N=9, **kw):
    o = oracle.GoOracle(1, N, **kw)
    for m in moves:
        assert o.terminated()[0] == 0
        a = N * N if m == pos.P else m[0] * N + m[1]
        assert o.legal_mask()[0, a] == 1, f"script move {m} must be legal"
        o.step([a])
    return o


def test_shapes_match_paper():
    F = facts()
    for N in (9, 19):
        o = oracle.GoOracle(3, N)
        assert list(o.observe().shape[1:]) == F[f"go_{N}x{N}_obs_shape"]
        assert o.legal_mask().shape[1] == F[f"go_{N}x{N}_num_actions"][0]
        assert o.observe().shape[-1] == F["history_plies"][0] * F["planes_per_ply"][0] + F["colour_planes"][0]
        assert o.rewards().shape == (3, F["num_players"][0])
        assert o.observe().dtype == np.uint8 and o.legal_mask().dtype == np.uint8
    o = oracle.GoOracle(1024, 19)
    assert list(o.observe().shape) == F["batch_obs_shape_example"]
    assert list(o.legal_mask().shape) == F["batch_mask_shape_example"]
    assert o.current_player().shape == (1024,) and set(np.unique(o.current_player())) <= {0, 1}


@pytest.mark.parametrize("name", sorted(pos.SCRIPTS))
def test_hand_built_position(name):
    sc = pos.SCRIPTS[name]
    o = run_script(sc["moves"])
    s = o.export_state()
    assert s.board[0].tolist() == sc["board"], name
    ko = -1 if sc["ko"] == -1 else sc["ko"][0] * 9 + sc["ko"][1]
    assert s.ko[0] == ko
    assert s.to_play[0] == sc["to_play"]
    assert s.steps[0] == len(sc["moves"])
    assert o.terminated()[0] == 0 and o.rewards()[0].tolist() == [0.0, 0.0]
    m = o.legal_mask()[0]
    for rc in sc.get("illegal_next", []):
        assert m[rc[0] * 9 + rc[1]] == 0, (name, rc)
    for rc in sc.get("legal_next", []):
        assert m[rc[0] * 9 + rc[1]] == 1, (name, rc)
    assert m[81] == 1                                # pass is the last action and always legal
    occupied = np.array(sc["board"]) != 0
    assert not m[:81][occupied].any()


def test_empty_board_closed_forms():
    for N in (2, 3, 5, 9, 19):
        o = oracle.GoOracle(1, N)
        m = o.legal_mask()[0]
        assert m.sum() == N * N + 1
        ob = o.observe()[0]
        assert ob[..., :16].sum() == 0 and (ob[..., 16] == 1).all()   # black to move on an empty board
        o.step([0])
        assert o.legal_mask()[0].sum() == N * N                        # every other point + pass
        ob = o.observe()[0]
        assert (ob[..., 16] == 0).all()                                # white to move
        assert ob[0, 0, 1] == 1 and ob[..., 1].sum() == 1 and ob[..., 0].sum() == 0   # opponent plane of the newest position
        assert ob[..., 2:16].sum() == 0


@pytest.mark.parametrize("black_seat_seed", range(6))
def test_pass_pass_and_lone_stone(black_seat_seed):
    N = 9
    o = oracle.GoOracle(1, N, seed=black_seat_seed)
    bp = int(o.export_state().black_player[0])
    assert o.current_player()[0] == bp                 # black moves first
    o.step([81])
    assert o.current_player()[0] == 1 - bp
    assert o.terminated()[0] == 0
    o.step([81])
    assert o.terminated()[0] == 1
    r = o.rewards()[0]
    assert r[bp] == -1.0 and r[1 - bp] == 1.0          # areas 0:0, komi decides for White
    # a lone black stone owns the whole board
    o = oracle.GoOracle(1, N, seed=black_seat_seed)
    o.step([40]); o.step([81]); o.step([81])
    assert o.terminated()[0] == 1
    r = o.rewards()[0]
    assert r[bp] == 1.0 and r[1 - bp] == -1.0
    # frozen afterwards (no auto-reset): zero rewards, flag stays, state unchanged
    before = o.export_state()
    o.step([3])
    assert o.rewards()[0].tolist() == [0.0, 0.0] and o.terminated()[0] == 1
    after = o.export_state()
    assert (before.board == after.board).all() and before.steps[0] == after.steps[0]


def test_seat_assignment_is_hash_bit_and_changes_by_episode():
    B = 64
    o = oracle.GoOracle(B, 9, seed=5, auto_reset=True)
    s = o.export_state()
    assert s.black_player.tolist() == [oracle.hash4(5, 1, e, 0) & 1 for e in range(B)]
    assert 10 < s.black_player.sum() < 54
    o.step(np.full(B, 81)); o.step(np.full(B, 81))     # everyone ends by two passes and is reset
    assert o.terminated().all()
    s = o.export_state()
    assert (s.episode == 1).all() and (s.terminated == 0).all() and (s.steps == 0).all()
    assert s.black_player.tolist() == [oracle.hash4(5, 1, e, 1) & 1 for e in range(B)]
    assert o.legal_mask().sum() == B * 82 and o.observe()[..., :16].sum() == 0


def test_draw_needs_even_komi():
    # 2x2 board, both pass: areas equal; komi_x2 = 0 gives a draw, komi_x2 = 1 a white win
    for komi_x2, want in ((0, 0.0), (1, -1.0), (-1, 1.0)):
        o = oracle.GoOracle(1, 2, komi_x2=komi_x2)
        bp = int(o.export_state().black_player[0])
        o.step([4]); o.step([4])
        assert o.rewards()[0, bp] == want and o.rewards()[0, 1 - bp] == -want


def test_illegal_action_ends_game_offender_loses():
    for bad in (0, 100, -7):                           # occupied point / out of range
        o = oracle.GoOracle(1, 9, seed=1)
        bp = int(o.export_state().black_player[0])
        o.step([0])                                    # black
        before = o.export_state()
        o.step([bad])                                  # white offends
        assert o.terminated()[0] == 1 and o.illegal_count()[0] == 1
        assert o.rewards()[0, 1 - bp] == -1.0 and o.rewards()[0, bp] == 1.0
        after = o.export_state()
        assert (before.board == after.board).all() and after.steps[0] == 1 and after.to_play[0] == -1


def test_skip_action_changes_nothing():
    o = oracle.GoOracle(2, 9, seed=2)
    o.step([10, 11])
    before, m0, ob0 = o.export_state(), o.legal_mask(), o.observe()
    o.step([-1, 12])
    after = o.export_state()
    assert (after.board[0] == before.board[0]).all() and after.steps[0] == 1 and after.steps[1] == 2
    assert (o.legal_mask()[0] == m0[0]).all() and (o.observe()[0] == ob0[0]).all()


def test_step_cap_terminates_and_scores():
    N, B = 9, 32
    o = oracle.GoOracle(B, N, seed=0)
    ended_at = np.full(B, -1)
    for t in range(2 * N * N):
        o.step(o.random_actions(0, t))
        term = o.terminated()
        ended_at[(ended_at < 0) & (term == 1)] = t + 1
    s = o.export_state()
    assert (s.terminated == 1).all() and (ended_at > 0).all()
    assert (s.steps <= 2 * N * N).all() and (s.steps == ended_at).all()
    capped = s.steps == 2 * N * N
    assert capped.any()


def test_history_planes_follow_the_last_eight_positions():
    o = run_script(pos.SCRIPTS["capture_four_chains"]["moves"])
    s = o.export_state()
    ob = o.observe()[0].reshape(81, 17)
    tp = int(s.to_play[0])
    for i in range(8):
        assert (ob[:, 2 * i] == (s.history[0, i] == tp)).all()
        assert (ob[:, 2 * i + 1] == (s.history[0, i] == -tp)).all()
    assert (s.history[0, 0] == s.board[0]).all()
    # position one ply ago still holds the four white stones that the last move removed
    assert (s.history[0, 1] == -1).sum() == 4 and (s.history[0, 0] == -1).sum() == 0
    # a pass repeats the position: plies 1 and 2 ago are identical (White passed at ply 16)
    assert (s.history[0, 1] == s.history[0, 2]).all()
