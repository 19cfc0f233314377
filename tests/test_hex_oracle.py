"""Pins of the CPU Hex oracle (Appendix C "Hex"): the paper's printed facts, hand-built paths, the no-draw
theorem, an independent Python implementation, symmetries.  No GPU."""
import itertools
import os

import numpy as np
import pytest

from oracle import hex as hx
from hex_pyref import RefHex

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def facts():
    out = {}
    with open(os.path.join(GOLDEN, "paper_hex_facts.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out[line[0]] = [int(x) for x in line[1:]]
    return out


def parse(rows):
    """'X' black, 'O' white, '.' empty; row 0 first.  Picture rows are meant to be read with row r drawn
    r half-cells further right than row 0 (the usual rhombus), so that (r, c) touches (r+1, c-1) and (r+1, c)."""
    return np.array([[{'X': 1, 'O': -1, '.': 0}[ch] for ch in row] for row in rows], np.int8)


def test_shapes_match_paper():
    F = facts()
    N = F["board_size"][0]
    o = hx.HexOracle(3, N)
    assert list(o.observe().shape[1:]) == F["hex_obs_shape"]
    assert o.legal_mask().shape[1] == F["hex_num_actions"][0]
    assert o.observe().shape[-1] == F["stone_planes"][0] + F["colour_planes"][0] + F["swap_planes"][0]
    assert o.rewards().shape == (3, F["num_players"][0])
    assert o.A - 1 == F["swap_action"][0]


def test_initial_state():
    o = hx.HexOracle(5, 11, seed=9)
    m, ob = o.legal_mask(), o.observe()
    assert (m[:, :121] == 1).all() and (m[:, 121] == 0).all()      # swap is not on offer on the first turn
    assert (ob[..., 0] == 0).all() and (ob[..., 1] == 0).all()
    assert (ob[..., 2] == 1).all() and (ob[..., 3] == 0).all()     # Black to move, no swap
    assert (o.terminated() == 0).all() and (o.rewards() == 0).all()
    s = o.export_state()
    assert (o.current_player() == s.black_player).all()


def test_swap_only_on_second_turn():
    F = facts()
    N, SW = 11, F["swap_action"][0]
    o = hx.HexOracle(1, N)
    o.step([2 * N + 5])                                            # Black at (2, 5)
    assert F["swap_turn"][0] == 2
    m, ob = o.legal_mask()[0], o.observe()[0]
    assert m[SW] == 1 and (ob[..., 3] == 1).all() and (ob[..., 2] == 0).all()
    assert m[2 * N + 5] == 0 and m.sum() == 121                    # 120 empty cells + swap
    assert ob[2, 5, 1] == 1 and ob[..., 1].sum() == 1 and ob[..., 0].sum() == 0
    o.step([SW])
    s = o.export_state()
    want = np.zeros((N, N), np.int8); want[5, 2] = -1              # the stone is now White's, at the mirrored cell
    assert (s.board[0].reshape(N, N) == want).all()
    assert s.to_play[0] == 1 and s.steps[0] == 2 and o.terminated()[0] == 0
    m, ob = o.legal_mask()[0], o.observe()[0]
    assert m[SW] == 0 and (ob[..., 3] == 0).all() and (ob[..., 2] == 1).all()
    assert ob[5, 2, 1] == 1 and ob[..., 0].sum() == 0 and m[5 * N + 2] == 0 and m.sum() == 120
    # a diagonal cell maps to itself
    o = hx.HexOracle(1, N); o.step([4 * N + 4]); o.step([SW])
    assert o.export_state().board[0].reshape(N, N)[4, 4] == -1
    # declining the swap: it is gone on the third turn
    o = hx.HexOracle(1, N); o.step([0]); o.step([1])
    assert o.legal_mask()[0, SW] == 0 and (o.observe()[0][..., 3] == 0).all()


@pytest.mark.parametrize("action,when", [(121, 0), (121, 2), (7, 1), (122, 0), (-5, 0), (1000, 3)])
def test_illegal_actions_end_the_game(action, when):
    N = 11
    o = hx.HexOracle(1, N, seed=4)
    for a in [7, 30, 55, 80][:when]:
        o.step([a])
    before = o.export_state()
    mover = o.current_player()[0]
    o.step([action])
    assert o.terminated()[0] == 1 and o.illegal_count()[0] == 1
    r = o.rewards()[0]
    assert r[mover] == -1 and r[1 - mover] == 1
    after = o.export_state()
    assert (after.board == before.board).all() and after.to_play[0] == before.to_play[0] and after.steps[0] == before.steps[0]
    o.step([0])                                                    # frozen afterwards
    assert (o.rewards() == 0).all() and o.terminated()[0] == 1 and o.illegal_count()[0] == 1


PICTURES = [
    # (rows, black joined, white joined)
    (["X....",
      "X....",
      "X....",
      "X....",
      "X...."], True, False),                                       # straight down a column
    (["....X",
      "...X.",
      "..X..",
      ".X...",
      "X...."], True, False),                                       # (r,c) - (r+1,c-1) touch: the anti-diagonal is a chain
    (["X....",
      ".X...",
      "..X..",
      "...X.",
      "....X"], False, False),                                      # (r,c) - (r+1,c+1) do not touch
    (["OOOOO",
      ".....",
      ".....",
      ".....",
      "....."], False, True),                                       # along a row
    (["....O",
      "...O.",
      "..O..",
      ".O...",
      "O...."], False, True),                                       # the same anti-diagonal serves White too
    ([".X...",
      ".X...",
      "XOOOO",
      "X....",
      "X...."], True, False),                                       # black (1,1)-(2,0) touch; white lacks column 0
    ([".X...",
      ".XOOO",
      "OOX..",
      "..X..",
      "..X.."], False, True),                                       # white (1,2)-(2,1) touch; black (1,1)-(2,2) do not
    (["..X..",
      "..X..",
      "OO.OO",
      "..X..",
      "..X.."], False, False),
    (["..X..",
      "..X..",
      "OOXOO",
      "..X..",
      "..X.."], True, False),
    (["XXXX.",
      "....O",
      "....O",
      "....O",
      "....O"], False, False),                                      # a side alone is not a connection
]


@pytest.mark.parametrize("k", range(len(PICTURES)))
def test_hand_built_paths(k):
    rows, bj, wj = PICTURES[k]
    b = parse(rows)
    assert hx.joined(b, len(rows), 1) == bj
    assert hx.joined(b, len(rows), -1) == wj


def test_shortest_game_and_rewards():
    """Black walks down column 3 while White answers in column 7: the game ends on ply 2N-1 and not before."""
    N = 11
    for seed in range(4):
        o = hx.HexOracle(1, N, seed=seed)
        bp = o.export_state().black_player[0]
        for r in range(N):
            assert o.terminated()[0] == 0
            o.step([r * N + 3])
            if r < N - 1:
                assert o.terminated()[0] == 0 and (o.rewards() == 0).all()
                o.step([r * N + 7])
        assert o.terminated()[0] == 1 and o.export_state().steps[0] == 2 * N - 1
        r = o.rewards()[0]
        assert r[bp] == 1 and r[1 - bp] == -1


def test_white_wins_by_row_with_lean():
    """White's chain steps down-left once ((4,5) -> (5,4)), which only the chosen lean connects."""
    N = 11
    o = hx.HexOracle(1, N, seed=1)
    bp = o.export_state().black_player[0]
    white = [(4, c) for c in range(10, 4, -1)] + [(5, c) for c in range(4, -1, -1)]
    black = [(9, c) for c in range(len(white))]
    for i, w in enumerate(white):
        o.step([black[i][0] * N + black[i][1]])
        assert o.terminated()[0] == 0
        o.step([w[0] * N + w[1]])
    assert o.terminated()[0] == 1
    r = o.rewards()[0]
    assert r[1 - bp] == 1 and r[bp] == -1


def test_no_draw_on_full_boards():
    """Hex theorem: a completely filled board has exactly one winner, whatever the numbers of stones."""
    rng = np.random.default_rng(5)
    for N in range(2, 12):
        for _ in range(300):
            b = rng.choice(np.array([1, -1], np.int8), size=(N, N), p=(lambda q: [q, 1 - q])(rng.uniform(0.3, 0.7)))
            assert hx.joined(b, N, 1) != hx.joined(b, N, -1)


def test_exhaustive_small_boards_against_python():
    for N, depth in ((2, 5), (3, 5)):
        A = N * N + 1
        for seq in itertools.product(range(A), repeat=depth):
            ref = RefHex(N)
            o = hx.HexOracle(1, N)
            for a in seq:
                res = ref.play(a)
                o.step([a])
                s = o.export_state()
                assert s.board[0].reshape(N, N).tolist() == ref.board()
                assert bool(o.terminated()[0]) == ref.over
                if ref.over:
                    bp = s.black_player[0]
                    winner_id = bp if ref.winner == 'B' else 1 - bp
                    r = o.rewards()[0]
                    assert r[winner_id] == 1 and r[1 - winner_id] == -1
                    assert (res == 'illegal') == (o.illegal_count()[0] == 1)
                    break
                assert o.legal_mask()[0].tolist() == [int(ref.legal(x)) for x in range(A)]


def test_random_games_against_python():
    rng = np.random.default_rng(11)
    for N in range(2, 12):
        for g in range(12 if N < 9 else 6):
            ref = RefHex(N)
            o = hx.HexOracle(1, N, seed=g)
            A = N * N + 1
            plies = 0
            while not ref.over:
                m = o.legal_mask()[0]
                assert m.tolist() == [int(ref.legal(x)) for x in range(A)]
                legal = np.flatnonzero(m)
                a = int(A - 1) if (m[A - 1] and rng.random() < 0.5) else int(rng.choice(legal))
                ref.play(a)
                o.step([a])
                plies += 1
                assert o.export_state().board[0].reshape(N, N).tolist() == ref.board()
                assert bool(o.terminated()[0]) == ref.over
            assert plies <= A                                       # every ply but the swap fills a cell
            s = o.export_state()
            bp = s.black_player[0]
            winner_id = bp if ref.winner == 'B' else 1 - bp
            assert o.rewards()[0][winner_id] == 1 and o.rewards()[0][1 - winner_id] == -1
            b = s.board[0]
            col = 1 if ref.winner == 'B' else -1
            assert hx.joined(b, N, col) and not hx.joined(b, N, -col)


def random_rollout(N, seed, B=8, auto_reset=False, plies=None):
    o = hx.HexOracle(B, N, seed=seed, auto_reset=auto_reset)
    trace = []
    for t in range(plies or (N * N + 1)):
        a = o.random_actions(seed, t)
        o.step(a)
        trace.append((a.copy(), o.export_state(), o.legal_mask(), o.observe(), o.rewards(), o.terminated()))
    return trace


def test_per_ply_invariants():
    N = 11
    for seed in (0, 1):
        prev_obs = None
        o = hx.HexOracle(16, N, seed=seed)
        for t in range(N * N + 1):
            was_over = o.terminated().copy()
            cur = o.current_player()
            a = o.random_actions(seed, t)
            o.step(a)
            s, m, ob = o.export_state(), o.legal_mask(), o.observe()
            bd = s.board.reshape(-1, N, N)
            assert ((ob[..., 0] + ob[..., 1]) == (bd != 0)).all()
            assert (m[:, :N * N].reshape(-1, N, N) == (bd == 0)).all()
            assert (m[:, N * N] == (s.steps == 1)).all()
            mine = np.where(s.to_play[:, None, None] == 1, bd == 1, bd == -1)
            assert (ob[..., 0] == mine).all()
            assert (ob[..., 2] == (s.to_play == 1)[:, None, None]).all()
            assert (ob[..., 3] == (s.steps == 1)[:, None, None]).all()
            live = was_over == 0
            # the seat alternates while the game goes on; a swap is a ply like any other
            assert (o.current_player()[live] == 1 - cur[live]).all()
            nb, nw = (bd == 1).sum((1, 2)), (bd == -1).sum((1, 2))
            swapped = (s.steps >= 2) & (nb + nw == s.steps - 1)
            assert ((nb + nw == s.steps) | swapped).all()
            r = o.rewards()
            fin = (o.terminated() == 1) & live
            assert (np.abs(r[fin]).sum(1) == 2).all() and (r[fin].sum(1) == 0).all() and (r[~fin] == 0).all()
        assert (o.terminated() == 1).all()                          # no game outlasts N*N+1 plies


def test_half_turn_symmetry():
    """Turning the board by 180 degrees keeps both the adjacency and the sides."""
    N = 11
    P = N * N
    for seed in range(3):
        a_ = hx.HexOracle(4, N, seed=seed)
        b_ = hx.HexOracle(4, N, seed=seed)
        for t in range(P + 1):
            a = a_.random_actions(seed, t)
            a_.step(a)
            b_.step(np.where((a >= 0) & (a < P), P - 1 - a, a))
            sa, sb = a_.export_state(), b_.export_state()
            assert (sa.board.reshape(-1, N, N)[:, ::-1, ::-1] == sb.board.reshape(-1, N, N)).all()
            assert (a_.terminated() == b_.terminated()).all() and (a_.rewards() == b_.rewards()).all()


def test_transpose_and_recolour_symmetry():
    rng = np.random.default_rng(2)
    for N in (4, 7, 11):
        for _ in range(200):
            b = rng.integers(-1, 2, size=(N, N)).astype(np.int8)
            assert hx.joined(b, N, 1) == hx.joined(-b.T, N, -1)
            assert hx.joined(b, N, -1) == hx.joined(-b.T, N, 1)


def test_auto_reset_and_seats():
    N = 11
    o = hx.HexOracle(32, N, seed=6, auto_reset=True)
    ends = 0
    for t in range(400):
        ep0 = o.export_state().episode.copy()
        o.step(o.random_actions(6, t))
        s = o.export_state()
        fin = o.terminated() == 1
        ends += int(fin.sum())
        assert (s.episode == ep0 + fin).all()
        assert (s.steps[fin] == 0).all() and (s.board[fin] == 0).all() and (s.to_play[fin] == 1).all() and (s.terminated[fin] == 0).all()
        for b in np.flatnonzero(fin):
            assert s.black_player[b] == (hx.hash4(6, 1, b, int(s.episode[b])) & 1)
            assert o.legal_mask()[b, :121].all() and o.legal_mask()[b, 121] == 0
    assert ends >= 64                                               # random games last ~100 plies
    assert {0, 1} <= set(o.export_state().black_player.tolist())


def test_env_ids_select_the_same_games():
    N = 11
    full = hx.HexOracle(40, N, seed=8, auto_reset=True)
    ids = np.array([3, 17, 39], np.int32)
    part = hx.HexOracle(3, N, seed=8, auto_reset=True, env_ids=ids)
    for t in range(260):
        full.step(full.random_actions(8, t))
        part.step(part.random_actions(8, t))
        assert (full.observe()[ids] == part.observe()).all() and (full.rewards()[ids] == part.rewards()).all()


def test_sampler_is_kth_legal_and_uniform():
    N = 11
    o = hx.HexOracle(64, N, seed=3)
    o.step(np.full(64, 60, np.int32))                               # swap is now on offer: 121 legal actions
    counts = np.zeros(122, np.int64)
    for t in range(400):
        a = o.random_actions(12345, t)
        m = o.legal_mask()
        for b in range(64):
            legal = np.flatnonzero(m[b])
            assert a[b] == legal[hx.hash4(12345, 0, b, t) % len(legal)]
        counts += np.bincount(a, minlength=122)
    assert counts[60] == 0 and counts[121] > 0
    exp = 64 * 400 / 121
    assert np.abs(counts[np.arange(122) != 60] - exp).max() < 6 * np.sqrt(exp)


def test_hash_matches_independent_expression():
    M = 0xFFFFFFFF

    def mix(x):
        x ^= x >> 16; x = (x * 0x7feb352d) & M
        x ^= x >> 15; x = (x * 0x846ca68b) & M
        return x ^ (x >> 16)

    for seed, tag, env, t in [(0, 0, 0, 0), (3, 1, 16383, 7), (0xDEADBEEF, 2, 65535, 1999)]:
        assert hx.hash4(seed, tag, env, t) == mix(mix(mix((seed + 0x9E3779B9 * (tag + 1)) & M) ^ env) ^ t)


def test_export_import_roundtrip():
    N = 11
    o = hx.HexOracle(8, N, seed=2)
    for t in range(30):
        o.step(o.random_actions(2, t))
    s = o.export_state()
    q = hx.HexOracle(8, N, seed=2)
    q.import_state(s)
    assert (q.legal_mask() == o.legal_mask()).all() and (q.observe() == o.observe()).all()
    for t in range(30, 122):
        a = o.random_actions(2, t)
        assert (a == q.random_actions(2, t)).all()
        o.step(a); q.step(a)
        assert (q.observe() == o.observe()).all() and (q.rewards() == o.rewards()).all() and (q.terminated() == o.terminated()).all()
