"""Invariants, symmetries and scoring properties that any correct Go environment satisfies."""
import numpy as np
import pytest

import oracle


def chains_all_have_liberties(board, N):
    return all(board[p] == 0 or oracle.chain(board, N, p)[1] >= 1 for p in range(N * N))


@pytest.mark.parametrize("N,B,T", [(9, 16, 200), (19, 4, 500)])
def test_per_ply_invariants(N, B, T):
    P = N * N
    o = oracle.GoOracle(B, N, seed=N, auto_reset=False)
    prev, prev_obs = o.export_state(), o.observe().reshape(B, P, 17)
    for t in range(T):
        a = o.random_actions(N, t)
        o.step(a)
        s, m, ob = o.export_state(), o.legal_mask(), o.observe().reshape(B, P, 17)
        for b in range(B):
            if prev.terminated[b]:
                continue
            col = int(prev.to_play[b])
            nb, pb = s.board[b], prev.board[b]
            assert chains_all_have_liberties(nb, N)
            if a[b] == P:
                assert (nb == pb).all() and s.ko[b] == -1
            else:
                assert pb[a[b]] == 0 and nb[a[b]] == col
                assert (nb == col).sum() == (pb == col).sum() + 1          # mover gains exactly the new stone
                changed = np.flatnonzero(nb != pb)
                removed = [q for q in changed if q != a[b]]
                assert all(pb[q] == -col and nb[q] == 0 for q in removed)   # only opponent stones disappear
            assert m[b, P] == 1 and not m[b, :P][nb != 0].any()
            assert s.ko[b] == -1 or (nb[s.ko[b]] == 0 and m[b, s.ko[b]] == 0)
            assert s.steps[b] == prev.steps[b] + 1 and s.to_play[b] == -col
            # planes 0/1 partition the occupied points
            assert not (ob[b, :, 0] & ob[b, :, 1]).any() and ((ob[b, :, 0] | ob[b, :, 1]) == (nb != 0)).all()
            # history shifts by one ply and the perspective flips
            for i in range(7):
                assert (ob[b, :, 2 * i + 2] == prev_obs[b, :, 2 * i + 1]).all()
                assert (ob[b, :, 2 * i + 3] == prev_obs[b, :, 2 * i]).all()
            assert (ob[b, :, 16] == (1 if s.to_play[b] == 1 else 0)).all()
        prev, prev_obs = s, ob


def sym_maps(N):
    """The 8 symmetries of the square as point permutations: new_index = perm[old_index]."""
    idx = np.arange(N * N).reshape(N, N)
    out = []
    for k in range(4):
        for flip in (False, True):
            g = np.rot90(idx, k)
            if flip:
                g = g.T
            perm = np.empty(N * N, np.int64)
            perm[g.reshape(-1)] = np.arange(N * N)   # old point g[r,c] moves to (r,c)
            out.append(perm)
    return out


@pytest.mark.parametrize("N", [5, 9])
def test_board_symmetries_commute_with_the_rules(N):
    P = N * N
    base = oracle.GoOracle(1, N, seed=3)
    script = []
    for t in range(120):
        a = int(base.random_actions(9, t)[0])
        script.append(a)
        base.step([a])
        if base.terminated()[0]:
            break
    for perm in sym_maps(N):
        o1 = oracle.GoOracle(1, N, seed=3)
        o2 = oracle.GoOracle(1, N, seed=3)
        for a in script:
            a2 = a if a == P else int(perm[a])
            o1.step([a]); o2.step([a2])
            s1, s2 = o1.export_state(), o2.export_state()
            moved = np.empty(P, np.int8); moved[perm] = s1.board[0]
            assert (moved == s2.board[0]).all()
            m1, m2 = o1.legal_mask()[0], o2.legal_mask()[0]
            mm = np.empty(P, np.uint8); mm[perm] = m1[:P]
            assert (mm == m2[:P]).all()
            ob1, ob2 = o1.observe()[0].reshape(P, 17), o2.observe()[0].reshape(P, 17)
            obm = np.empty_like(ob1); obm[perm] = ob1
            assert (obm == ob2).all()
            assert (o1.rewards() == o2.rewards()).all() and (o1.terminated() == o2.terminated()).all()
            assert s2.ko[0] == (-1 if s1.ko[0] < 0 else perm[s1.ko[0]])


def test_area_properties():
    rng = np.random.default_rng(3)
    N = 7
    for _ in range(200):
        board = rng.choice([0, 1, -1], size=N * N, p=[0.5, 0.25, 0.25]).astype(np.int8)
        ab, aw = oracle.area(board, N)
        assert oracle.area(-board, N) == (aw, ab)                        # colour swap
        assert ab + aw <= N * N and ab >= (board == 1).sum() and aw >= (board == -1).sum()
        for perm in sym_maps(N):
            moved = np.empty_like(board); moved[perm] = board
            assert oracle.area(moved, N) == (ab, aw)


def parse(rows):
    return np.array([{"X": 1, "O": -1, ".": 0}[ch] for line in rows for ch in line.replace(" ", "")], np.int8)


def test_area_hand_counted_positions():
    # wall splits the board: left region touches only black, right only white
    b = parse([". X O . .",
               ". X O . .",
               ". X O . .",
               ". X O . .",
               ". X O . ."])
    assert oracle.area(b, 5) == (10, 15)
    # an empty region touching both colours counts for nobody
    b = parse([". X . O .",
               ". X . O .",
               ". X . O .",
               ". X . O .",
               ". X . O ."])
    assert oracle.area(b, 5) == (10, 10)
    # a one-point black eye inside a black wall, the rest neutral
    b = parse([". X . . .",
               "X X . . .",
               ". . . O .",
               ". . . . .",
               ". . . . ."])
    assert oracle.area(b, 5) == (4, 1)
    assert oracle.area(parse(["." * 3] * 3), 3) == (0, 0)
    assert oracle.area(parse(["...", ".X.", "..."]), 3) == (9, 0)
    assert oracle.area(parse(["...", ".O.", "..."]), 3) == (0, 9)


def test_final_reward_equals_area_score_sign():
    N, B = 9, 64
    o = oracle.GoOracle(B, N, seed=21, komi_x2=15)
    done = np.zeros(B, bool)
    for t in range(2 * N * N):
        o.step(o.random_actions(21, t))
        term, rew, s = o.terminated(), o.rewards(), o.export_state()
        for b in np.flatnonzero((term == 1) & ~done):
            ab, aw = oracle.area(s.board[b], N)
            d = 2 * (ab - aw) - 15
            want = 1.0 if d > 0 else -1.0
            bp = int(s.black_player[b])
            assert rew[b, bp] == want and rew[b, 1 - bp] == -want
        assert (rew[term == 0] == 0).all()
        done |= term == 1
    assert done.all()
