"""Pins of the oracle's positional superko option (Appendix C "Go": Tromp-Taylor rules): a hand-built
send-two-return-one cycle, a triple ko, and the independent Python implementation on small boards.  No GPU."""
import itertools

import numpy as np
import pytest

import oracle
from pyref import RefGame

N9 = 9
PASS = N9 * N9


def a9(r, c):
    return r * N9 + c


# Black sends two stones, White takes them, Black takes back one: the position before Black's first stone returns.
SEND_TWO = [a9(0, 1), a9(1, 0), a9(0, 3), a9(1, 1), a9(1, 2), a9(8, 8),     # set-up: B (0,1) (0,3) (1,2), W (1,0) (1,1) (8,8)
            a9(0, 0),                                                      # B joins (0,1): two stones, one liberty
            a9(0, 2)]                                                      # W takes both
RETURN_ONE = a9(0, 1)                                                      # B takes the white stone back: the set-up position again


def play(o, moves):
    for m in moves:
        assert o.terminated()[0] == 0 and o.legal_mask()[0, m] == 1
        o.step([m])


def test_send_two_return_one():
    for superko in (False, True):
        o = oracle.GoOracle(1, N9, superko=superko)
        play(o, SEND_TWO)
        before = o.export_state()
        assert before.board[0, a9(0, 0)] == 0 and before.board[0, a9(0, 1)] == 0 and before.board[0, a9(0, 2)] == -1
        assert before.ko[0] == -1                                          # two stones were taken: no simple ko
        assert o.legal_mask()[0, RETURN_ONE] == 1                          # the mask shows the simple-ko set either way
        mover = o.current_player()[0]
        o.step([RETURN_ONE])
        if superko:
            assert o.terminated()[0] == 1 and o.illegal_count()[0] == 1
            assert o.rewards()[0, mover] == -1 and o.rewards()[0, 1 - mover] == 1
            assert (o.export_state().board == before.board).all()         # the position stays as it was
        else:
            assert o.terminated()[0] == 0 and o.illegal_count()[0] == 0
            assert o.export_state().board[0, a9(0, 2)] == 0


def test_other_moves_stay_legal_with_superko():
    o = oracle.GoOracle(1, N9, superko=True)
    play(o, SEND_TWO)
    o.step([a9(5, 5)])
    assert o.terminated()[0] == 0
    o.step([PASS]); o.step([RETURN_ONE])                                   # now a white stone more stands on the board: no repeat
    assert o.terminated()[0] == 0 and o.illegal_count()[0] == 0


def test_pass_never_violates():
    o = oracle.GoOracle(1, N9, superko=True)
    o.step([a9(4, 4)]); o.step([PASS])
    assert o.terminated()[0] == 0
    o.step([PASS])
    assert o.terminated()[0] == 1 and o.illegal_count()[0] == 0           # two passes end the game normally


def test_auto_reset_forgets_the_old_game():
    o = oracle.GoOracle(1, N9, superko=True, auto_reset=True)
    play(o, SEND_TWO)
    o.step([RETURN_ONE])                                                   # violation: game over, fresh game
    assert o.terminated()[0] == 1 and o.export_state().episode[0] == 1
    for m in SEND_TWO:                                                     # the same positions are new in the new game
        o.step([m])
        assert o.terminated()[0] == 0
    assert o.illegal_count()[0] == 1 and o.export_state().episode[0] == 1


@pytest.mark.parametrize("N,depth", [(2, 7), (3, 4)])
def test_exhaustive_against_python(N, depth):
    A = N * N + 1
    hits = 0
    for seq in itertools.product(range(A), repeat=depth):
        ref = RefGame(N, superko=True)
        o = oracle.GoOracle(1, N, superko=True)
        for a in seq:
            was = 0 <= a <= N * N and ref.legal(a) and ref.recreates(a)
            ref.step(a)
            o.step([a])
            assert o.export_state().board[0].tolist() == ref.board()
            assert bool(o.terminated()[0]) == ref.terminated and o.rewards()[0].tolist() == ref.rewards
            hits += was
            if ref.terminated:
                break
    assert hits > 0 or N > 2                                               # 3x3 cannot cycle within 4 plies; 2x2 does within 7


def test_random_games_against_python():
    rng = np.random.default_rng(17)
    hits = 0
    for N in (3, 4, 5, 6):
        for g in range(150 if N < 5 else 25):
            ref = RefGame(N, superko=True, black_player=0)
            o = oracle.GoOracle(1, N, seed=g, superko=True)
            bp = int(o.export_state().black_player[0])
            ref.black_player = bp
            while not ref.terminated:
                m = o.legal_mask()[0]
                assert m.tolist() == ref.mask()
                legal = np.flatnonzero(m[:-1])
                a = int(rng.choice(legal)) if (len(legal) and rng.random() < 0.93) else N * N
                hits += ref.legal(a) and ref.recreates(a)
                ref.step(a)
                o.step([a])
                assert o.export_state().board[0].tolist() == ref.board()
                assert bool(o.terminated()[0]) == ref.terminated and o.rewards()[0].tolist() == ref.rewards
    assert hits >= 4                                                       # small boards cycle now and then


def test_superko_differs_from_simple_ko_only_at_violations():
    """Same actions with and without the option: identical until the first violation, which ends only the superko game."""
    seed, B = 5, 2048
    a_ = oracle.GoOracle(B, 5, seed=seed)
    b_ = oracle.GoOracle(B, 5, seed=seed, superko=True)
    alive = np.ones(B, bool)
    ended_by_rule = 0
    for t in range(50):
        act = a_.random_actions(seed, t)
        a_.step(act); b_.step(act)
        diverged = alive & (b_.illegal_count() > 0) & (a_.illegal_count() == 0)
        ended_by_rule += int(diverged.sum())
        alive &= ~diverged
        sa, sb = a_.export_state(), b_.export_state()
        assert (sa.board[alive] == sb.board[alive]).all() and (a_.terminated()[alive] == b_.terminated()[alive]).all()
    assert ended_by_rule > 0


def test_import_keeps_the_history_window():
    o = oracle.GoOracle(1, N9, superko=True)
    play(o, SEND_TWO)
    s = o.export_state()
    q = oracle.GoOracle(1, N9, superko=True)
    q.import_state(s)                                                      # the set-up position is 2 plies back: inside the 8-position window
    q.step([RETURN_ONE])
    assert q.terminated()[0] == 1 and q.illegal_count()[0] == 1
    q2 = oracle.GoOracle(1, N9)
    q2.import_state(s)
    q2.set_superko(True)                                                   # switching on later rebuilds the set from the window as well
    q2.step([RETURN_ONE])
    assert q2.terminated()[0] == 1
