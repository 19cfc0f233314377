"""Pins of the oracle's positional superko option (Appendix C "Go": Tromp-Taylor rules) in both readings -- the rule
proper, honoured by the legal mask ("mask"), and the one enforced only when the move is played (True): a hand-built
send-two-return-one cycle, hand-built histories with a repeating play that captures nothing / something, the
independent Python implementation on small boards, and the literal whole-board comparison.  No GPU."""
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


# ---- the rule proper: the legal mask leaves out every play that would recreate an earlier position -------------------

def test_mask_leaves_out_the_returning_stone():
    o = oracle.GoOracle(1, N9, superko="mask")
    play(o, SEND_TWO)
    m = o.legal_mask()[0]
    assert m[RETURN_ONE] == 0 and m[PASS] == 1
    simple = oracle.legal_chains(o.export_state().board[0], N9, 1, -1)
    assert simple[RETURN_ONE] == 1 and (m == simple).sum() == N9 * N9          # the only point the rule takes away
    mover = o.current_player()[0]
    before = o.export_state().board.copy()
    o.step([RETURN_ONE])                                                       # played anyway: an illegal action like any other
    assert o.terminated()[0] == 1 and o.illegal_count()[0] == 1 and o.rewards()[0, mover] == -1
    assert (o.export_state().board == before).all()
    q = oracle.GoOracle(1, N9, superko="mask")
    play(q, SEND_TWO)
    q.step([a9(5, 5)]); q.step([PASS])
    assert q.legal_mask()[0, RETURN_ONE] == 1                                  # another stone stands elsewhere now: no repeat


def hand_history(cur, earlier, to_play):
    """State whose current board is `cur` and whose previous position (one ply ago) is `earlier` (dicts point -> colour)."""
    s = oracle.State(1, N9 * N9)
    for p, v in cur.items():
        s.board[0, p] = v
    s.history[0, 0] = s.board[0]
    for p, v in earlier.items():
        s.history[0, 1, p] = v
    s.ko[0] = -1; s.to_play[0] = to_play; s.steps[0] = 20
    return s


def test_repeating_play_that_captures_nothing():
    # the earlier position is the current one plus a black stone on (4,4): Black's play there would bring it back
    cur = {a9(2, 2): 1, a9(6, 6): -1, a9(3, 7): -1}
    earlier = dict(cur); earlier[a9(4, 4)] = 1
    for mode, expect in ((0, 1), (1, 1), ("mask", 0)):
        o = oracle.GoOracle(1, N9, superko=mode)
        o.import_state(hand_history(cur, earlier, 1))
        m = o.legal_mask()[0]
        assert m[a9(4, 4)] == expect and m[a9(4, 5)] == 1
        o.step([a9(4, 4)])
        assert o.terminated()[0] == (0 if mode == 0 else 1)
    w = oracle.GoOracle(1, N9, superko="mask")                                  # White's stone on the same point gives another position
    w.import_state(hand_history(cur, earlier, -1))
    assert w.legal_mask()[0, a9(4, 4)] == 1


def test_repeating_play_that_captures():
    # White stones (0,0),(0,1) have one liberty left at (0,2) next to black (1,0),(1,1); Black takes them there.
    # An earlier position equal to the result makes that capture a repetition; a different capture size or stone does not.
    cur = {a9(0, 0): -1, a9(0, 1): -1, a9(1, 0): 1, a9(1, 1): 1, a9(7, 7): -1}
    after = {a9(1, 0): 1, a9(1, 1): 1, a9(7, 7): -1, a9(0, 2): 1}
    o = oracle.GoOracle(1, N9, superko="mask")
    o.import_state(hand_history(cur, after, 1))
    assert o.legal_mask()[0, a9(0, 2)] == 0
    near = dict(after); near[a9(0, 1)] = -1                                    # only one of the two stones gone: not what the capture gives
    o.import_state(hand_history(cur, near, 1))
    assert o.legal_mask()[0, a9(0, 2)] == 1


@pytest.mark.parametrize("N,depth", [(2, 7), (3, 4)])
def test_mask_level_exhaustive_against_python(N, depth):
    A = N * N + 1
    taken = 0
    for seq in itertools.product(range(A), repeat=depth):
        ref = RefGame(N, superko=True)
        o = oracle.GoOracle(1, N, superko="mask")
        for a in seq:
            want = [1 if (ref.legal(x) and not ref.recreates(x)) else 0 for x in range(A)]
            assert o.legal_mask()[0].tolist() == want
            taken += sum(ref.mask()) - sum(want)
            ref.step(a)
            o.step([a])
            assert o.export_state().board[0].tolist() == ref.board()
            assert bool(o.terminated()[0]) == ref.terminated and o.rewards()[0].tolist() == ref.rewards
            if ref.terminated:
                break
    assert taken > 0 or N > 2


def test_mask_level_random_games_against_python():
    rng = np.random.default_rng(23)
    taken = played_forbidden = 0
    for N in (3, 4, 5, 6):
        for g in range(150 if N < 5 else 25):
            ref = RefGame(N, superko=True)
            o = oracle.GoOracle(1, N, seed=g, superko="mask")
            ref.black_player = int(o.export_state().black_player[0])
            while not ref.terminated:
                want = [1 if (ref.legal(x) and not ref.recreates(x)) else 0 for x in range(N * N + 1)]
                m = o.legal_mask()[0]
                assert m.tolist() == want
                forbidden = [x for x in range(N * N) if ref.legal(x) and ref.recreates(x)]
                taken += len(forbidden)
                if forbidden and rng.random() < 0.1:
                    a = int(rng.choice(forbidden)); played_forbidden += 1     # now and then play a forbidden point: game over
                else:
                    legal = np.flatnonzero(m[:-1])
                    a = int(rng.choice(legal)) if (len(legal) and rng.random() < 0.93) else N * N
                ref.step(a)
                o.step([a])
                assert o.export_state().board[0].tolist() == ref.board()
                assert bool(o.terminated()[0]) == ref.terminated and o.rewards()[0].tolist() == ref.rewards
    assert taken >= 20 and played_forbidden >= 2


@pytest.mark.parametrize("N,B,plies", [(5, 64, 60), (9, 24, 170)])
def test_counted_comparison_equals_the_literal_one(N, B, plies):
    """The mask uses the comparison that skips earlier positions with other stone counts; it must agree with the literal
    comparison against every earlier position, point by point, and the two readings must differ only in the mask."""
    seed = 3
    o = oracle.GoOracle(B, N, seed=seed, superko="mask", auto_reset=True)
    taken = 0
    for t in range(plies):
        st = o.export_state()
        m = o.legal_mask()
        for b in range(B):
            simple = oracle.legal_chains(st.board[b], N, int(st.to_play[b]), int(st.ko[b]))
            for p_ in np.flatnonzero(simple[:-1]):
                rep = o.repeats_literal(b, int(p_))
                assert m[b, p_] == (0 if rep else 1)
                taken += rep
            assert (m[b][simple == 0] == 0).all() and m[b, -1] == 1
        o.step(o.random_actions(seed, t))
    assert taken > 0 or N == 9                                                 # 9x9 games rarely offer a repeating play


def test_the_two_readings_agree_on_what_is_a_violation():
    seed, B = 5, 1024
    a_ = oracle.GoOracle(B, 5, seed=seed, superko=True)                         # enforced at play time
    b_ = oracle.GoOracle(B, 5, seed=seed, superko="mask")                        # honoured by the mask
    differ = 0
    for t in range(60):
        act = a_.random_actions(seed, t)                                         # drawn from the simple-ko mask
        ma, mb = a_.legal_mask(), b_.legal_mask()
        assert (mb <= ma).all()
        differ += int((ma != mb).sum())
        a_.step(act); b_.step(act)
        sa, sb = a_.export_state(), b_.export_state()
        assert (sa.board == sb.board).all() and (a_.terminated() == b_.terminated()).all() and (a_.rewards() == b_.rewards()).all()
        assert (a_.illegal_count() == b_.illegal_count()).all()
    assert differ > 0 and a_.illegal_count().sum() > 0
