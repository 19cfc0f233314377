"""Pins of the CPU oracle against an independent pure-Python implementation (tests/pyref.py)
on tiny boards, and of the chain-based legality against literal trial placement."""
import itertools
import random

import numpy as np
import pytest

import oracle
import pyref


def compare_game(o, g, N):
    s = o.export_state()
    assert s.board[0].tolist() == g.board()
    assert s.to_play[0] == g.to_play
    assert s.ko[0] == (-1 if g.ko is None else g.ko[0] * N + g.ko[1])
    assert s.steps[0] == g.steps and s.passes[0] == g.passes
    assert bool(o.terminated()[0]) == g.terminated
    assert o.rewards()[0].tolist() == g.rewards
    if not g.terminated:
        assert o.legal_mask()[0].tolist() == g.mask()
    assert o.observe()[0].tolist() == g.observation()


@pytest.mark.parametrize("N,depth", [(2, 7), (3, 4)])
def test_exhaustive_short_sequences(N, depth):
    """Every action sequence (illegal ones included) up to `depth` plies on a tiny board."""
    A = N * N + 1
    count = 0
    for seq in itertools.product(range(A), repeat=depth):
        o = oracle.GoOracle(1, N, seed=7)
        g = pyref.RefGame(N, black_player=int(o.export_state().black_player[0]))
        for a in seq:
            o.step([a]); g.step(a)
            compare_game(o, g, N)
            count += 1
            if g.terminated:
                break
    assert count > 1000


@pytest.mark.parametrize("N,games", [(3, 60), (4, 40), (5, 40), (7, 10)])
def test_random_games_against_python_reference(N, games):
    rng = random.Random(1234 + N)
    for gi in range(games):
        o = oracle.GoOracle(1, N, seed=gi)
        g = pyref.RefGame(N, black_player=int(o.export_state().black_player[0]))
        while not g.terminated:
            legal = [a for a, ok in enumerate(g.mask()) if ok]
            # mostly board moves so that boards fill up and captures happen; sometimes an illegal one
            if rng.random() < 0.01:
                a = rng.randrange(N * N)
            else:
                pts = [a for a in legal if a != N * N]
                a = rng.choice(pts) if pts and rng.random() < 0.97 else N * N
            o.step([a]); g.step(a)
            compare_game(o, g, N)


@pytest.mark.parametrize("N", [5, 9, 19])
def test_chain_legality_equals_trial_placement_on_rollouts(N):
    B = 8
    o = oracle.GoOracle(B, N, seed=N, auto_reset=True)
    checked = 0
    for t in range(3 * N * N):
        o.step(o.random_actions(N, t))
        if t % 3 == 0 or N == 5:
            s, m = o.export_state(), o.legal_mask()
            for b in range(B):
                assert (m[b] == oracle.legal_trial(s.board[b], N, int(s.to_play[b]), int(s.ko[b]))).all()
                checked += 1
    assert checked > 100


def test_chain_legality_equals_trial_placement_on_random_dense_boards():
    """Arbitrary (even unreachable) stone patterns in which every chain has a liberty, both colours to move."""
    rng = np.random.default_rng(5)
    N = 6
    done = 0
    while done < 300:
        board = rng.choice([0, 1, -1], size=N * N, p=[0.3, 0.35, 0.35]).astype(np.int8)
        if any(board[p] != 0 and oracle.chain(board, N, p)[1] == 0 for p in range(N * N)):
            continue
        for col in (1, -1):
            assert (oracle.legal_chains(board, N, col) == oracle.legal_trial(board, N, col)).all()
        done += 1


def test_liberty_recount_and_area_against_python_reference():
    rng = np.random.default_rng(11)
    for N in (3, 4, 5):
        for _ in range(150):
            board = rng.choice([0, 1, -1], size=N * N, p=[0.4, 0.3, 0.3]).astype(np.int8)
            stones = {divmod(p, N): int(board[p]) for p in range(N * N) if board[p]}
            for p in range(N * N):
                if board[p]:
                    cells, libs = pyref.group(stones, N, divmod(p, N))
                    assert oracle.chain(board, N, p) == (len(cells), len(libs))
            assert oracle.area(board, N) == pyref.area(stones, N)
