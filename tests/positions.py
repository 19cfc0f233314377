"""Hand-built rule positions as action scripts through the public API.

Each script alternates Black, White, Black, ... from the empty 9x9 board; an entry is a
(row, col) point or "P" (pass).  Same-colour stones are placed by letting the other side
pass or play far away; nobody passes twice in a row, so no script ends a game early.
The expected boards were written out by hand from the rules ('X' black, 'O' white,
'.' empty, only the top-left corner rows given; every other row is empty unless the
script's far-away stones are listed in `extra`).  The same scripts drive the CPU oracle
tests and the GPU parity tests; this module contains no rule arithmetic.
"""
N = 9
P = "P"


def idx(rc):
    return N * N if rc == P else rc[0] * N + rc[1]


def parse(rows, extra=()):
    """rows: list of strings for the top rows, each of N chars.  extra: ((r,c), 'X'|'O')."""
    board = [0] * (N * N)
    for r, line in enumerate(rows):
        line = line.replace(" ", "")
        assert len(line) == N, line
        for c, ch in enumerate(line):
            board[r * N + c] = {"X": 1, "O": -1, ".": 0}[ch]
    for (r, c), ch in extra:
        board[r * N + c] = {"X": 1, "O": -1}[ch]
    return board


SCRIPTS = {}

# 1. corner capture: the white corner stone loses its two liberties.
SCRIPTS["corner_capture"] = dict(
    moves=[(0, 1), (0, 0), (1, 0)],
    board=parse([". X . . . . . . .",
                 "X . . . . . . . ."]),
    ko=-1, to_play=-1,
    illegal_next=[(0, 0)],          # suicide for White: both neighbours are black chains with spare liberties
    legal_next=[(1, 1), (0, 2)],
)

# 2. two stones on the edge captured at once; capturing two stones never makes a ko.
SCRIPTS["edge_capture_two"] = dict(
    moves=[(0, 2), (0, 3), (1, 3), (0, 4), (1, 4), P, (0, 5)],
    board=parse([". . X . . X . . .",
                 ". . . X X . . . ."]),
    ko=-1, to_play=-1,
    legal_next=[(0, 3), (0, 4)],    # two adjacent empty points: each has an empty neighbour
)

# 3. ko: Black takes one stone with a lone stone left in atari.
_ko_moves = [(0, 1), (0, 2), (1, 0), (1, 3), (2, 1), (2, 2), (8, 8), (1, 1), (1, 2)]
SCRIPTS["ko_created"] = dict(
    moves=_ko_moves,
    board=parse([". X O . . . . . .",
                 "X . X O . . . . .",
                 ". X O . . . . . ."], extra=[((8, 8), "X")]),
    ko=(1, 1), to_play=-1,
    illegal_next=[(1, 1)],
)
# 3b. the ko ban lasts one ply: after a move elsewhere by each side White may retake, which makes a new ko for Black.
SCRIPTS["ko_retaken_later"] = dict(
    moves=_ko_moves + [(7, 7), (8, 0), (1, 1)],
    board=parse([". X O . . . . . .",
                 "X O . O . . . . .",
                 ". X O . . . . . ."], extra=[((8, 8), "X"), ((7, 7), "O"), ((8, 0), "X")]),
    ko=(1, 2), to_play=1,
    illegal_next=[(1, 2)],
)
# 3c. a pass also lifts the ban.
SCRIPTS["ko_cleared_by_pass"] = dict(
    moves=_ko_moves + [P],
    board=parse([". X O . . . . . .",
                 "X . X O . . . . .",
                 ". X O . . . . . ."], extra=[((8, 8), "X")]),
    ko=-1, to_play=1,
    legal_next=[(1, 1)],            # Black may fill the ko
)
SCRIPTS["ko_retake_after_pass"] = dict(
    moves=_ko_moves + [P, (8, 0), (1, 1)],
    board=parse([". X O . . . . . .",
                 "X O . O . . . . .",
                 ". X O . . . . . ."], extra=[((8, 8), "X"), ((8, 0), "X")]),
    ko=(1, 2), to_play=1,
)

# 4. multi-stone suicide is illegal; the same point is a capture for the other side.
SCRIPTS["multi_stone_suicide"] = dict(
    moves=[(0, 2), (0, 0), (1, 1), (8, 8), (1, 0)],
    board=parse(["O . X . . . . . .",
                 "X X . . . . . . ."], extra=[((8, 8), "O")]),
    ko=-1, to_play=-1,
    illegal_next=[(0, 1)],          # would join the corner stone into a two-stone chain without liberties
)
SCRIPTS["capture_instead_of_suicide"] = dict(
    moves=[(0, 2), (0, 0), (1, 1), (8, 8), (1, 0), (8, 7), (0, 1)],
    board=parse([". X X . . . . . .",
                 "X X . . . . . . ."], extra=[((8, 8), "O"), ((8, 7), "O")]),
    ko=-1, to_play=-1,              # the capturing stone has own-colour neighbours: no ko
    illegal_next=[(0, 0)],
)

# 5. one stone captures two separate one-stone chains; legal only because it captures.
SCRIPTS["capture_two_chains"] = dict(
    moves=[(0, 2), (0, 1), (1, 1), (1, 0), (2, 0), (8, 8), (0, 0)],
    board=parse(["X . X . . . . . .",
                 ". X . . . . . . .",
                 "X . . . . . . . ."], extra=[((8, 8), "O")]),
    ko=-1, to_play=-1,
)

# 6. one stone captures four separate chains around it.
SCRIPTS["capture_four_chains"] = dict(
    moves=[(2, 4), (3, 4), (3, 3), (5, 4), (3, 5), (4, 3), (6, 4), (4, 5), (5, 3), P, (5, 5), P, (4, 2), P, (4, 6), P, (4, 4)],
    board=parse([". . . . . . . . .",
                 ". . . . . . . . .",
                 ". . . . X . . . .",
                 ". . . X . X . . .",
                 ". . X . X . X . .",
                 ". . . X . X . . .",
                 ". . . . X . . . ."]),
    ko=-1, to_play=-1,
    illegal_next=[(3, 4), (4, 3), (4, 5), (5, 4)],   # each vacated point is now surrounded by safe black chains
)

# 7. snapback: the throw-in stone is taken (one stone, but by a stone with a friend: no ko) and
#    Black retakes five stones on the vacated point.
_snap = [(2, 0), (1, 0), (2, 1), (1, 1), (2, 2), (1, 2), (1, 3), (0, 2), (0, 3), P, (0, 1)]
SCRIPTS["snapback_throw_in"] = dict(
    moves=_snap,
    board=parse([". X O X . . . . .",
                 "O O O X . . . . .",
                 "X X X . . . . . ."]),
    ko=-1, to_play=-1,
    legal_next=[(0, 0)],
)
SCRIPTS["snapback_taken"] = dict(
    moves=_snap + [(0, 0)],
    board=parse(["O . O X . . . . .",
                 "O O O X . . . . .",
                 "X X X . . . . . ."]),
    ko=-1, to_play=1,
    legal_next=[(0, 1)],
)
SCRIPTS["snapback_recapture"] = dict(
    moves=_snap + [(0, 0), (0, 1)],
    board=parse([". X . X . . . . .",
                 ". . . X . . . . .",
                 "X X X . . . . . ."]),
    ko=-1, to_play=-1,
)

# 8. a lone stone takes two stones and is left with one liberty: still no ko.
SCRIPTS["two_stone_capture_no_ko"] = dict(
    moves=[(1, 0), (0, 0), (1, 1), (0, 1), (8, 8), (0, 3), (8, 7), (1, 2), (0, 2)],
    board=parse([". . X O . . . . .",
                 "X X O . . . . . ."], extra=[((8, 8), "X"), ((8, 7), "X")]),
    ko=-1, to_play=-1,
    legal_next=[(0, 1), (0, 0)],
)

# 9. pass on the first ply, then a stone: nothing special, passes reset.
SCRIPTS["pass_then_play"] = dict(
    moves=[P, (4, 4), (4, 5)],
    board=parse([". . . . . . . . ."] * 4 + [". . . . O X . . ."]),
    ko=-1, to_play=-1,
)
