"""Independent pure-Python Go rules used only to pin the C++ oracle on small cases.

Written with sets and recursion-free graph search on (row, col) tuples; it shares no
code with oracle/ or with the HIP library.  Rules: Tromp-Taylor area scoring with
komi for White (paper Appendix C "Go"), suicide illegal, simple ko, pass = action N*N,
game over after two consecutive passes or 2*N*N plies.
"""
BLACK, WHITE, EMPTY = 1, -1, 0


def nbrs(N, rc):
    r, c = rc
    for dr, dc in ((-1, 0), (1, 0), (0, -1), (0, 1)):
        rr, cc = r + dr, c + dc
        if 0 <= rr < N and 0 <= cc < N:
            yield (rr, cc)


def group(stones, N, rc):
    """stones: dict (r,c)->colour.  Returns (set of cells of the chain at rc, set of its liberties)."""
    col = stones[rc]
    todo, cells, libs = [rc], {rc}, set()
    while todo:
        x = todo.pop()
        for y in nbrs(N, x):
            if y not in stones:
                libs.add(y)
            elif stones[y] == col and y not in cells:
                cells.add(y)
                todo.append(y)
    return cells, libs


def try_play(stones, N, rc, col):
    """Returns (new stones dict, captured cell set) or None when rc is occupied or the move is suicide."""
    if rc in stones:
        return None
    new = dict(stones)
    new[rc] = col
    captured = set()
    for y in nbrs(N, rc):
        if y in new and new[y] == -col:
            cells, libs = group(new, N, y)
            if not libs:
                captured |= cells
                for z in cells:
                    del new[z]
    _, libs = group(new, N, rc)
    if not libs:
        return None
    return new, captured


def area(stones, N):
    seen, score = set(), {BLACK: 0, WHITE: 0}
    for v in stones.values():
        score[v] += 1
    for r in range(N):
        for c in range(N):
            if (r, c) in stones or (r, c) in seen:
                continue
            region, touch, todo = {(r, c)}, set(), [(r, c)]
            while todo:
                x = todo.pop()
                for y in nbrs(N, x):
                    if y in stones:
                        touch.add(stones[y])
                    elif y not in region:
                        region.add(y)
                        todo.append(y)
            seen |= region
            if len(touch) == 1:
                score[touch.pop()] += len(region)
    return score[BLACK], score[WHITE]


class RefGame:
    """One game with the same observable behaviour as one oracle environment."""

    def __init__(self, N, komi_x2=15, max_steps=None, black_player=0, superko=False):
        self.N, self.P = N, N * N
        self.komi_x2 = komi_x2
        self.max_steps = max_steps or 2 * N * N
        self.stones = {}
        self.to_play = BLACK
        self.ko = None
        self.passes = 0
        self.steps = 0
        self.terminated = False
        self.black_player = black_player
        self.rewards = [0.0, 0.0]
        self.past = []  # positions after each ply, newest last
        self.superko = superko                 # positional superko, enforced when the move is played
        self.shown = {frozenset()}             # every position the game has shown, as a set of (cell, colour) pairs

    def legal(self, a):
        if a == self.P:
            return True
        rc = divmod(a, self.N)
        if rc == self.ko:
            return False
        return try_play(self.stones, self.N, rc, self.to_play) is not None

    def recreates(self, a):
        """With superko on: would this (otherwise legal) play bring back a position the game has already shown?"""
        if not self.superko or a == self.P:
            return False
        res = try_play(self.stones, self.N, divmod(a, self.N), self.to_play)
        return res is not None and frozenset(res[0].items()) in self.shown

    def mask(self):
        return [1 if self.legal(a) else 0 for a in range(self.P + 1)]

    def board(self):
        return [self.stones.get(divmod(p, self.N), 0) for p in range(self.P)]

    def step(self, a):
        assert not self.terminated
        self.rewards = [0.0, 0.0]
        col = self.to_play
        mover = self.black_player if col == BLACK else 1 - self.black_player
        if not (0 <= a <= self.P) or not self.legal(a) or self.recreates(a):
            self.rewards[mover], self.rewards[1 - mover] = -1.0, 1.0
            self.terminated = True
            return
        if a == self.P:
            self.passes += 1
            self.ko = None
        else:
            rc = divmod(a, self.N)
            alone = all(self.stones.get(y) != col for y in nbrs(self.N, rc))
            self.stones, captured = try_play(self.stones, self.N, rc, col)
            cells, libs = group(self.stones, self.N, rc)
            self.ko = next(iter(captured)) if (len(captured) == 1 and alone and len(cells) == 1 and libs == captured) else None
            self.passes = 0
        self.steps += 1
        self.shown.add(frozenset(self.stones.items()))
        self.past.append(dict(self.stones))
        self.to_play = -col
        if self.passes == 2 or self.steps >= self.max_steps:
            ab, aw = area(self.stones, self.N)
            d = 2 * (ab - aw) - self.komi_x2
            s = (d > 0) - (d < 0)
            self.rewards[self.black_player], self.rewards[1 - self.black_player] = float(s), float(-s)
            self.terminated = True

    def observation(self):
        """[N][N][17] nested lists: mover/opponent stones for the last 8 positions, then the colour plane."""
        N = self.N
        hist = list(reversed(self.past))[:8]
        out = [[[0] * 17 for _ in range(N)] for _ in range(N)]
        for i, pos in enumerate(hist):
            for (r, c), v in pos.items():
                out[r][c][2 * i + (0 if v == self.to_play else 1)] = 1
        if self.to_play == BLACK:
            for r in range(N):
                for c in range(N):
                    out[r][c][16] = 1
        return out
