"""An independent, pure-Python Hex used to pin the C++ oracle (Appendix C "Hex").

Written differently on purpose: cells are cube coordinates (x, y, z) with x + y + z = 0 and two cells touch
when their coordinates differ by at most one on every axis; groups are tracked incrementally by a union-find
with four virtual nodes for the sides; nothing here looks at an array board.
"""


class Sets:
    def __init__(self):
        self.up = {}

    def find(self, a):
        self.up.setdefault(a, a)
        while self.up[a] != a:
            self.up[a] = self.up[self.up[a]]
            a = self.up[a]
        return a

    def join(self, a, b):
        self.up[self.find(a)] = self.find(b)


def cube(r, c):
    return (c, -c - r, r)


def touching(p, q):
    return p != q and max(abs(p[0] - q[0]), abs(p[1] - q[1]), abs(p[2] - q[2])) == 1


class RefHex:
    def __init__(self, N):
        self.N = N
        self.stones = {}       # (r, c) -> 'B' / 'W'
        self.turn = 'B'
        self.plies = 0
        self.over = False
        self.winner = None
        self.groups = Sets()

    def swap_offered(self):
        return self.plies == 1

    def legal(self, a):
        N = self.N
        if a == N * N:
            return self.swap_offered()
        return 0 <= a < N * N and divmod(a, N) not in self.stones

    def _put(self, r, c, who):
        N = self.N
        self.stones[(r, c)] = who
        me = (who, r, c)
        self.groups.find(me)
        if who == 'B':
            if r == 0: self.groups.join(me, 'top')
            if r == N - 1: self.groups.join(me, 'bottom')
        else:
            if c == 0: self.groups.join(me, 'left')
            if c == N - 1: self.groups.join(me, 'right')
        for (rr, cc), w in self.stones.items():
            if w == who and touching(cube(r, c), cube(rr, cc)):
                self.groups.join(me, (who, rr, cc))

    def has_joined(self, who):
        a, b = ('top', 'bottom') if who == 'B' else ('left', 'right')
        return self.groups.find(a) == self.groups.find(b)

    def play(self, a):
        """Returns 'illegal', 'win' or None."""
        assert not self.over
        if not self.legal(a):
            self.over = True
            self.winner = 'W' if self.turn == 'B' else 'B'
            return 'illegal'
        who = self.turn
        if a == self.N * self.N:
            ((r, c), _), = self.stones.items()
            self.stones = {}
            self.groups = Sets()
            self._put(c, r, who)
        else:
            self._put(*divmod(a, self.N), who)
        self.plies += 1
        self.turn = 'W' if who == 'B' else 'B'
        if self.has_joined(who):
            self.over = True
            self.winner = who
            return 'win'
        return None

    def board(self):
        N = self.N
        return [[{'B': 1, 'W': -1}.get(self.stones.get((r, c)), 0) for c in range(N)] for r in range(N)]
