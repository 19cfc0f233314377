"""ctypes front end of the CPU oracle (oracle/go_oracle.cpp).

TEST INFRASTRUCTURE: only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import this package.  It never touches the HIP library.
All arrays are host numpy arrays.
"""
import ctypes as C
import os

import numpy as np

from .build import LIB, build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(os.path.join(os.path.dirname(LIB), "go_oracle.cpp")):
            _build()
        L = C.CDLL(LIB)
        L.oracle_create.restype = C.c_void_p
        L.oracle_create.argtypes = [C.c_int, C.c_int, C.c_uint32, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.oracle_destroy.argtypes = [C.c_void_p]
        L.oracle_reset.argtypes = [C.c_void_p]
        L.oracle_step.argtypes = [C.c_void_p, C.c_void_p]
        L.oracle_random_actions.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]
        L.oracle_hash.restype = C.c_uint32
        L.oracle_hash.argtypes = [C.c_uint32] * 4
        for name in ("legal_mask", "observe", "rewards", "terminated", "current_player", "illegal_count"):
            getattr(L, "oracle_" + name).argtypes = [C.c_void_p, C.c_void_p]
        L.oracle_export_state.argtypes = [C.c_void_p] * 10
        L.oracle_import_state.argtypes = [C.c_void_p] * 10
        L.oracle_legal_trial.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.oracle_legal_chains.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.oracle_area.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.oracle_chain.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.oracle_set_superko.argtypes = [C.c_void_p, C.c_int]
        L.oracle_repeats_literal.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.oracle_seen_count.argtypes = [C.c_void_p, C.c_int]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def hash4(seed, tag, env, t):
    return int(lib().oracle_hash(seed & 0xFFFFFFFF, tag & 0xFFFFFFFF, env & 0xFFFFFFFF, t & 0xFFFFFFFF))


def superko_mode(mode):
    """False / 0 -> 0 (off), True / 1 -> 1 (at play time), "mask" / 2 -> 2 (honoured by the legal mask)."""
    if mode == "mask":
        return 2
    m = int(mode)
    if m not in (0, 1, 2):
        raise ValueError("superko mode must be 0, 1, 2 or 'mask'")
    return m


class State:
    """Canonical per-environment state arrays (host)."""

    __slots__ = ("board", "history", "ko", "to_play", "steps", "passes", "terminated", "black_player", "episode")

    def __init__(self, B, P):
        self.board = np.zeros((B, P), np.int8)
        self.history = np.zeros((B, 8, P), np.int8)
        self.ko = np.zeros(B, np.int32)
        self.to_play = np.zeros(B, np.int8)
        self.steps = np.zeros(B, np.int32)
        self.passes = np.zeros(B, np.int8)
        self.terminated = np.zeros(B, np.uint8)
        self.black_player = np.zeros(B, np.uint8)
        self.episode = np.zeros(B, np.uint32)

    def fields(self):
        return [getattr(self, k) for k in self.__slots__]


class GoOracle:
    """Batched Go environment on the CPU (paper Fig. 2 API: init / step / observation /
    legal_action_mask / rewards / terminated / current_player)."""

    def __init__(self, batch, board_size, seed=0, komi_x2=15, max_steps=0, auto_reset=False, env_ids=None, superko=False):
        self.B, self.N = int(batch), int(board_size)
        self.P = self.N * self.N
        self.A = self.P + 1
        ids = None if env_ids is None else np.ascontiguousarray(env_ids, np.int32)
        self._h = lib().oracle_create(self.B, self.N, seed & 0xFFFFFFFF, komi_x2, max_steps, int(auto_reset), _p(ids))
        if not self._h:
            raise ValueError("oracle_create rejected its arguments")
        if superko:
            self.set_superko(superko)

    def set_superko(self, mode):
        """Positional superko.  False / 0: off.  "mask" / 2: the rule proper, the legal mask leaves out every play that
        would recreate an earlier position of the game.  True / 1: looked at only when the move is played (the
        offender loses), the mask keeps showing the simple-ko set."""
        lib().oracle_set_superko(self._h, superko_mode(mode))

    def repeats_literal(self, b, p):
        """Would the mover's play on empty point p recreate an earlier position of environment b (literal comparison)?"""
        return bool(lib().oracle_repeats_literal(self._h, int(b), int(p)))

    def seen_count(self, b):
        return int(lib().oracle_seen_count(self._h, int(b)))

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and lib is not None:   # module globals are gone when the interpreter shuts down
            lib().oracle_destroy(h)

    def reset(self):
        lib().oracle_reset(self._h)

    def step(self, actions):
        a = np.ascontiguousarray(actions, np.int32)
        assert a.shape == (self.B,)
        lib().oracle_step(self._h, _p(a))

    def random_actions(self, seed, t, start_t=None):
        out = np.empty(self.B, np.int32)
        st = None if start_t is None else np.ascontiguousarray(start_t, np.int32)
        lib().oracle_random_actions(self._h, seed & 0xFFFFFFFF, t & 0xFFFFFFFF, _p(st), _p(out))
        return out

    def legal_mask(self):
        out = np.empty((self.B, self.A), np.uint8)
        lib().oracle_legal_mask(self._h, _p(out))
        return out

    def observe(self):
        out = np.empty((self.B, self.N, self.N, 17), np.uint8)
        lib().oracle_observe(self._h, _p(out))
        return out

    def rewards(self):
        out = np.empty((self.B, 2), np.float32)
        lib().oracle_rewards(self._h, _p(out))
        return out

    def terminated(self):
        out = np.empty(self.B, np.uint8)
        lib().oracle_terminated(self._h, _p(out))
        return out

    def current_player(self):
        out = np.empty(self.B, np.uint8)
        lib().oracle_current_player(self._h, _p(out))
        return out

    def illegal_count(self):
        out = np.empty(self.B, np.uint32)
        lib().oracle_illegal_count(self._h, _p(out))
        return out

    def export_state(self):
        s = State(self.B, self.P)
        lib().oracle_export_state(self._h, *[_p(f) for f in s.fields()])
        return s

    def import_state(self, s):
        lib().oracle_import_state(self._h, *[_p(np.ascontiguousarray(f)) for f in s.fields()])


# ---- stand-alone rule functions on one board (int8 array of N*N cells, 0/+1/-1) ----
def legal_trial(board, N, to_play, ko=-1):
    b = np.ascontiguousarray(board, np.int8).reshape(-1)
    out = np.empty(N * N + 1, np.uint8)
    lib().oracle_legal_trial(_p(b), N, to_play, ko, _p(out))
    return out


def legal_chains(board, N, to_play, ko=-1):
    b = np.ascontiguousarray(board, np.int8).reshape(-1)
    out = np.empty(N * N + 1, np.uint8)
    lib().oracle_legal_chains(_p(b), N, to_play, ko, _p(out))
    return out


def area(board, N):
    b = np.ascontiguousarray(board, np.int8).reshape(-1)
    ab, aw = np.zeros(1, np.int32), np.zeros(1, np.int32)
    lib().oracle_area(_p(b), N, _p(ab), _p(aw))
    return int(ab[0]), int(aw[0])


def chain(board, N, p):
    b = np.ascontiguousarray(board, np.int8).reshape(-1)
    s, l = np.zeros(1, np.int32), np.zeros(1, np.int32)
    lib().oracle_chain(_p(b), N, int(p), _p(s), _p(l))
    return int(s[0]), int(l[0])
