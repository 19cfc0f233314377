"""ctypes front end of the CPU Hex oracle (oracle/hex_oracle.cpp).

TEST INFRASTRUCTURE: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this module.  It never touches the HIP library.  All arrays are host numpy arrays.
"""
import ctypes as C

import numpy as np

from .build import build_hex as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build(force=False))
        L.hexo_create.restype = C.c_void_p
        L.hexo_create.argtypes = [C.c_int, C.c_int, C.c_uint32, C.c_int, C.c_void_p]
        L.hexo_destroy.argtypes = [C.c_void_p]
        L.hexo_reset.argtypes = [C.c_void_p]
        L.hexo_step.argtypes = [C.c_void_p, C.c_void_p]
        L.hexo_random_actions.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]
        L.hexo_hash.restype = C.c_uint32
        L.hexo_hash.argtypes = [C.c_uint32] * 4
        for name in ("legal_mask", "observe", "rewards", "terminated", "current_player", "illegal_count"):
            getattr(L, "hexo_" + name).argtypes = [C.c_void_p, C.c_void_p]
        L.hexo_export_state.argtypes = [C.c_void_p] * 7
        L.hexo_import_state.argtypes = [C.c_void_p] * 7
        L.hexo_joined.restype = C.c_int
        L.hexo_joined.argtypes = [C.c_void_p, C.c_int, C.c_int]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class HexState:
    """Canonical per-environment state arrays (host)."""

    __slots__ = ("board", "to_play", "steps", "terminated", "black_player", "episode")

    def __init__(self, B, P):
        self.board = np.zeros((B, P), np.int8)
        self.to_play = np.zeros(B, np.int8)
        self.steps = np.zeros(B, np.int32)
        self.terminated = np.zeros(B, np.uint8)
        self.black_player = np.zeros(B, np.uint8)
        self.episode = np.zeros(B, np.uint32)

    def fields(self):
        return [getattr(self, k) for k in self.__slots__]


class HexOracle:
    """Batched Hex environment on the CPU (paper Fig. 2 API; Appendix C "Hex")."""

    def __init__(self, batch, board_size=11, seed=0, auto_reset=False, env_ids=None):
        self.B, self.N = int(batch), int(board_size)
        self.P = self.N * self.N
        self.A = self.P + 1
        ids = None if env_ids is None else np.ascontiguousarray(env_ids, np.int32)
        self._h = lib().hexo_create(self.B, self.N, seed & 0xFFFFFFFF, int(auto_reset), _p(ids))
        if not self._h:
            raise ValueError("hexo_create rejected its arguments")

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and lib is not None:   # module globals are gone when the interpreter shuts down
            lib().hexo_destroy(h)

    def reset(self):
        lib().hexo_reset(self._h)

    def step(self, actions):
        a = np.ascontiguousarray(actions, np.int32)
        assert a.shape == (self.B,)
        lib().hexo_step(self._h, _p(a))

    def random_actions(self, seed, t, start_t=None):
        out = np.empty(self.B, np.int32)
        st = None if start_t is None else np.ascontiguousarray(start_t, np.int32)
        lib().hexo_random_actions(self._h, seed & 0xFFFFFFFF, t & 0xFFFFFFFF, _p(st), _p(out))
        return out

    def _get(self, name, shape, dtype):
        out = np.empty(shape, dtype)
        getattr(lib(), "hexo_" + name)(self._h, _p(out))
        return out

    def legal_mask(self):
        return self._get("legal_mask", (self.B, self.A), np.uint8)

    def observe(self):
        return self._get("observe", (self.B, self.N, self.N, 4), np.uint8)

    def rewards(self):
        return self._get("rewards", (self.B, 2), np.float32)

    def terminated(self):
        return self._get("terminated", self.B, np.uint8)

    def current_player(self):
        return self._get("current_player", self.B, np.uint8)

    def illegal_count(self):
        return self._get("illegal_count", self.B, np.uint32)

    def export_state(self):
        s = HexState(self.B, self.P)
        lib().hexo_export_state(self._h, *[_p(f) for f in s.fields()])
        return s

    def import_state(self, s):
        lib().hexo_import_state(self._h, *[_p(np.ascontiguousarray(f)) for f in s.fields()])


def joined(board, N, col):
    """Has colour col (+1 black: top-bottom, -1 white: left-right) joined its sides on this int8 board?"""
    b = np.ascontiguousarray(board, np.int8).reshape(-1)
    return bool(lib().hexo_joined(_p(b), N, col))


def hash4(seed, tag, env, t):
    return int(lib().hexo_hash(seed & 0xFFFFFFFF, tag & 0xFFFFFFFF, env & 0xFFFFFFFF, t & 0xFFFFFFFF))
