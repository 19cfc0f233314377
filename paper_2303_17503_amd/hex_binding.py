"""ctypes binding of the Hex entry points of libpgxgo.so; names follow include/pgxhex.h (pgxhex_<name> -> HexEnv.<name>)."""
import ctypes as C

import torch

from .binding import PgxGoError, _need, _ptr, lib as _golib

N, P, A, OBS = 11, 121, 122, 484
_ready = False


class _Opts(C.Structure):
    _fields_ = [("auto_reset", C.c_int32), ("stream", C.c_void_p)]


def lib():
    """The shared library with the pgxhex_* prototypes declared; raises if it has not been built (no fallback)."""
    global _ready
    L = _golib()
    if not _ready:
        vp, i32, u32 = C.c_void_p, C.c_int32, C.c_uint32
        L.pgxhex_state_bytes.restype = C.c_size_t
        L.pgxhex_state_bytes.argtypes = [i32]
        L.pgxhex_init.argtypes = [C.POINTER(vp), i32, u32, C.POINTER(_Opts), vp, C.c_size_t]
        L.pgxhex_destroy.argtypes = [vp]
        L.pgxhex_reset.argtypes = [vp]
        L.pgxhex_bind_outputs.argtypes = [vp, vp, vp, vp, vp]
        L.pgxhex_set_output_buffers.argtypes = [vp, vp, vp, vp, vp]
        L.pgxhex_step.argtypes = [vp, vp]
        L.pgxhex_random_actions.argtypes = [vp, u32, u32, vp, vp]
        L.pgxhex_step_sample.argtypes = [vp, vp, u32, u32, vp, vp]
        L.pgxhex_rollout.argtypes = [vp, i32, i32, u32, u32, vp, vp, vp, vp, vp, vp]
        for n in ("legal_mask", "observe", "rewards", "terminated", "current_player"):
            getattr(L, "pgxhex_" + n).argtypes = [vp, vp]
        L.pgxhex_export_state.argtypes = [vp] * 8
        L.pgxhex_import_state.argtypes = [vp] * 7
        L.pgxhex_sync.argtypes = [vp]
        L.pgxhex_set_mapping.argtypes = [vp, i32]
        L.pgxhex_boards_per_wavefront.restype = i32
        L.pgxhex_boards_per_wavefront.argtypes = []
        L.pgxhex_strerror.restype = C.c_char_p
        L.pgxhex_strerror.argtypes = [C.c_int]
        L.pgxhex_last_hip_error.restype = C.c_int
        _ready = True
    return L


def _check(rc, what):
    if rc != 0:
        L = lib()
        raise PgxGoError(f"{what}: {L.pgxhex_strerror(rc).decode()} (code {rc}, hip error {L.pgxhex_last_hip_error()})")


class HexEnv:
    """`batch` games of 11x11 Hex on one GPU (paper Fig. 2 API; Appendix C "Hex")."""

    N, P, A, OBS = N, P, A, OBS

    def __init__(self, batch, seed=0, auto_reset=False, device="cuda:0"):
        L = lib()
        self.B = int(batch)
        self.device = torch.device(device)
        nbytes = L.pgxhex_state_bytes(self.B)
        if nbytes == 0:
            raise PgxGoError("batch must be positive")
        with torch.cuda.device(self.device):
            self._state = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self._stream = torch.cuda.current_stream(self.device)
            opts = _Opts(int(bool(auto_reset)), C.c_void_p(self._stream.cuda_stream))
            h = C.c_void_p()
            _check(L.pgxhex_init(C.byref(h), self.B, seed & 0xFFFFFFFF, C.byref(opts), _ptr(self._state), nbytes), "pgxhex_init")
        self._h = h
        self.mask_out = self.obs_out = self.rewards_out = self.terminated_out = None

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and lib is not None:   # module globals are gone when the interpreter shuts down
            lib().pgxhex_destroy(h)

    def new_mask(self):
        return torch.empty((self.B, A), dtype=torch.uint8, device=self.device)

    def new_obs(self):
        return torch.empty((self.B, OBS), dtype=torch.uint8, device=self.device)

    def bind_outputs(self, mask=None, obs=None, rewards=None, terminated=None):
        if mask is not None: _need(mask, torch.uint8, (self.B, A), "mask")
        if obs is not None: _need(obs, torch.uint8, (self.B, OBS), "obs")
        if rewards is not None: _need(rewards, torch.float32, (self.B, 2), "rewards")
        if terminated is not None: _need(terminated, torch.uint8, (self.B,), "terminated")
        _check(lib().pgxhex_bind_outputs(self._h, _ptr(mask), _ptr(obs), _ptr(rewards), _ptr(terminated)), "pgxhex_bind_outputs")
        self.mask_out, self.obs_out, self.rewards_out, self.terminated_out = mask, obs, rewards, terminated

    def set_output_buffers(self, mask=None, obs=None, rewards=None, terminated=None):
        """Switch the buffers the step calls write to without emitting or copying anything (trajectory recording)."""
        if mask is not None: _need(mask, torch.uint8, (self.B, A), "mask")
        if obs is not None: _need(obs, torch.uint8, (self.B, OBS), "obs")
        if rewards is not None: _need(rewards, torch.float32, (self.B, 2), "rewards")
        if terminated is not None: _need(terminated, torch.uint8, (self.B,), "terminated")
        _check(lib().pgxhex_set_output_buffers(self._h, _ptr(mask), _ptr(obs), _ptr(rewards), _ptr(terminated)), "pgxhex_set_output_buffers")
        self.mask_out, self.obs_out, self.rewards_out, self.terminated_out = mask, obs, rewards, terminated

    def set_mapping(self, mapping=0):
        """Launch shape of the step kernels: 1 = a board row per lane, 2 = a board per lane, 0 = automatic; returns the one in use."""
        rc = lib().pgxhex_set_mapping(self._h, int(mapping))
        if rc <= 0:
            _check(rc if rc < 0 else -1, "pgxhex_set_mapping")
        return rc

    def reset(self):
        _check(lib().pgxhex_reset(self._h), "pgxhex_reset")

    def step(self, actions):
        _need(actions, torch.int32, (self.B,), "actions")
        _check(lib().pgxhex_step(self._h, _ptr(actions)), "pgxhex_step")

    def random_actions(self, seed, t, start_t=None, out=None):
        if out is None:
            out = torch.empty(self.B, dtype=torch.int32, device=self.device)
        _need(out, torch.int32, (self.B,), "actions")
        if start_t is not None: _need(start_t, torch.int32, (self.B,), "start_t")
        _check(lib().pgxhex_random_actions(self._h, seed & 0xFFFFFFFF, t & 0xFFFFFFFF, _ptr(start_t), _ptr(out)), "pgxhex_random_actions")
        return out

    def step_sample(self, actions, seed, t, start_t=None, out=None):
        _need(actions, torch.int32, (self.B,), "actions")
        if out is None:
            out = torch.empty(self.B, dtype=torch.int32, device=self.device)
        _need(out, torch.int32, (self.B,), "next_actions")
        if start_t is not None: _need(start_t, torch.int32, (self.B,), "start_t")
        _check(lib().pgxhex_step_sample(self._h, _ptr(actions), seed & 0xFFFFFFFF, t & 0xFFFFFFFF, _ptr(start_t), _ptr(out)), "pgxhex_step_sample")
        return out

    def rollout(self, steps, seed, t0, start_t=None, slices=1, actions=None, rewards=None, terminated=None, mask=None, obs=None):
        """`steps` plies of random legal play in one launch; ply i writes slice i % slices of the given buffers."""
        S = int(slices)
        if actions is not None: _need(actions, torch.int32, (S, self.B), "actions")
        if rewards is not None: _need(rewards, torch.float32, (S, self.B, 2), "rewards")
        if terminated is not None: _need(terminated, torch.uint8, (S, self.B), "terminated")
        if mask is not None: _need(mask, torch.uint8, (S, self.B, A), "mask")
        if obs is not None: _need(obs, torch.uint8, (S, self.B, OBS), "obs")
        if start_t is not None: _need(start_t, torch.int32, (self.B,), "start_t")
        _check(lib().pgxhex_rollout(self._h, int(steps), S, seed & 0xFFFFFFFF, t0 & 0xFFFFFFFF, _ptr(start_t), _ptr(actions), _ptr(rewards),
                                    _ptr(terminated), _ptr(mask), _ptr(obs)), "pgxhex_rollout")

    def _get(self, name, shape, dtype, out):
        out = torch.empty(shape, dtype=dtype, device=self.device) if out is None else _need(out, dtype, shape, name)
        _check(getattr(lib(), "pgxhex_" + name)(self._h, _ptr(out)), "pgxhex_" + name)
        return out

    def legal_mask(self, out=None):
        return self._get("legal_mask", (self.B, A), torch.uint8, out)

    def observe(self, out=None):
        return self._get("observe", (self.B, OBS), torch.uint8, out)

    def rewards(self, out=None):
        return self._get("rewards", (self.B, 2), torch.float32, out)

    def terminated(self, out=None):
        return self._get("terminated", (self.B,), torch.uint8, out)

    def current_player(self, out=None):
        return self._get("current_player", (self.B,), torch.uint8, out)

    def sync(self):
        _check(lib().pgxhex_sync(self._h), "pgxhex_sync")

    STATE_FIELDS = (("board", torch.int8), ("to_play", torch.int8), ("steps", torch.int32), ("terminated", torch.uint8),
                    ("black_player", torch.uint8), ("episode", torch.int32), ("illegal", torch.int32))

    def _state_shape(self, name):
        return (self.B, P) if name == "board" else (self.B,)

    def export_state(self):
        """dict of device tensors in the canonical layout of pgxhex_export_state."""
        out = {n: torch.empty(self._state_shape(n), dtype=dt, device=self.device) for n, dt in self.STATE_FIELDS}
        _check(lib().pgxhex_export_state(self._h, *[_ptr(out[n]) for n, _ in self.STATE_FIELDS]), "pgxhex_export_state")
        return out

    def import_state(self, st):
        args = [_ptr(_need(st[n], dt, self._state_shape(n), n)) for n, dt in self.STATE_FIELDS[:-1]]
        _check(lib().pgxhex_import_state(self._h, *args), "pgxhex_import_state")
