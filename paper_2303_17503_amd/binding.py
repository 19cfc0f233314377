"""ctypes binding of libpgxgo.so; names follow include/pgxgo.h (pgxgo_<name> -> GoEnv.<name>)."""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("PGXGO_LIB") or os.path.join(HERE, "libpgxgo.so")   # PGXGO_LIB: load another build of the same library

_lib = None


class PgxGoError(RuntimeError):
    pass


class _Opts(C.Structure):
    _fields_ = [("komi_x2", C.c_int32), ("max_steps", C.c_int32), ("auto_reset", C.c_int32),
                ("obs_pitch", C.c_int32), ("mask_pitch", C.c_int32), ("stream", C.c_void_p)]


def lib():
    """Loads the HIP library; raises if it has not been built (no fallback of any kind)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise PgxGoError(f"{LIB_PATH} is missing: build it with `python paper_2303_17503_amd/build.py` "
                             "(or __graft_entry__.build()); there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        vp, i32, u32 = C.c_void_p, C.c_int32, C.c_uint32
        L.pgxgo_state_bytes.restype = C.c_size_t
        L.pgxgo_state_bytes.argtypes = [i32, i32]
        L.pgxgo_init.argtypes = [C.POINTER(vp), i32, i32, u32, C.POINTER(_Opts), vp, C.c_size_t]
        L.pgxgo_init_static.argtypes = [C.POINTER(vp), i32, i32, u32, C.POINTER(_Opts)]
        L.pgxgo_destroy.argtypes = [vp]
        L.pgxgo_reset.argtypes = [vp]
        L.pgxgo_bind_outputs.argtypes = [vp, vp, vp, vp, vp]
        L.pgxgo_set_output_buffers.argtypes = [vp, vp, vp, vp, vp]
        L.pgxgo_emit.argtypes = [vp, vp, vp]
        L.pgxgo_fill_probe.argtypes = [vp, C.c_size_t, u32, i32, vp]
        L.pgxgo_empty_probe.argtypes = [vp, i32]
        L.pgxgo_step.argtypes = [vp, vp]
        L.pgxgo_random_actions.argtypes = [vp, u32, u32, vp, vp]
        L.pgxgo_step_sample.argtypes = [vp, vp, u32, u32, vp, vp]
        L.pgxgo_rollout.argtypes = [vp, i32, i32, u32, u32, vp, vp, vp, vp, vp, vp]
        L.pgxgo_step_slots.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp]
        L.pgxgo_copy_slots.argtypes = [vp, i32, vp, vp]
        for n in ("legal_mask", "observe", "rewards", "terminated", "current_player"):
            getattr(L, "pgxgo_" + n).argtypes = [vp, vp]
        L.pgxgo_export_state.argtypes = [vp] * 11
        L.pgxgo_import_state.argtypes = [vp] * 10
        L.pgxgo_sync.argtypes = [vp]
        L.pgxgo_set_boards_per_wavefront.argtypes = [vp, i32]
        L.pgxgo_superko_bytes.restype = C.c_size_t
        L.pgxgo_superko_bytes.argtypes = [i32, i32]
        L.pgxgo_enable_superko.argtypes = [vp, i32, vp, C.c_size_t]
        for n in ("boards_per_wavefront", "num_actions", "obs_bytes"):
            getattr(L, "pgxgo_" + n).argtypes = [i32]
            getattr(L, "pgxgo_" + n).restype = i32
        L.pgxgo_strerror.restype = C.c_char_p
        L.pgxgo_strerror.argtypes = [C.c_int]
        L.pgxgo_last_hip_error.restype = C.c_int
        L.pgxgo_lane_shift_probe.argtypes = [vp, vp, vp]
        _lib = L
    return _lib


def _check(rc, what):
    if rc != 0:
        L = lib()
        raise PgxGoError(f"{what}: {L.pgxgo_strerror(rc).decode()} (code {rc}, hip error {L.pgxgo_last_hip_error()})")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _need(t, dtype, shape, name):
    if t.dtype != dtype or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise PgxGoError(f"{name}: expected contiguous cuda {dtype} tensor of shape {tuple(shape)}, got {t.dtype} {tuple(t.shape)} on {t.device}")
    return t


class GoEnv:
    """`batch` Go games on one GPU (paper Fig. 2 API)."""

    def __init__(self, batch, board_size, seed=0, komi_x2=15, max_steps=0, auto_reset=False, obs_pitch=0, mask_pitch=0,
                 device="cuda:0", static_state=False, line_padded=False):
        """line_padded: use the pitches at which every environment's mask and observation start on a 128-byte line
        (N*N+1 and N*N*17 rounded up to multiples of 128; the pad bytes are written as zeros).  Outputs that have to
        reach DRAM, such as recorded trajectories, are written faster in this layout; mask_view / obs_view give the
        [B][N*N+1] and [B][N][N][17] views."""
        L = lib()
        self.B, self.N = int(batch), int(board_size)
        self.P = self.N * self.N
        self.A = self.P + 1
        if line_padded:
            obs_pitch, mask_pitch = (self.P * 17 + 127) // 128 * 128, (self.A + 127) // 128 * 128
        self.device = torch.device(device)
        nbytes = L.pgxgo_state_bytes(self.B, self.N)
        if nbytes == 0:
            raise PgxGoError("unsupported batch or board size (board_size must be 9 or 19, batch > 0)")
        self.obs_pitch = int(obs_pitch) or self.P * 17
        self.mask_pitch = int(mask_pitch) or self.A
        with torch.cuda.device(self.device):
            self._stream = torch.cuda.current_stream(self.device)
            opts = _Opts(int(komi_x2), int(max_steps), int(bool(auto_reset)), int(obs_pitch), int(mask_pitch),
                         C.c_void_p(self._stream.cuda_stream))
            h = C.c_void_p()
            if static_state:     # pgxgo_init_static: the state lives in the library's own static buffer, nothing is allocated
                self._state = None
                _check(L.pgxgo_init_static(C.byref(h), self.B, self.N, seed & 0xFFFFFFFF, C.byref(opts)), "pgxgo_init_static")
            else:
                self._state = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
                _check(L.pgxgo_init(C.byref(h), self.B, self.N, seed & 0xFFFFFFFF, C.byref(opts), _ptr(self._state), nbytes), "pgxgo_init")
        self._h = h
        self.mask_out = self.obs_out = self.rewards_out = self.terminated_out = None

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and lib is not None:   # module globals are gone when the interpreter shuts down
            lib().pgxgo_destroy(h)

    # ---- buffers -------------------------------------------------------------------------------------
    def new_mask(self):
        return torch.empty((self.B, self.mask_pitch), dtype=torch.uint8, device=self.device)

    def new_obs(self):
        return torch.empty((self.B, self.obs_pitch), dtype=torch.uint8, device=self.device)

    def mask_view(self, t):
        return t[:, : self.A]

    def obs_view(self, t):
        """[B][N][N][17] view of an observation buffer (strided when the pitch is padded; no copy)."""
        return t.as_strided((t.shape[0], self.N, self.N, 17), (self.obs_pitch, self.N * 17, 17, 1), t.storage_offset())

    def bind_outputs(self, mask=None, obs=None, rewards=None, terminated=None):
        if mask is not None: _need(mask, torch.uint8, (self.B, self.mask_pitch), "mask")
        if obs is not None: _need(obs, torch.uint8, (self.B, self.obs_pitch), "obs")
        if rewards is not None: _need(rewards, torch.float32, (self.B, 2), "rewards")
        if terminated is not None: _need(terminated, torch.uint8, (self.B,), "terminated")
        _check(lib().pgxgo_bind_outputs(self._h, _ptr(mask), _ptr(obs), _ptr(rewards), _ptr(terminated)), "pgxgo_bind_outputs")
        self.mask_out, self.obs_out, self.rewards_out, self.terminated_out = mask, obs, rewards, terminated

    def set_output_buffers(self, mask=None, obs=None, rewards=None, terminated=None):
        """Switch the buffers step() writes to without emitting or copying anything (trajectory recording)."""
        if mask is not None: _need(mask, torch.uint8, (self.B, self.mask_pitch), "mask")
        if obs is not None: _need(obs, torch.uint8, (self.B, self.obs_pitch), "obs")
        if rewards is not None: _need(rewards, torch.float32, (self.B, 2), "rewards")
        if terminated is not None: _need(terminated, torch.uint8, (self.B,), "terminated")
        _check(lib().pgxgo_set_output_buffers(self._h, _ptr(mask), _ptr(obs), _ptr(rewards), _ptr(terminated)), "pgxgo_set_output_buffers")
        self.mask_out, self.obs_out, self.rewards_out, self.terminated_out = mask, obs, rewards, terminated

    def emit(self, mask=None, obs=None):
        """Legal mask and observation of the current state in one launch."""
        if mask is not None: _need(mask, torch.uint8, (self.B, self.mask_pitch), "mask")
        if obs is not None: _need(obs, torch.uint8, (self.B, self.obs_pitch), "obs")
        _check(lib().pgxgo_emit(self._h, _ptr(mask), _ptr(obs)), "pgxgo_emit")

    # ---- the environment API ------------------------------------------------------------------------------
    def reset(self):
        _check(lib().pgxgo_reset(self._h), "pgxgo_reset")

    def step(self, actions):
        _need(actions, torch.int32, (self.B,), "actions")
        _check(lib().pgxgo_step(self._h, _ptr(actions)), "pgxgo_step")

    def random_actions(self, seed, t, start_t=None, out=None):
        if out is None:
            out = torch.empty(self.B, dtype=torch.int32, device=self.device)
        _need(out, torch.int32, (self.B,), "actions")
        if start_t is not None: _need(start_t, torch.int32, (self.B,), "start_t")
        _check(lib().pgxgo_random_actions(self._h, seed & 0xFFFFFFFF, t & 0xFFFFFFFF, _ptr(start_t), _ptr(out)), "pgxgo_random_actions")
        return out

    def step_sample(self, actions, seed, t, start_t=None, out=None):
        _need(actions, torch.int32, (self.B,), "actions")
        if out is None:
            out = torch.empty(self.B, dtype=torch.int32, device=self.device)
        _need(out, torch.int32, (self.B,), "next_actions")
        if start_t is not None: _need(start_t, torch.int32, (self.B,), "start_t")
        _check(lib().pgxgo_step_sample(self._h, _ptr(actions), seed & 0xFFFFFFFF, t & 0xFFFFFFFF, _ptr(start_t), _ptr(out)), "pgxgo_step_sample")
        return out

    def rollout(self, steps, seed, t0, start_t=None, slices=1, actions=None, rewards=None, terminated=None, mask=None, obs=None):
        """`steps` plies of random legal play in one launch; ply i writes slice i % slices of the given buffers."""
        S = int(slices)
        if actions is not None: _need(actions, torch.int32, (S, self.B), "actions")
        if rewards is not None: _need(rewards, torch.float32, (S, self.B, 2), "rewards")
        if terminated is not None: _need(terminated, torch.uint8, (S, self.B), "terminated")
        if mask is not None: _need(mask, torch.uint8, (S, self.B, self.mask_pitch), "mask")
        if obs is not None: _need(obs, torch.uint8, (S, self.B, self.obs_pitch), "obs")
        if start_t is not None: _need(start_t, torch.int32, (self.B,), "start_t")
        _check(lib().pgxgo_rollout(self._h, int(steps), S, seed & 0xFFFFFFFF, t0 & 0xFFFFFFFF, _ptr(start_t), _ptr(actions), _ptr(rewards),
                                   _ptr(terminated), _ptr(mask), _ptr(obs)), "pgxgo_rollout")

    def step_slots(self, src, actions, dst, mask=None, obs=None, rewards=None, terminated=None):
        """state[dst[i]] = step(state[src[i]], actions[i]); outputs of entry i in row i of the optional buffers."""
        n = int(src.shape[0])
        _need(src, torch.int32, (n,), "src"); _need(dst, torch.int32, (n,), "dst")
        if actions is not None: _need(actions, torch.int32, (n,), "actions")
        if mask is not None: _need(mask, torch.uint8, (n, self.mask_pitch), "mask")
        if obs is not None: _need(obs, torch.uint8, (n, self.obs_pitch), "obs")
        if rewards is not None: _need(rewards, torch.float32, (n, 2), "rewards")
        if terminated is not None: _need(terminated, torch.uint8, (n,), "terminated")
        _check(lib().pgxgo_step_slots(self._h, n, _ptr(src), _ptr(actions), _ptr(dst), _ptr(mask), _ptr(obs), _ptr(rewards), _ptr(terminated)),
               "pgxgo_step_slots")

    def copy_slots(self, src, dst):
        n = int(src.shape[0])
        _need(src, torch.int32, (n,), "src"); _need(dst, torch.int32, (n,), "dst")
        _check(lib().pgxgo_copy_slots(self._h, n, _ptr(src), _ptr(dst)), "pgxgo_copy_slots")

    def legal_mask(self, out=None):
        out = self.new_mask() if out is None else _need(out, torch.uint8, (self.B, self.mask_pitch), "mask")
        _check(lib().pgxgo_legal_mask(self._h, _ptr(out)), "pgxgo_legal_mask")
        return out

    def observe(self, out=None):
        out = self.new_obs() if out is None else _need(out, torch.uint8, (self.B, self.obs_pitch), "obs")
        _check(lib().pgxgo_observe(self._h, _ptr(out)), "pgxgo_observe")
        return out

    def rewards(self, out=None):
        out = torch.empty((self.B, 2), dtype=torch.float32, device=self.device) if out is None else _need(out, torch.float32, (self.B, 2), "rewards")
        _check(lib().pgxgo_rewards(self._h, _ptr(out)), "pgxgo_rewards")
        return out

    def terminated(self, out=None):
        out = torch.empty(self.B, dtype=torch.uint8, device=self.device) if out is None else _need(out, torch.uint8, (self.B,), "terminated")
        _check(lib().pgxgo_terminated(self._h, _ptr(out)), "pgxgo_terminated")
        return out

    def current_player(self, out=None):
        out = torch.empty(self.B, dtype=torch.uint8, device=self.device) if out is None else _need(out, torch.uint8, (self.B,), "current_player")
        _check(lib().pgxgo_current_player(self._h, _ptr(out)), "pgxgo_current_player")
        return out

    def sync(self):
        _check(lib().pgxgo_sync(self._h), "pgxgo_sync")

    def set_boards_per_wavefront(self, boards=0):
        """Launch-shape knob of the step and rollout kernels (0 = automatic); returns the value in use."""
        rc = lib().pgxgo_set_boards_per_wavefront(self._h, int(boards))
        if rc <= 0:
            _check(rc if rc < 0 else -1, "pgxgo_set_boards_per_wavefront")
        return rc

    def enable_superko(self, mode=1):
        """Positional superko.  "mask" / 2: the rule proper, the legal mask leaves out every play that would recreate an
        earlier position of the game.  True / 1: looked at only when the move is played (the offender loses), the mask
        keeps showing the simple-ko set.  False / 0: off."""
        mode = 2 if mode == "mask" else int(mode)
        if mode == 0:
            _check(lib().pgxgo_enable_superko(self._h, 0, None, 0), "pgxgo_enable_superko")
            self._superko = None
            return
        nbytes = lib().pgxgo_superko_bytes(self.B, self.N)
        self._superko = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        _check(lib().pgxgo_enable_superko(self._h, mode, _ptr(self._superko), nbytes), "pgxgo_enable_superko")

    # ---- canonical state ------------------------------------------------------------------------------------
    STATE_FIELDS = (("board", torch.int8), ("history", torch.int8), ("ko", torch.int32), ("to_play", torch.int8),
                    ("steps", torch.int32), ("passes", torch.int8), ("terminated", torch.uint8), ("black_player", torch.uint8),
                    ("episode", torch.int32), ("illegal", torch.int32))

    def _state_shape(self, name):
        return {"board": (self.B, self.P), "history": (self.B, 8, self.P)}.get(name, (self.B,))

    def export_state(self):
        """dict of device tensors in the canonical layout of pgxgo_export_state."""
        out = {n: torch.empty(self._state_shape(n), dtype=dt, device=self.device) for n, dt in self.STATE_FIELDS}
        _check(lib().pgxgo_export_state(self._h, *[_ptr(out[n]) for n, _ in self.STATE_FIELDS]), "pgxgo_export_state")
        return out

    def import_state(self, st):
        args = []
        for n, dt in self.STATE_FIELDS[:-1]:
            args.append(_ptr(_need(st[n], dt, self._state_shape(n), n)))
        _check(lib().pgxgo_import_state(self._h, *args), "pgxgo_import_state")


def fill_probe(dst, value=0, kind=2):
    """One fill of the uint8 cuda tensor `dst` (16-byte aligned, size a multiple of 16) with 16-byte stores; kind: 0 ordinary,
    1 non-temporal, 2 written through the L2."""
    _check(lib().pgxgo_fill_probe(_ptr(dst), dst.numel() * dst.element_size(), value & 0xFFFFFFFF, int(kind),
                                  C.c_void_p(torch.cuda.current_stream().cuda_stream)), "pgxgo_fill_probe")


def empty_probe(count=1):
    """`count` back-to-back launches of an empty kernel on the current stream, enqueued by one C loop."""
    _check(lib().pgxgo_empty_probe(C.c_void_p(torch.cuda.current_stream().cuda_stream), int(count)), "pgxgo_empty_probe")


def lane_shift_probe(values):
    """values: int32 cuda tensor [64] -> (from lane below, from lane above)."""
    out = torch.empty(128, dtype=torch.int32, device=values.device)
    _check(lib().pgxgo_lane_shift_probe(_ptr(values), _ptr(out), C.c_void_p(torch.cuda.current_stream().cuda_stream)), "pgxgo_lane_shift_probe")
    return out[:64], out[64:]
