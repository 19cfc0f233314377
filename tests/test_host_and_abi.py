"""CPU-only checks of the boundary: the library loads, exports every declared symbol, and rejects bad arguments."""
import ctypes as C
import os
import re

import numpy as np

import oracle
import paper_2303_17503_amd as pg
import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="pgxgo.h", prefix="pgxgo_"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(" + prefix + r"[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 20 and "pgxgo_step" in names and "pgxgo_init" in names
    L = C.CDLL(pg.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n


def test_library_exports_every_declared_hex_symbol():
    names = declared_functions("pgxhex.h", "pgxhex_")
    assert len(names) >= 18 and "pgxhex_step" in names and "pgxhex_init" in names and "pgxhex_step_sample" in names
    L = C.CDLL(pg.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n


def test_hex_argument_errors_need_no_gpu():
    from paper_2303_17503_amd import hex_binding
    L = hex_binding.lib()
    h = C.c_void_p()
    assert L.pgxhex_boards_per_wavefront() == 5
    assert L.pgxhex_state_bytes(0) == 0 and L.pgxhex_state_bytes(-3) == 0
    b1, b2 = L.pgxhex_state_bytes(1000), L.pgxhex_state_bytes(2000)
    assert 1000 * (11 * 4 + 16 + 8 + 1) <= b1 < b2 < 2 * b1 + 4096
    assert L.pgxhex_init(C.byref(h), 4, 0, None, None, 0) == -1                      # null state buffer
    assert L.pgxhex_init(C.byref(h), 0, 0, None, C.c_void_p(256), 1 << 20) == -1     # batch
    assert L.pgxhex_init(C.byref(h), 4, 0, None, C.c_void_p(256), 16) == -1          # buffer too small
    assert L.pgxhex_init(C.byref(h), 4, 0, None, C.c_void_p(260), 1 << 20) == -1     # misaligned
    assert L.pgxhex_init(None, 4, 0, None, C.c_void_p(256), 1 << 20) == -1
    assert L.pgxhex_step(None, None) == -1 and L.pgxhex_destroy(None) == -1 and L.pgxhex_step_sample(None, None, 0, 0, None, None) == -1
    assert L.pgxhex_strerror(-1) == b"invalid argument" and L.pgxhex_strerror(0) == b"ok"
    header = open(os.path.join(ROOT, "include", "pgxhex.h")).read()
    assert "#define PGXHEX_ACTIONS 122" in header and "#define PGXHEX_OBS_BYTES 484" in header   # Table 1


def test_size_queries_match_the_paper_tables():
    L = pg.lib()
    assert L.pgxgo_num_actions(9) == 82 and L.pgxgo_num_actions(19) == 362          # Table 1
    assert L.pgxgo_obs_bytes(9) == 9 * 9 * 17 and L.pgxgo_obs_bytes(19) == 19 * 19 * 17
    assert L.pgxgo_num_actions(13) == 0 and L.pgxgo_boards_per_wavefront(13) == 0
    assert L.pgxgo_boards_per_wavefront(19) == 3 and L.pgxgo_boards_per_wavefront(9) == 6
    assert L.pgxgo_state_bytes(0, 19) == 0 and L.pgxgo_state_bytes(4, 7) == 0
    b1, b2 = L.pgxgo_state_bytes(1000, 19), L.pgxgo_state_bytes(2000, 19)
    assert 0 < b1 < b2 < 2 * b1 + 4096


def test_argument_errors_need_no_gpu():
    L = pg.lib()
    h = C.c_void_p()
    assert L.pgxgo_init(C.byref(h), 4, 19, 0, None, None, 0) == -1          # null state buffer
    assert L.pgxgo_init(C.byref(h), 4, 13, 0, None, C.c_void_p(256), 1 << 20) == -1   # board size
    assert L.pgxgo_init(C.byref(h), 0, 19, 0, None, C.c_void_p(256), 1 << 20) == -1   # batch
    assert L.pgxgo_init(C.byref(h), 4, 19, 0, None, C.c_void_p(256), 16) == -1         # buffer too small
    assert L.pgxgo_init(C.byref(h), 4, 19, 0, None, C.c_void_p(260), 1 << 20) == -1   # misaligned
    assert L.pgxgo_init(None, 4, 19, 0, None, C.c_void_p(256), 1 << 20) == -1
    assert L.pgxgo_step(None, None) == -1 and L.pgxgo_destroy(None) == -1
    assert L.pgxgo_strerror(-1) == b"invalid argument" and L.pgxgo_strerror(0) == b"ok"


def test_workload_hash_matches_oracle_hash():
    ids = np.array([0, 1, 2, 777, 65535])
    for seed, tag, t in ((4, 2, 0), (0, 0, 5), (3, 1, 1999)):
        got = workloads.counter_hash(seed, tag, ids, t)
        assert got.tolist() == [oracle.hash4(seed, tag, int(e), t) for e in ids]
    st = workloads.start_times(workloads.CONFIGS[4])
    assert st.shape == (65536,) and st.min() == 0 and st.max() == 300
    assert abs(st.mean() - 150) < 2
    assert workloads.start_times(workloads.CONFIGS[3]) is None


def test_superko_entry_points_and_key_table():
    L = pg.lib()
    assert L.pgxgo_superko_bytes(0, 19) == 0 and L.pgxgo_superko_bytes(4, 13) == 0
    assert L.pgxgo_superko_bytes(100, 19) >= 100 * (2048 * 8 + 8) and L.pgxgo_superko_bytes(100, 9) >= 100 * (512 * 8 + 8)
    assert L.pgxgo_enable_superko(None, 2, None, 0) == -1
    # the position keys are one 64-bit word per (point, colour); their low halves must all differ, or two stones could cancel
    M = 0xFFFFFFFF

    def mix(x):
        x ^= x >> 16; x = (x * 0x7feb352d) & M
        x ^= x >> 15; x = (x * 0x846ca68b) & M
        return x ^ (x >> 16)

    lows = [mix((0x9E3779B9 * (2 * p + c + 1)) & M) for p in range(361) for c in range(2)]
    assert len(set(lows)) == 722 and 0 not in lows
