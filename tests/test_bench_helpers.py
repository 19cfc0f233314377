"""CPU checks of the benchmark's byte model and of the workload table."""
import bench
import workloads


def test_algorithmic_bytes_per_ply():
    # 4 action + 644 older positions + 24 scalars + 92 new position + 362 mask + 6137 observation + 9 rewards/terminated
    assert bench.algorithmic_bytes_per_ply(19, True) == 7272
    assert bench.algorithmic_bytes_per_ply(19, False) == 583
    assert bench.algorithmic_bytes_per_ply(9, True) == 1672
    assert bench.algorithmic_bytes_per_ply(9, False) == 163


def test_workload_table_matches_the_five_configurations():
    c = workloads.CONFIGS
    assert [(x.board_size, x.batch, x.seed, x.auto_reset, x.steps) for x in c] == [
        (9, 256, 0, False, 162), (9, 4096, 1, True, 1000), (19, 1024, 2, False, 722), (19, 16384, 3, True, 2000), (19, 65536, 4, True, 500)]
    assert c[4].warmup_max == 300 and all(x.komi_x2 == 15 for x in c)


def test_hex_bytes_per_ply():
    # 4 action + 32 position read + 24 scalars + 32 position written + 122 mask + 484 observation + 9 rewards/terminated
    assert bench.hex_bytes_per_ply(True) == 707
    assert bench.hex_bytes_per_ply(False) == 223
    h = workloads.HEX_CONFIGS
    assert [(x.board_size, x.batch, x.game) for x in h] == [(11, 1024, "hex"), (11, 16384, "hex"), (11, 262144, "hex")]


def test_more_than_one_gpu_is_refused():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, bench.__file__, "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout == ""


def test_rotation_and_default_steps():
    go3 = 16384 * (362 + 361 * 17)
    assert bench.rotation_slices(go3) == 8 and bench.rotation_slices(4 * go3) == 2 and bench.rotation_slices(100) == 8
    assert bench.rotation_slices(go3) * go3 > 3 * bench.MEMORY_SIDE_CACHE          # a rotation writes far beyond the memory-side cache
    c = workloads.CONFIGS
    assert bench.default_steps(c[3]) == 2000 and bench.default_steps(c[1]) == 1000 and bench.default_steps(c[4]) == 500
    for cfg in (c[0], c[2], workloads.HEX_CONFIGS[0]):                                # without auto-reset the timed windows end before the games do
        assert cfg.warmup_max + cfg.preroll + 20 + 2 * bench.default_steps(cfg) <= cfg.steps
    assert c[3].preroll >= 600 and c[4].warmup_max == 300                           # the timed plies lie in the dense regime


def test_bound_statement_rule():
    assert bench.bound_statement(6.0, 5.0, 1.0, 0.1)["bound_by"].startswith("launch gap")
    assert bench.bound_statement(22.0, 5.5, 17.0, 5.3)["bound_by"].startswith("hbm")
    assert bench.bound_statement(40.0, 5.0, 23.0, 51.0)["bound_by"] == "valu issue"
