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
