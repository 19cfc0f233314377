"""Every environment and every ply of every benchmark configuration, HIP path against CPU oracle, bit for bit
(drawn actions, masks, observations, rewards, terminated flags every ply; exported state every 100 plies).
The oracle side runs on 16 host threads; the two largest cases take ~40 s each."""
import importlib.util
import os

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
spec = importlib.util.spec_from_file_location("full_parity", os.path.join(HERE, "full_parity.py"))
full_parity = importlib.util.module_from_spec(spec)
spec.loader.exec_module(full_parity)

EXPECTED = {("go", 0): 256 * 162, ("go", 1): 4096 * 1000, ("go", 2): 1024 * 722, ("go", 3): 16384 * 2000,
            ("hex", 0): 1024 * 122, ("hex", 1): 16384 * 1000, ("hex", 2): 262144 * 500}


@pytest.mark.parametrize("game,config", [("go", 0), ("go", 1), ("go", 2), ("go", 3), ("go", 4), ("hex", 0), ("hex", 1), ("hex", 2)])
def test_every_environment_every_ply(game, config):
    n = full_parity.run(full_parity.Args(game=game, config=config))
    if (game, config) in EXPECTED:
        assert n == EXPECTED[(game, config)]
    else:
        assert n > 65536 * 500          # configuration 4: 500 measured plies plus each game's own warm-up


@pytest.mark.parametrize("config,mapping", [(1, 2), (2, 1)])
def test_every_environment_every_ply_hex_in_the_other_mapping(config, mapping):
    """The largest Hex workload is stepped with a board per lane and the others with a board row per lane by default;
    here the other way round: 16384 games with a board per lane, 262144 with a board row per lane."""
    n = full_parity.run(full_parity.Args(game="hex", config=config, mapping=mapping))
    assert n == EXPECTED[("hex", config)]


@pytest.mark.parametrize("config,mode", [(1, 1), (2, 1), (3, 1), (1, 2), (2, 2), (3, 2)])
def test_every_environment_every_ply_with_superko(config, mode):
    """The same with the positional-superko rule on, enforced at play time (mode 1) and honoured by the legal mask (mode 2);
    the oracle keeps every position of every game literally, and in mode 2 tries every legal point of every ply against
    them, which bounds how many plies of the headline batch fit into the suite."""
    plies = (800 if mode == 1 else 400) if config == 3 else 0
    n = full_parity.run(full_parity.Args(game="go", config=config, superko=mode, plies=plies))
    assert n == (16384 * plies if config == 3 else EXPECTED[("go", config)])


@pytest.mark.parametrize("config", [1, 2])
def test_every_environment_every_ply_with_superko_through_the_rollout_kernel(config):
    """The rule proper through the rollout kernel, 8 plies per launch with every ply recorded in its own slice."""
    n = full_parity.run(full_parity.Args(game="go", config=config, superko=2, rollout=8))
    assert n == EXPECTED[("go", config)]


def test_every_environment_every_ply_hex_rollout_with_a_board_per_lane():
    """The Hex rollout kernel in the board-per-lane mapping, 8 plies per launch, every ply in its own slice."""
    n = full_parity.run(full_parity.Args(game="hex", config=1, rollout=8, mapping=2))
    assert n == EXPECTED[("hex", 1)]


@pytest.mark.parametrize("game,config", [("go", 1), ("go", 3), ("hex", 1)])
def test_every_environment_every_ply_through_the_rollout_kernel(game, config):
    """The rollout kernel, 8 plies per launch with every ply recorded in its own slice."""
    plies = 800 if (game, config) == ("go", 3) else 0
    n = full_parity.run(full_parity.Args(game=game, config=config, rollout=8, plies=plies))
    assert n == (16384 * 800 if plies else EXPECTED[(game, config)])


@pytest.mark.parametrize("config,rollout,plies", [(3, 0, 800), (2, 0, 0), (3, 8, 400)])
def test_every_environment_every_ply_with_line_padded_pitches(config, rollout, plies):
    """The layout bench.py --line-padded times: pitches of 6144 / 384 bytes, the pad bytes written as zeros; one launch per
    ply (the headline batch and a small one) and the rollout kernel with every ply in its own slice."""
    n = full_parity.run(full_parity.Args(game="go", config=config, rollout=rollout, plies=plies, line_padded=True))
    assert n > 0
