"""The benchmark configurations against the numbers the paper prints (fixtures under tests/golden/)."""
import ast
import os

from paper_1907_03329_amd.synth import CONFIGS

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [[c.strip() for c in line.split("|")] for line in f if line.strip() and not line.startswith("#")]


def test_network_shapes_are_those_of_table_1():
    table = rows("table1_network_parameters.txt")
    assert len(table) == 3
    for frame, dilations, size in table:
        cfg = CONFIGS[frame]
        assert cfg.blocks == ast.literal_eval("(" + dilations + ")"), frame
        assert cfg.hidden == int(size), frame
    # the small configuration is the quarterly network on a small batch
    assert CONFIGS["tiny_quarterly"].blocks == CONFIGS["quarterly"].blocks
    assert CONFIGS["tiny_quarterly"].hidden == CONFIGS["quarterly"].hidden


def test_quarterly_series_length_is_the_papers_minimum_length():
    table = dict(rows("section5_2_minimum_series_length.txt"))
    assert CONFIGS["quarterly"].T == int(table["quarterly"])
    assert CONFIGS["tiny_quarterly"].T == int(table["quarterly"])
