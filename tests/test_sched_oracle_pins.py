"""Pins of the schedule reference (oracle/sched_oracle.py) against hand-worked lists and counts."""
from oracle import sched_oracle as so


def test_config1_by_hand():
    lengths = [1, 7, 64, 184]                      # configuration 1
    # tile 64: 1, 1, 1 and 3 tiles; the 184-token sequence contributes levels 3, 2, 1
    assert so.items(lengths, 64) == [(3, 3), (3, 2), (0, 1), (1, 1), (2, 1), (3, 1)]
    assert so.records(lengths, 64) == [(3, 3, 72, 184), (3, 2, 72, 184), (0, 1, 0, 1), (1, 1, 1, 7), (2, 1, 8, 64), (3, 1, 72, 184)]
    assert so.total_cost(lengths, 64) == 1 + 1 + 1 + 6
    # tile 128: the last sequence has two tiles; tile 256: one item per sequence
    assert so.items(lengths, 128) == [(3, 2), (0, 1), (1, 1), (2, 1), (3, 1)]
    assert so.items(lengths, 256) == [(0, 1), (1, 1), (2, 1), (3, 1)]


def test_empty_and_boundary_lengths():
    assert so.items([0, 128, 129, 0], 128) == [(2, 2), (1, 1), (2, 1)]
    assert so.items([], 64) == [] and so.items([0], 64) == []
    # counts: sum of ceil(L / tile); cost: triangular numbers
    lengths = [300, 5, 1000]
    assert len(so.items(lengths, 256)) == 2 + 1 + 4
    assert so.total_cost(lengths, 256) == 3 + 1 + 10
    levels = [c for _, c in so.items(lengths, 256)]
    assert levels == sorted(levels, reverse=True) == [4, 3, 2, 2, 1, 1, 1]
