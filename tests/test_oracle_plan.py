"""Pins of the oracle's control logic: which stages rebuild a lost stage
(Algorithm 1; section "CheckFree+: First and Last Stage Recovery"; the paper's
comparison table and limitations paragraph) and the CheckFree+ execution order."""
import itertools
import os

import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "plus_stage_orders.txt")


def golden_orders():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        s, std, swp = (part.split() for part in line.split("|"))
        rows.append((int(s[0]), [int(x) for x in std], [int(x) for x in swp]))
    return rows


@pytest.mark.parametrize("s,standard,exchanged", golden_orders())
def test_orders_printed_in_the_paper(s, standard, exchanged):
    # the paper numbers stages from 1
    assert [p + 1 for p in oracle.plus_stage_order(s, 0)] == standard
    assert [p + 1 for p in oracle.plus_stage_order(s, 1)] == exchanged


@pytest.mark.parametrize("s", [4, 5, 8, 13])
def test_order_properties(s):
    for mb in range(6):
        order = oracle.plus_stage_order(s, mb)
        assert sorted(order) == list(range(s))                      # every stage runs once
        assert order[2:s - 2] == list(range(2, s - 2))              # the middle never moves
    # over any two consecutive microbatches the second stage stands in the first one's place once,
    # and the second to last in the last one's place once: "half the time they take their places"
    for mb in range(5):
        a, b = oracle.plus_stage_order(s, mb), oracle.plus_stage_order(s, mb + 1)
        assert sorted([a[0], b[0]]) == [0, 1] and sorted([a[1], b[1]]) == [0, 1]
        assert sorted([a[-1], b[-1]]) == [s - 2, s - 1] and sorted([a[-2], b[-2]]) == [s - 2, s - 1]


def test_order_needs_four_different_stages():
    for s in (0, 1, 2, 3):
        with pytest.raises(IndexError):
            oracle.plus_stage_order(s, 1)


def test_intermediate_stage_takes_both_neighbours():
    # Algorithm 1: stage i receives W_{i-1}, omega_{i-1}, W_{i+1}, omega_{i+1}
    for s in (3, 4, 8):
        for i in range(1, s - 1):
            assert oracle.recovery_plan(s, [i]) == [("average", i - 1, i + 1)]
            assert oracle.recovery_plan(s, [i], plus=True) == [("average", i - 1, i + 1)]


def test_end_stages_only_with_checkfree_plus():
    for s in (2, 3, 8):
        for i in (0, s - 1):
            with pytest.raises(ValueError):
                oracle.recovery_plan(s, [i])
        assert oracle.recovery_plan(s, [0], plus=True) == [("copy", 1)]              # first <- second
        assert oracle.recovery_plan(s, [s - 1], plus=True) == [("copy", s - 2)]      # last <- second to last


def test_the_comparison_table_rows():
    # "non-consecutive stages: yes" / "consecutive stages: no", for both methods
    s = 8
    for plus in (False, True):
        assert oracle.recovery_plan(s, [2, 4, 6], plus) == [("average", 1, 3), ("average", 3, 5), ("average", 5, 7)]
        for pair in ([3, 4], [4, 3], [1, 2], [5, 6]):
            with pytest.raises(ValueError):
                oracle.recovery_plan(s, pair, plus)
    for pair in ([0, 1], [6, 7]):
        with pytest.raises(ValueError):
            oracle.recovery_plan(s, pair, plus=True)
    assert oracle.recovery_plan(s, [0, 7, 3], plus=True) == [("copy", 1), ("copy", 6), ("average", 2, 4)]
    assert oracle.recovery_plan(s, [], plus=False) == []


def test_plan_against_brute_force():
    # every subset of a 6-stage pipeline: recoverable exactly when no two lost stages are adjacent
    # and (without CheckFree+) neither end is lost; a source is always alive and adjacent
    s = 6
    for n in range(s + 1):
        for lost in itertools.combinations(range(s), n):
            adjacent = any(b - a == 1 for a, b in zip(lost, lost[1:]))
            for plus in (False, True):
                ok = not adjacent and (plus or (0 not in lost and s - 1 not in lost))
                if not ok:
                    with pytest.raises(ValueError):
                        oracle.recovery_plan(s, lost, plus)
                    continue
                for i, step in zip(lost, oracle.recovery_plan(s, lost, plus)):
                    assert all(abs(src - i) == 1 and src not in lost for src in step[1:])
                    assert (step[0] == "average") == (0 < i < s - 1) and len(step) == (3 if 0 < i < s - 1 else 2)


def test_plan_argument_errors():
    with pytest.raises(IndexError):
        oracle.recovery_plan(4, [4])
    with pytest.raises(IndexError):
        oracle.recovery_plan(4, [1, 1])
    with pytest.raises(IndexError):
        oracle.recovery_plan(1, [0], plus=True)
