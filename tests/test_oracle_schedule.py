"""Pins for the schedule oracle (CPU only): hand expansions of the paper's
BuildSchedule algorithm and the invariants the paper states for it."""
import os

import pytest

from oracle import schedule_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "schedule_hand_expansions.txt")


def golden_rows():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, sched = line.split("|")
        M, us, W, gen = [int(t) for t in head.split()]
        rows.append((M, us, W, gen, sched.strip()))
    return rows


@pytest.mark.parametrize("M,us,W,gen,expected", golden_rows())
def test_hand_expansions(M, us, W, gen, expected):
    cols = so.llm_schedule_1f1b(M, us, 3)
    assert so.format_schedule(so.build_schedule(cols, M, us, W, bool(gen))) == expected


def test_1f1b_order_by_hand():
    flat = [op for c in so.llm_schedule_1f1b(5, 1, 3) for op in c]
    assert so.format_schedule(flat) == "F0 F1 F2 B0 F3 B1 F4 B2 B3 B4"


@pytest.mark.parametrize("M", [1, 2, 3, 4, 7, 8, 16, 32])
@pytest.mark.parametrize("us", [1, 2, 4])
@pytest.mark.parametrize("gen", [False, True])
def test_invariants(M, us, gen):
    cols = so.llm_schedule_1f1b(M, us, 3)
    llm = [op for c in cols for op in c]
    s = so.build_schedule(cols, M, us, 3, gen)
    # the LLM order is untouched (Sec. 3.1: nesting keeps the LLM schedule unchanged)
    assert [op for op in s if op[0] in "FB"] == llm
    units = so.partition_microbatches(M, us)
    pos = {op: i for i, op in enumerate(s)}
    assert len(pos) == len(s)                                   # every op exactly once
    for u, mbs in enumerate(units):
        assert pos[("E", u)] < pos[("F", mbs[0])]               # LLM fwd consumes encoder output
        assert pos[("B", mbs[-1])] < pos[("e", u)]              # encoder bwd needs the LLM input grad
        if gen:
            assert pos[("F", mbs[-1])] < pos[("G", u)] < pos[("H", u)]
            for m in mbs:
                assert pos[("H", u)] < pos[("B", m)]            # LLM bwd needs the generator's grad
        for m in mbs:
            assert pos[("F", m)] < pos[("B", m)]
    peak = so.live_counts(s, M, us)
    assert peak["enc"] <= 3                                     # W = 3 encoder units suffice
    assert peak["gen"] <= (1 if gen else 0)                     # one generator unit
    # order property F_i, F_{i+1}, F_{i+2} < G_i < F_{i+3} at unit level
    U = len(units)
    for i in range(U):
        g_i = pos[("B", units[i][-1])]
        for j in (i, i + 1, i + 2):
            if j < U:
                assert pos[("F", units[j][0])] < g_i
        if i + 3 < U:
            assert g_i < pos[("F", units[i + 3][0])]
    # the compute-efficient baseline keeps every encoder unit alive (peak ~ M/P units)
    base = so.compute_efficient_schedule(cols, M, us, gen)
    assert so.live_counts(base, M, us)["enc"] == U
    assert [op for op in base if op[0] in "FB"] == llm
    seq = so.sequential_schedule(M, us, gen)
    assert sorted(seq) == sorted(s)
    assert so.live_counts(seq, M, us)["enc"] == 1
