"""Pins of the multi-rank schedule oracle and its replay (CPU only): hand expansions,
the closed forms of Sec. 2.2 "Performance analysis", the order property of Sec. 3.1
"Analysis", dependency safety and the memory bounds the paper states."""
import os
import re

import pytest

from oracle import pipeline_oracle as po

GOLD = os.path.join(os.path.dirname(__file__), "golden", "pipeline_hand_expansions.txt")
GRID = [(2, 1, 8), (4, 1, 16), (4, 2, 16), (4, 2, 64), (8, 2, 32), (4, 4, 16), (3, 3, 9), (2, 2, 8),
        (8, 1, 16), (4, 3, 8), (4, 2, 4), (2, 1, 2), (1, 1, 4), (1, 2, 3)]


def fmt(op):
    kind, i, c = op
    return f"{kind}{i}" if c == 0 else f"{kind}{i}.{c}"


def gold_lines(prefix):
    for line in open(GOLD):
        if line.startswith(prefix):
            yield line.strip()


def test_hand_expansions_token_for_token():
    n = 0
    for line in list(gold_lines("nested")) + list(gold_lines("compute_efficient")):
        m = re.match(r"(\w+) P=(\d+) V=(\d+) M=(\d+) W=(\d+) gen=(\d) rank=(\d+): (.*)", line)
        order, P, V, M, W, gen, rank = m.group(1), *map(int, m.groups()[1:7])
        got = " ".join(fmt(o) for o in po.build_rank_schedule(order, P, V, M, W, bool(gen), rank))
        assert got == m.group(8), line
        n += 1
    assert n == 5


def test_hand_replay():
    line = next(gold_lines("replay"))
    m = re.match(r"replay P=2 V=1 M=2 tf=1 tb=2: makespan=(\d+) busy=(\d+),(\d+)", line)
    r = po.replay(po.MEMORY_EFFICIENT, 2, 1, 2, 3, False, [1.0, 1.0], [2.0, 2.0], [0, 0], [0, 0], [0, 0], [0, 0])
    assert r["makespan"] == float(m.group(1))
    assert r["busy"] == [float(m.group(2)), float(m.group(3))]
    assert abs(r["bubble"] - 1.0 / 3.0) < 1e-15


@pytest.mark.parametrize("P,V,M", GRID)
def test_llm_schedule_is_a_valid_pipeline_order(P, V, M):
    for r in range(P):
        ops = po.llm_rank_schedule(P, V, M, r)
        assert len(ops) == 2 * M * V and len(set(ops)) == len(ops)
        pos = {op: i for i, op in enumerate(ops)}
        for m in range(M):
            for c in range(V):
                assert pos[("F", m, c)] < pos[("B", m, c)]
                if c > 0:      # chunks of one microbatch in model order
                    assert pos[("F", m, c - 1)] < pos[("F", m, c)]
                    assert pos[("B", m, c)] < pos[("B", m, c - 1)]
        # every cross-rank input was produced no later than the same column of the neighbour
        if r > 0:
            prev = {op: i for i, op in enumerate(po.llm_rank_schedule(P, V, M, r - 1))}
            for op, i in pos.items():
                if op[0] == "F":
                    assert prev[op] <= i
                else:
                    assert i <= prev[op]


@pytest.mark.parametrize("P,V,M", GRID)
def test_uniform_llm_replay_matches_closed_forms(P, V, M):
    # Sec. 2.2: 1F1B fill/drain only, bubble rate (P-1)/(M+P-1); with V chunks per rank
    # the fill/drain shrinks by V: makespan (M V + P - 1)(tf + tb) for per-chunk times.
    tf, tb = 0.75, 1.5
    n = P * V
    r = po.replay(po.MEMORY_EFFICIENT, P, V, M, 3, False, [tf] * n, [tb] * n, [0] * M, [0] * M,
                  [0] * M, [0] * M, act_llm=1.0)
    assert r["makespan"] == pytest.approx((M * V + P - 1) * (tf + tb), rel=1e-12)
    assert r["bubble"] == pytest.approx((P - 1) / (M * V + P - 1), rel=1e-12)
    for rank in range(P):
        assert r["busy"][rank] == pytest.approx(M * V * (tf + tb), rel=1e-12)
        # in-flight microbatch-chunks: warm-up depth + 1 (P - rank for the classic order)
        depth = P - rank if V == 1 else 2 * (P - rank - 1) + (V - 1) * P + 1
        assert r["peak_llm"][rank] == min(depth, M * V)


def unit_level(ops, P, V):
    """First entry-side forward F_i and gradient-complete point G_i of every unit on rank 0."""
    pos = {op: i for i, op in enumerate(ops)}
    U = max(op[1] for op in ops) // P + 1
    F = [min(pos[("F", u * P + k, 0)] for k in range(P)) for u in range(U)]
    G = [pos[("B", u * P + P - 1, 0)] for u in range(U)]
    return F, G


@pytest.mark.parametrize("P,V,M", [(4, 2, 64), (4, 2, 32), (8, 2, 64), (4, 4, 32), (3, 3, 18), (8, 3, 48)])
def test_order_property_of_interleaved_schedules(P, V, M):
    # Sec. 3.1 "Analysis": F_i, F_{i+1}, F_{i+2} < G_i < F_{i+3} for vpp >= 2
    F, G = unit_level(po.llm_rank_schedule(P, V, M, 0), P, V)
    for i in range(len(F) - 3):
        assert F[i] < F[i + 1] < F[i + 2] < G[i] < F[i + 3]


@pytest.mark.parametrize("P,V,M", GRID)
@pytest.mark.parametrize("gen", [False, True])
def test_nested_programs_keep_llm_order_and_dependencies(P, V, M, gen):
    W = 3
    U = M // P
    progs = [po.build_rank_schedule(po.NESTED, P, V, M, W, gen, r) for r in range(P)]
    unit_ops = None
    for r, prog in enumerate(progs):
        assert [op for op in prog if op[0] in "FB"] == po.llm_rank_schedule(P, V, M, r)
        seq = [op for op in prog if op[0] not in "FB"]
        assert sorted(seq) == sorted([(k, u, 0) for u in range(U) for k in ("E", "e") + (("G", "H") if gen else ())])
        enc_seq = [op for op in seq if op[0] in "Ee"]
        if unit_ops is None:
            unit_ops = enc_seq
        assert enc_seq == unit_ops                       # same encoder order on every rank
        pos = {op: i for i, op in enumerate(prog)}
        for u in range(U):
            m = u * P + r
            assert pos[("E", u, 0)] < pos[("e", u, 0)]
            if r == 0:                                   # entry stage consumes encoder outputs
                for k in range(P):
                    assert pos[("E", u, 0)] < pos[("F", u * P + k, 0)]
                assert pos[("B", u * P + P - 1, 0)] < pos[("e", u, 0)]
            if gen:
                assert pos[("G", u, 0)] + 1 == pos[("H", u, 0)]
                if r == P - 1:                           # exit stage: output, generator, then backward
                    assert pos[("F", m, V - 1)] < pos[("G", u, 0)] < pos[("B", m, V - 1)]


@pytest.mark.parametrize("P,V,M", GRID)
@pytest.mark.parametrize("gen", [False, True])
def test_replay_is_deadlock_free_and_memory_is_bounded(P, V, M, gen):
    n = P * V
    enc_f = [0.2 + 0.05 * (m % 7) for m in range(M)]       # uneven modality work
    enc_b = [2 * t for t in enc_f]
    gen_f = [0.1 + 0.03 * (m % 5) for m in range(M)]
    gen_b = [2 * t for t in gen_f]
    kw = dict(act_llm=1.0, act_enc=[1.0] * M, act_gen=[1.0] * M)
    args = (P, V, M, 3, gen, [1.0] * n, [2.0] * n, enc_f, enc_b, gen_f, gen_b)
    nested = po.replay(po.NESTED, *args, **kw)
    ce = po.replay(po.COMPUTE_EFFICIENT, *args, **kw)
    me = po.replay(po.MEMORY_EFFICIENT, *args, **kw)
    U = M // P
    for r in range(P):
        assert nested["peak_enc"][r] == min(3, U)           # W = 3 units, one microbatch each
        assert ce["peak_enc"][r] == U                       # (M / P) A_m, Sec. 2.2
        assert nested["peak_gen"][r] == (1.0 if gen else 0.0)
        assert nested["peak_llm"][r] == me["peak_llm"][r]   # LLM in-flight depth untouched
    # memory-efficient: modality activations of the first stage follow its in-flight depth
    depth0 = P if V == 1 else min(M, 2 * P)                 # microbatches with chunk 0 in flight
    assert me["peak_enc"][0] <= depth0
    assert me["peak_enc"][0] >= min(P, M)
    # work is conserved: the three orders execute the same operators
    total = lambda r: sum(r["busy"])
    assert total(nested) == pytest.approx(total(ce), rel=1e-12) == pytest.approx(total(me), rel=1e-12)
    lower = (M * V + P - 1) * 3.0
    assert nested["makespan"] >= lower and ce["makespan"] >= lower and me["makespan"] >= lower


@pytest.mark.parametrize("P,V,M", [(4, 2, 16), (4, 2, 64), (8, 2, 32), (4, 4, 16), (3, 3, 9)])
def test_free_unit_ops_do_not_slow_an_interleaved_llm(P, V, M):
    # Sec. 3.1: nesting leaves the LLM pipeline untouched -- with zero-cost unit ops and no
    # generator the nested makespan equals the LLM-only makespan for vpp >= 2 (the waits of
    # the encoder backward cost less than one backward slot on 8 ranks)
    n = P * V
    z = [0.0] * M
    r = po.replay(po.NESTED, P, V, M, 3, False, [1.0] * n, [2.0] * n, z, z, z, z)
    llm_only = (M * V + P - 1) * 3.0
    if P <= 4:
        assert r["makespan"] == pytest.approx(llm_only, rel=1e-12)
    else:
        assert llm_only <= r["makespan"] <= llm_only + 2.0


def test_too_small_a_warm_up_deadlocks():
    z = [0.0] * 16
    with pytest.raises(RuntimeError):
        po.replay(po.NESTED, 4, 2, 16, 2, False, [1.0] * 8, [2.0] * 8, z, z, z, z)
    with pytest.raises(RuntimeError):
        po.replay(po.NESTED, 4, 1, 16, 1, False, [1.0] * 4, [2.0] * 4, z, z, z, z)
    po.replay(po.NESTED, 4, 1, 16, 2, False, [1.0] * 4, [2.0] * 4, z, z, z, z)   # classic order: 2 suffice


def test_transfer_latency_and_heterogeneous_stage_times():
    # two ranks, one microbatch: F0@0, +latency, F0@1, B0@1, +latency, B0@0
    r = po.replay(po.MEMORY_EFFICIENT, 2, 1, 2, 3, False, [1.0, 3.0], [2.0, 5.0], [0, 0], [0, 0], [0, 0],
                  [0, 0], p2p=0.5)
    # rank0: F0 [0,1] F1 [1,2]; rank1: F0 [1.5,4.5] B0 [4.5,9.5] F1 [9.5,12.5] B1 [12.5,17.5];
    # rank0: B0 [10,12] B1 [18,20]
    assert r["makespan"] == 20.0 and r["busy"] == [6.0, 16.0]


# ------------------------------------------------------------------ communication operators

def fmt_comm(op):
    if op[0] == "SEND":
        return f"S:{op[2]}{op[3]}@{op[4]}>{op[1]}"
    if op[0] == "RECV":
        return f"R:{op[2]}{op[3]}@{op[4]}<{op[1]}"
    return fmt(op)


def test_comm_hand_expansion():
    n = 0
    for line in gold_lines("comm"):
        m = re.match(r"comm (\w+) P=(\d+) V=(\d+) M=(\d+) W=(\d+) gen=(\d) rank=(\d+): (.*)", line)
        order, P, V, M, W, gen, rank = m.group(1), *map(int, m.groups()[1:7])
        got = " ".join(fmt_comm(o) for o in po.comm_rank_schedule(order, P, V, M, W, bool(gen), rank))
        assert got == m.group(8), line
        n += 1
    assert n == 2


@pytest.mark.parametrize("P,V,M", GRID)
@pytest.mark.parametrize("gen", [False, True])
def test_comm_ops_wrap_the_compute_program_and_match_up(P, V, M, gen):
    for order in (po.NESTED, po.COMPUTE_EFFICIENT, po.MEMORY_EFFICIENT):
        for r in range(P):
            prog = po.comm_rank_schedule(order, P, V, M, 3, gen, r)
            assert [op for op in prog if op[0] not in ("SEND", "RECV")] == \
                po.build_rank_schedule(order, P, V, M, 3, gen, r)
            assert all(op[1] != r for op in prog if op[0] in ("SEND", "RECV"))      # never to itself
        res = po.check_comm(order, P, V, M, 3, gen)
        assert res["unmatched"] == 0
        # one activation and one gradient per microbatch and pipeline edge, plus the
        # encoder and generator handoffs of the microbatches another rank owns
        edges = (P * V - 1) if P > 1 else 0
        want = 2 * M * edges
        if order != po.MEMORY_EFFICIENT and P > 1:
            want += 2 * (M - M // P) * (2 if gen else 1)
        assert res["messages"] == want
        needs_w3 = order == po.NESTED and V >= 2 and P >= 3 and M // P > 3
        assert res["deadlock"] is False or not needs_w3


@pytest.mark.parametrize("P,V,M,W,expect", [(4, 2, 16, 2, True), (4, 2, 16, 3, False), (4, 1, 16, 1, True),
                                            (4, 1, 16, 2, False), (3, 3, 9, 2, True), (3, 3, 9, 3, False),
                                            (8, 2, 32, 3, False), (2, 2, 8, 2, False)])
def test_deadlock_check_agrees_with_the_replay(P, V, M, W, expect):
    for gen in (False, True):
        assert po.check_comm(po.NESTED, P, V, M, W, gen)["deadlock"] is expect
        z = [0.0] * M
        try:
            po.replay(po.NESTED, P, V, M, W, gen, [1.0] * (P * V), [1.0] * (P * V), z, z, z, z)
            stuck = False
        except RuntimeError:
            stuck = True
        assert stuck is expect


def test_llm_only_traffic_is_in_order_per_pair_and_nested_traffic_is_not():
    # a transport that matches messages by order alone is enough for the plain pipeline; the
    # nested programs interleave handoff messages differently on the two ends of a pair, which
    # is why every operator carries (what, microbatch, chunk) metadata (Sec. 3.1)
    for P, V, M in [(2, 1, 8), (4, 1, 16), (4, 2, 16), (8, 2, 32), (3, 3, 9)]:
        assert po.check_comm(po.MEMORY_EFFICIENT, P, V, M, 3, False)["fifo"] is True
        assert po.check_comm(po.NESTED, P, V, M, 3, True)["fifo"] is False


def test_a_program_that_runs_a_consumer_before_its_local_producer_is_reported():
    # W = 1: rank 0 would forward a microbatch of unit 1 before its own encoder forward
    assert po.check_comm(po.NESTED, 2, 1, 8, 1, False)["deadlock"] is True
