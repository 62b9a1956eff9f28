"""Host-side parity of the library's multi-rank schedule generator and replay with the
pipeline oracle (no GPU): rank programs token for token, replay figures to the last bit
(both sides add the same doubles in the same order)."""
import numpy as np
import pytest

from oracle import pipeline_oracle as po
from paper_2605_25451_amd import binding as bm

CODE = {"E": bm.OP_ENC_FWD, "e": bm.OP_ENC_BWD, "F": bm.OP_LLM_FWD, "B": bm.OP_LLM_BWD,
        "G": bm.OP_GEN_FWD, "H": bm.OP_GEN_BWD}
ORDERS = {po.NESTED: bm.ORDER_NESTED, po.COMPUTE_EFFICIENT: bm.ORDER_COMPUTE_EFFICIENT,
          po.MEMORY_EFFICIENT: bm.ORDER_MEMORY_EFFICIENT}
GRID = [(1, 1, 1), (1, 1, 5), (1, 3, 2), (2, 1, 2), (2, 1, 8), (2, 2, 2), (2, 2, 8), (3, 3, 9), (4, 1, 4),
        (4, 1, 16), (4, 2, 4), (4, 2, 16), (4, 2, 64), (4, 4, 16), (8, 1, 16), (8, 2, 32), (4, 3, 8),
        (5, 2, 20), (8, 4, 8)]


@pytest.mark.parametrize("P,V,M", GRID)
def test_llm_schedule_matches_oracle(P, V, M):
    for r in range(P):
        got = bm.pipeline_llm_schedule(P, V, M, r)
        want = po.llm_rank_schedule(P, V, M, r)
        assert [(o, i, c) for o, i, c, _ in got] == [(CODE[k], i, c) for k, i, c in want]
        assert [col for *_, col in got] == list(range(len(want)))


@pytest.mark.parametrize("P,V,M", GRID)
@pytest.mark.parametrize("gen", [0, 1])
@pytest.mark.parametrize("W", [1, 3])
def test_rank_programs_match_oracle(P, V, M, gen, W):
    for name, order in ORDERS.items():
        for r in range(P):
            got = bm.pipeline_build_schedule(order, P, V, M, W, gen, r)
            want = po.build_rank_schedule(name, P, V, M, W, bool(gen), r)
            assert [(o, i, c) for o, i, c, _ in got] == [(CODE[k], i, c) for k, i, c in want]


@pytest.mark.parametrize("P,V,M", GRID)
@pytest.mark.parametrize("gen", [0, 1])
def test_replay_matches_oracle_bit_for_bit(P, V, M, gen):
    rng = np.random.default_rng(P * 100 + V * 10 + M + gen)
    n = P * V
    d = dict(llm_fwd=rng.uniform(0.5, 1.5, n), llm_bwd=rng.uniform(1.0, 3.0, n),
             enc_fwd=rng.uniform(0.05, 0.6, M), enc_bwd=rng.uniform(0.1, 1.2, M),
             gen_fwd=rng.uniform(0.05, 0.4, M), gen_bwd=rng.uniform(0.1, 0.8, M))
    acts = dict(act_llm=3.5, act_enc=rng.uniform(0.5, 2.0, M), act_gen=rng.uniform(0.1, 0.7, M))
    for name, order in ORDERS.items():
        for p2p in (0.0, 0.037):
            want = po.replay(name, P, V, M, 3, bool(gen), d["llm_fwd"], d["llm_bwd"], d["enc_fwd"],
                             d["enc_bwd"], d["gen_fwd"], d["gen_bwd"], p2p=p2p, **acts) \
                if not (name == po.NESTED and needs_more_warmup(P, V, M)) else None
            if want is None:
                continue
            got = bm.pipeline_replay(order, P, V, M, 3, gen, d["llm_fwd"], d["llm_bwd"], d["enc_fwd"],
                                     d["enc_bwd"], d["gen_fwd"], d["gen_bwd"], p2p=p2p, **acts)
            assert got["makespan"] == want["makespan"] and got["bubble"] == want["bubble"]
            for k in ("busy", "peak", "peak_enc", "peak_gen", "peak_llm"):
                assert got[k] == list(want[k]), k


def needs_more_warmup(P, V, M):
    try:
        z = [0.0] * M
        po.replay(po.NESTED, P, V, M, 3, False, [1.0] * (P * V), [1.0] * (P * V), z, z, z, z)
        return False
    except RuntimeError:
        return True


def test_deadlock_and_argument_errors_are_reported():
    z = [0.0] * 16
    with pytest.raises(bm.BmError) as e:
        bm.pipeline_replay(bm.ORDER_NESTED, 4, 2, 16, 2, 0, [1.0] * 8, [2.0] * 8, z, z)
    assert "deadlock" in str(e.value)
    with pytest.raises(bm.BmError):
        bm.pipeline_llm_schedule(4, 2, 6, 0)            # M not a multiple of P
    with pytest.raises(bm.BmError):
        bm.pipeline_llm_schedule(4, 2, 8, 4)            # rank out of range
    with pytest.raises(bm.BmError):
        bm.pipeline_build_schedule(bm.ORDER_SEQUENTIAL, 4, 2, 8, 3, 0, 0)
    with pytest.raises(bm.BmError):
        bm.pipeline_replay(bm.ORDER_NESTED, 4, 2, 8, 3, 1, [1.0] * 8, [2.0] * 8, [0.0] * 8, [0.0] * 8)  # no generator times


def test_paper_figure_configuration_properties():
    # the configuration of the paper's scheme figure: pp 4, vpp 2, batch 64, W = 3
    P, V, M = 4, 2, 64
    n = P * V
    enc_f = [0.3 + 0.1 * (m % 5) for m in range(M)]
    enc_b = [2 * t for t in enc_f]
    res = {}
    for order in (bm.ORDER_NESTED, bm.ORDER_COMPUTE_EFFICIENT, bm.ORDER_MEMORY_EFFICIENT):
        res[order] = bm.pipeline_replay(order, P, V, M, 3, 0, [1.0] * n, [2.0] * n, enc_f, enc_b,
                                        act_llm=1.0, act_enc=[1.0] * M)
    assert res[bm.ORDER_NESTED]["peak_enc"] == [3.0] * P                 # W units
    assert res[bm.ORDER_COMPUTE_EFFICIENT]["peak_enc"] == [16.0] * P     # M / P units
    assert res[bm.ORDER_MEMORY_EFFICIENT]["peak_enc"][0] == 8.0          # first stage's in-flight depth
    # uneven encoder work stalls the coupled pipeline; the nested order hides it
    assert res[bm.ORDER_NESTED]["makespan"] < res[bm.ORDER_MEMORY_EFFICIENT]["makespan"]


@pytest.mark.parametrize("P,V,M", GRID)
@pytest.mark.parametrize("gen", [0, 1])
def test_comm_programs_and_report_match_oracle(P, V, M, gen):
    msg = {n: i for i, n in enumerate(bm.MSG_NAMES)}
    for name, order in ORDERS.items():
        for W in (1, 3):
            for r in range(P):
                got = bm.pipeline_comm_schedule(order, P, V, M, W, gen, r)
                want = []
                for op in po.comm_rank_schedule(name, P, V, M, W, bool(gen), r):
                    if op[0] in ("SEND", "RECV"):
                        want.append((bm.OP_SEND if op[0] == "SEND" else bm.OP_RECV, op[3], op[4], op[1], msg[op[2]]))
                    else:
                        want.append((CODE[op[0]], op[1], op[2], -1, -1))
                assert got == want
            assert bm.pipeline_check_comm(order, P, V, M, W, gen) == po.check_comm(name, P, V, M, W, bool(gen))


def test_check_comm_reports_the_w2_deadlock_of_the_interleaved_schedule():
    assert bm.pipeline_check_comm(bm.ORDER_NESTED, 4, 2, 16, 2, 0)["deadlock"] is True
    rep = bm.pipeline_check_comm(bm.ORDER_NESTED, 4, 2, 64, 3, 1)
    assert rep == {"deadlock": False, "unmatched": 0, "fifo": False, "max_inflight": rep["max_inflight"],
                   "messages": 2 * 64 * 7 + 2 * 48 * 2}
