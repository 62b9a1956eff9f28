"""Host-side checks of the C-ABI library (no GPU): it loads, exports every
symbol the header declares, validates arguments, and its schedule generator
agrees with the schedule oracle."""
import os
import re

import pytest

from oracle import schedule_oracle as so
from paper_2605_25451_amd import binding as bm
from paper_2605_25451_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CODE = {"E": bm.OP_ENC_FWD, "e": bm.OP_ENC_BWD, "F": bm.OP_LLM_FWD, "B": bm.OP_LLM_BWD,
        "G": bm.OP_GEN_FWD, "H": bm.OP_GEN_BWD}


def test_library_exports_every_declared_symbol():
    text = ""
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        text += re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, f)).read(), flags=re.S)
    names = set(re.findall(r"\b(bm_[a-z_0-9]+)\s*\(", text))
    assert {"bm_block_forward", "bm_block_backward", "bm_block_sizes", "bm_gemm",
            "bm_attention_forward", "bm_attention_backward", "bm_build_schedule"} <= names
    lib = bm.lib()
    for n in names:
        assert hasattr(lib, n), n


@pytest.mark.parametrize("M", [1, 2, 3, 5, 8, 16, 32])
@pytest.mark.parametrize("us", [1, 2, 4])
@pytest.mark.parametrize("gen", [0, 1])
def test_schedule_matches_oracle(M, us, gen):
    cols = so.llm_schedule_1f1b(M, us, 3)
    want = {
        bm.ORDER_NESTED: so.build_schedule(cols, M, us, 3, bool(gen)),
        bm.ORDER_COMPUTE_EFFICIENT: so.compute_efficient_schedule(cols, M, us, bool(gen)),
        bm.ORDER_SEQUENTIAL: so.sequential_schedule(M, us, bool(gen)),
    }
    for order, ref in want.items():
        got = bm.build_schedule(order, M, us, 3, 3, gen)
        assert got == [(CODE[k], i) for k, i in ref]
        peak = bm.check_schedule(got, M, us, gen)
        ref_peak = so.live_counts(ref, M, us)
        assert peak == (ref_peak["enc"], ref_peak["gen"], ref_peak["llm"])


@pytest.mark.parametrize("depth", [1, 2, 3, 4])
@pytest.mark.parametrize("extra_w", [0, 1, 3])
@pytest.mark.parametrize("us", [1, 2, 3])
@pytest.mark.parametrize("gen", [0, 1])
def test_nested_schedule_properties_for_any_depth_and_warm_up(depth, extra_w, us, gen):
    """What Sec. 3.1 states about the nested order, checked on the library's output without the
    oracle's generator: dependencies hold, the LLM order is untouched, at most W encoder units
    and one generator unit are alive, every nested op sits at the first point where its inputs
    exist, and the order property F_i, F_{i+1}, F_{i+2} < G_i < F_{i+3} holds at depth 3 (G_i = the
    backward that completes unit i's gradient at the LLM entry)."""
    W = depth + extra_w
    for M in (1, 2, 3, 5, 7, 12, 13):
        U = -(-M // us)
        ops = bm.build_schedule(bm.ORDER_NESTED, M, us, W, depth, gen)
        peak = bm.check_schedule(ops, M, us, gen)                       # raises on a broken dependency
        assert peak[0] == min(W, U) and peak[1] == (1 if gen else 0) and peak[2] <= depth * us
        llm = [op for op in ops if op[0] in (bm.OP_LLM_FWD, bm.OP_LLM_BWD)]
        flat = [(CODE[k], i) for col in so.llm_schedule_1f1b(M, us, depth) for k, i in col]
        assert llm == flat                                              # the LLM schedule is kept verbatim
        pos = {op: i for i, op in enumerate(ops)}
        last = lambda u: min((u + 1) * us, M) - 1
        for u in range(U):
            if gen:                                                     # right behind the unit's last forward
                assert pos[(bm.OP_GEN_FWD, u)] == pos[(bm.OP_LLM_FWD, last(u))] + 1
                assert pos[(bm.OP_GEN_BWD, u)] == pos[(bm.OP_GEN_FWD, u)] + 1
            assert pos[(bm.OP_ENC_BWD, u)] == pos[(bm.OP_LLM_BWD, last(u))] + 1
            if u + W < U:                                               # the freed slot is taken at once
                assert pos[(bm.OP_ENC_FWD, u + W)] == pos[(bm.OP_ENC_BWD, u)] + 1
            if u < min(W, U):
                assert pos[(bm.OP_ENC_FWD, u)] == u                     # warm-up fills every slot
        if depth == 3:                               # G_i: the unit's gradient reaches the entry stage
            first = lambda u: u * us
            for i in range(U):
                g = pos[(bm.OP_LLM_BWD, last(i))]
                assert all(pos[(bm.OP_LLM_FWD, first(j))] < g for j in range(i, min(i + 3, U)))
                if i + 3 < U:
                    assert g < pos[(bm.OP_LLM_FWD, first(i + 3))]


def test_check_schedule_rejects_unsafe_orders():
    ops = bm.build_schedule(bm.ORDER_NESTED, 4, 1, 3, 3, 1)
    i = ops.index((bm.OP_LLM_FWD, 0)); j = ops.index((bm.OP_ENC_FWD, 0))
    bad = list(ops); bad[i], bad[j] = bad[j], bad[i]          # LLM forward before its encoder unit
    with pytest.raises(bm.BmError):
        bm.check_schedule(bad, 4, 1, 1)
    i = ops.index((bm.OP_GEN_BWD, 0)); j = ops.index((bm.OP_LLM_BWD, 0))
    bad = list(ops); bad[i], bad[j] = bad[j], bad[i]          # LLM backward before generator backward
    with pytest.raises(bm.BmError):
        bm.check_schedule(bad, 4, 1, 1)
    with pytest.raises(bm.BmError):
        bm.check_schedule(ops[:-1], 4, 1, 1)                   # an op is missing
    with pytest.raises(bm.BmError):
        bm.check_schedule(ops + [ops[-1]], 4, 1, 1)            # an op appears twice


def test_build_schedule_argument_errors():
    with pytest.raises(bm.BmError):
        bm.build_schedule(bm.ORDER_NESTED, 0, 1, 3, 3, 1)
    with pytest.raises(bm.BmError):
        bm.build_schedule(bm.ORDER_NESTED, 8, 1, 2, 3, 1)      # W too small for 3 units in flight
    with pytest.raises(bm.BmError):
        bm.build_schedule(7, 8, 1, 3, 3, 1)


def test_block_sizes_and_descriptor_validation():
    desc = bm.make_desc(synth.vit_large())
    saved, scratch = bm.block_sizes(desc, 16384, 26, 1024)
    T, d, F = 16384, 1024, 4096
    assert saved >= T * (3 * d + d + d + F) * 2 + 16 * T * 4
    assert scratch >= T * F * 2
    s2, _ = bm.block_sizes(desc, 2 * T, 52, 1024)
    assert 1.9 < s2 / saved < 2.1                              # activation bytes scale with tokens
    bad = bm.make_desc(synth.scaled(synth.vit_large(), n_kv_heads=5))
    with pytest.raises(bm.BmError) as e:
        bm.block_sizes(bad, 128, 1, 128)
    assert e.value.status == bm.BM_ERR_INVALID_ARG
    bad = bm.make_desc(synth.scaled(synth.vit_large(), hidden=1000))
    with pytest.raises(bm.BmError):
        bm.block_sizes(bad, 128, 1, 128)
    odd = bm.make_desc(synth.scaled(synth.vit_large(), n_q_heads=16, n_kv_heads=16, head_dim=40, hidden=640))
    with pytest.raises(bm.BmError) as e:
        bm.block_sizes(odd, 128, 1, 128)
    assert e.value.status == bm.BM_ERR_UNSUPPORTED
    with pytest.raises(bm.BmError):
        bm.block_sizes(desc, 0, 1, 1)
    # no tensor of a call may reach 2^31 elements: 2^19 tokens x 4096 columns is refused, half of it is not
    with pytest.raises(bm.BmError) as e:
        bm.block_sizes(desc, 1 << 19, 512, 1024)
    assert e.value.status == bm.BM_ERR_INVALID_ARG and "2^31" in str(e.value)
    bm.block_sizes(desc, (1 << 18), 256, 1024)
    moe = bm.make_desc(synth.decoder_moe())
    with pytest.raises(bm.BmError):
        bm.block_sizes(moe, 1 << 28, 1 << 10, 1 << 18)         # tokens x choices leaves the int range


def test_static_workspace_entry_refuses_oversized_packs_without_a_gpu():
    """The size check of the allocation-free attention backward comes before any device call."""
    import numpy as np
    cap = bm.attention_backward_static_capacity()
    assert cap == 64 << 20
    Hq, Hkv, dh, T = 32, 8, 128, 8192
    assert bm.attention_backward_scratch_bytes(Hq, Hkv, dh, T) > cap
    cu = np.array([0, T], dtype=np.int32)
    p, ld = 4096, (Hq + 2 * Hkv) * dh          # never dereferenced: the call stops at the size check
    with pytest.raises(bm.BmError) as e:
        bm.attention_backward_static(synth.DTYPE_BF16, 1, Hq, Hkv, dh, p, p, p, ld, p, p, p, p, cu, 1, T, T,
                                     p, p, p, ld, stream=0)
    assert e.value.status == -3
    assert "built-in workspace" in str(e.value)


def test_mfma_yardstick_refuses_unknown_switches_without_a_gpu():
    """bm_probe_mfma_ex checks its arguments before it launches anything."""
    import ctypes as C
    l = bm.lib()
    dummy = C.c_void_p(256)                      # never dereferenced: the call is refused first
    for blocks, iters, shape16, rnd in ((0, 1, 0, 0), (1, 0, 0, 0), (1, 1, 2, 0), (1, 1, 0, 3)):
        assert l.bm_probe_mfma_ex(blocks, iters, shape16, rnd, dummy, None) == bm.BM_ERR_INVALID_ARG
    assert l.bm_probe_mfma_ex(1, 1, 0, 0, None, None) == bm.BM_ERR_INVALID_ARG


def test_lds_and_issue_yardsticks_refuse_unknown_switches_without_a_gpu():
    """bm_probe_lds / bm_probe_issue check their arguments before they launch anything."""
    import ctypes as C
    l = bm.lib()
    dummy = C.c_void_p(16)
    for what in (0, 3, 6, 7, 10, 16, -1):
        assert l.bm_probe_lds(what, 1, dummy, 1 << 20, dummy, None) == bm.BM_ERR_INVALID_ARG
    assert l.bm_probe_lds(1, 0, dummy, 1 << 20, dummy, None) == bm.BM_ERR_INVALID_ARG
    assert l.bm_probe_lds(8, 1, None, 0, dummy, None) == bm.BM_ERR_INVALID_ARG          # direct loads need a source
    assert l.bm_probe_lds(9, 1, dummy, 1024, dummy, None) == bm.BM_ERR_INVALID_ARG      # ... of 512 KiB
    assert l.bm_probe_lds(1, 1, None, 0, None, None) == bm.BM_ERR_INVALID_ARG
    for nv in (1, 2, 3, 5, 16, -4):
        assert l.bm_probe_issue(nv, 1, dummy, None) == bm.BM_ERR_INVALID_ARG
    assert l.bm_probe_issue(4, 0, dummy, None) == bm.BM_ERR_INVALID_ARG
    assert l.bm_probe_issue(4, 1, None, None) == bm.BM_ERR_INVALID_ARG
