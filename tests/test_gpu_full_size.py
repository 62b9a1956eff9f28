"""Parity at the full benchmark sizes (needs a GPU), in the launch configuration
bench.py times: configs 2 and 3 in full against the oracle; config 4 on sampled
documents (every non-attention op is per token and attention is per document, so
y and dx rows of a document equal that document run alone -- pinned for the oracle
in test_oracle_block.py) plus the additivity of weight gradients over documents."""
import numpy as np
import pytest

from oracle import block_oracle as bo
from paper_2605_25451_amd import synth

pytestmark = pytest.mark.gpu
TOL = 2e-2


def rel_err(got, ref):
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def run_hip(case):
    from paper_2605_25451_amd.runner import CaseOnDevice
    dev = CaseOnDevice(case)
    dev.step()
    return dev.results()


def check_all(case, got, ref):
    y, dx, grads, _ = got
    ry, rdx, rgrads, _ = ref
    errs = {"y": rel_err(y, ry), "dx": rel_err(dx, rdx)}
    errs.update({"d" + k: rel_err(grads[k], rgrads[k]) for k in rgrads})
    print(case.name, {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    assert max(errs.values()) <= TOL, errs


def test_config2_full():
    case = synth.config2()
    print("config2 full", case.T, case.S, flush=True)
    check_all(case, run_hip(case), bo.block_fwd_bwd(case.cfg, case.params, case.x, case.cu_seqlens, case.dy))


def test_config3_full():
    case = synth.config3()
    print("config3 full", case.T, case.S, flush=True)
    check_all(case, run_hip(case), bo.block_fwd_bwd(case.cfg, case.params, case.x, case.cu_seqlens, case.dy))


def test_config4_sampled_documents_and_gradient_additivity():
    case = synth.config4()
    lens = np.diff(case.cu_seqlens)
    print("config4 full", case.T, case.S, "lens", lens.tolist(), flush=True)
    y, dx, grads, _ = run_hip(case)
    # sampled documents: the two shortest and the longest one not above 4096 tokens
    order = np.argsort(lens)
    mid = [int(i) for i in order if lens[i] <= 4096][-1]
    picks = sorted({int(order[0]), int(order[1]), mid})
    for s in picks:
        sub = synth.sub_case(case, [s])
        ry, rdx, _, _ = bo.block_fwd_bwd(sub.cfg, sub.params, sub.x, sub.cu_seqlens, sub.dy)
        lo, hi = case.cu_seqlens[s], case.cu_seqlens[s + 1]
        scale_y, scale_dx = np.abs(ry).max(), np.abs(rdx).max()
        ey = np.abs(y[lo:hi] - ry).max() / scale_y
        edx = np.abs(dx[lo:hi] - rdx).max() / scale_dx
        print(f"  doc {s} len {lens[s]}: y {ey:.2e} dx {edx:.2e}", flush=True)
        assert ey <= TOL and edx <= TOL
    # weight gradients: sum over two halves of the documents == the full pack
    half = case.S // 2
    parts = [synth.sub_case(case, list(range(0, half))), synth.sub_case(case, list(range(half, case.S)))]
    acc = None
    for p in parts:
        _, _, g, _ = run_hip(p)
        acc = g if acc is None else {k: acc[k] + g[k] for k in g}
    for k in grads:
        assert rel_err(acc[k], grads[k]) <= 5e-3, k
    # and the oracle agrees on the gradients of a small sub-pack
    small = synth.sub_case(case, picks[:2])
    _, _, g_small, _ = run_hip(small)
    _, _, rg, _ = bo.block_fwd_bwd(small.cfg, small.params, small.x, small.cu_seqlens, small.dy)
    for k in rg:
        assert rel_err(g_small[k], rg[k]) <= TOL, k
