"""Parity of the two-stream (text / image) block with joint attention against its CPU oracle,
through the C-ABI (needs a GPU).

Bar: per output tensor max|gpu - ref| / max|ref| <= 1e-5 on the fp32 check path and <= 2e-2 for
bf16 storage with fp32 accumulation.
"""
import numpy as np
import pytest

from oracle import mmdit_oracle as mo
from paper_2605_25451_amd import synth

pytestmark = pytest.mark.gpu

TOL = {synth.DTYPE_FP32: 1e-5, synth.DTYPE_BF16: 2e-2}
QK_EPS = 1e-6


def rel_err(got, ref):
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def run_hip(case):
    from paper_2605_25451_amd.runner import TwoStreamOnDevice
    dev = TwoStreamOnDevice(case, qk_norm_eps=QK_EPS)
    dev.step()
    return dev.results()


def run_oracle(case):
    ys, cache = mo.mmdit_forward(case.cfg, case.params, case.x, case.cu, case.cond, bool(case.qk_norm), QK_EPS)
    dxs, grads, dcond = mo.mmdit_backward(case.cfg, cache, case.dy, bool(case.qk_norm))
    return ys, dxs, grads, dcond


def compare(case, got, ref):
    tol = TOL[case.cfg.dtype]
    ys, dxs, grads, dcond = got
    rys, rdxs, rgrads, rdcond = ref
    errs = {"dcond": rel_err(dcond, rdcond)}
    for s, tag in enumerate(("text", "img")):
        errs[f"y_{tag}"] = rel_err(ys[s], rys[s])
        errs[f"dx_{tag}"] = rel_err(dxs[s], rdxs[s])
        for k, v in rgrads[s].items():
            errs[f"d{k}_{tag}"] = rel_err(grads[s][k], v)
    print(case.name, {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"{case.name}: above {tol}: {bad}"


def fp32_cases():
    f32 = synth.DTYPE_FP32
    tiny = synth.scaled(synth.dit_block(), hidden=64, n_q_heads=4, n_kv_heads=4, head_dim=16, mlp_hidden=96,
                        dtype=f32)
    dh72 = synth.scaled(synth.dit_block(), hidden=144, n_q_heads=2, n_kv_heads=2, head_dim=72, mlp_hidden=160,
                        dtype=f32)
    dh8 = synth.scaled(synth.dit_block(), hidden=32, n_q_heads=4, n_kv_heads=4, head_dim=8, mlp_hidden=64,
                       dtype=f32)
    out = []
    out.append(synth.make_two_stream_case(tiny, [3, 17, 1], [16, 40, 130], 60, 1, "mmdit_tiny_fp32", 0.1))
    out.append(synth.make_two_stream_case(tiny, [3, 17, 1], [16, 40, 130], 61, 0, "mmdit_tiny_noqknorm_fp32", 0.1))
    out.append(synth.make_two_stream_case(dh72, [50, 2], [21, 77], 62, 1, "mmdit_dh72_fp32", 0.1))
    out.append(synth.make_two_stream_case(dh8, [1], [1], 63, 1, "mmdit_one_token_each_fp32", 0.1))
    out.append(synth.make_two_stream_case(tiny, [140, 5], [7, 1], 64, 1, "mmdit_text_heavy_fp32", 0.1))
    return out


def bf16_cases():
    out = []
    out.append(synth.make_two_stream_case(synth.dit_block(), [77, 20, 150], [256, 256, 576], 70, 1,
                                          "mmdit_d1152_bf16"))
    cfg128 = synth.scaled(synth.dit_block(), hidden=1024, n_q_heads=8, n_kv_heads=8, head_dim=128, mlp_hidden=2048)
    out.append(synth.make_two_stream_case(cfg128, [33, 129], [300, 64], 71, 1, "mmdit_dh128_bf16"))
    cfg64 = synth.scaled(synth.dit_block(), hidden=512, n_q_heads=8, n_kv_heads=8, head_dim=64, mlp_hidden=1024)
    out.append(synth.make_two_stream_case(cfg64, [64, 1, 19], [256, 130, 3], 72, 0, "mmdit_dh64_noqknorm_bf16"))
    return out


@pytest.mark.parametrize("case", fp32_cases(), ids=lambda c: c.name)
def test_fp32_matches_oracle(case):
    compare(case, run_hip(case), run_oracle(case))


@pytest.mark.parametrize("case", bf16_cases(), ids=lambda c: c.name)
def test_bf16_matches_oracle(case):
    compare(case, run_hip(case), run_oracle(case))


def test_gradients_accumulate_and_runs_are_bit_identical():
    import torch
    from paper_2605_25451_amd.runner import TwoStreamOnDevice
    case = bf16_cases()[1]
    dev = TwoStreamOnDevice(case, qk_norm_eps=QK_EPS)
    dev.step()
    ys1, dxs1, g1, dc1 = dev.results()
    dev.step()                                    # second step adds into the same accumulators
    ys2, dxs2, g2, dc2 = dev.results()
    for s in range(2):
        assert np.array_equal(ys1[s], ys2[s]) and np.array_equal(dxs1[s], dxs2[s])
        for k in g1[s]:
            ref = np.abs(g1[s][k]).max()
            assert np.abs(g2[s][k] - 2.0 * g1[s][k]).max() <= 1e-6 * max(ref, 1e-30), k
    assert np.array_equal(dc1, dc2)
    fresh = TwoStreamOnDevice(case, qk_norm_eps=QK_EPS)
    fresh.step()
    _, _, g3, _ = fresh.results()
    for s in range(2):
        for k in g1[s]:
            assert np.array_equal(g1[s][k], g3[s][k]), k
    torch.cuda.synchronize()


def test_descriptor_and_sequence_errors():
    from paper_2605_25451_amd import binding as bm
    from paper_2605_25451_amd.runner import TwoStreamOnDevice
    cfg = synth.scaled(synth.dit_block(), hidden=64, n_q_heads=4, n_kv_heads=4, head_dim=16, mlp_hidden=96,
                       dtype=synth.DTYPE_FP32)
    with pytest.raises(bm.BmError) as e:
        bm.mmdit_sizes(bm.make_mmdit_desc(synth.scaled(synth.vit_tiny(synth.DTYPE_FP32)), 1), 8, 8, 1)
    assert e.value.status == bm.BM_ERR_UNSUPPORTED
    case = synth.make_two_stream_case(cfg, [3, 2], [4, 5], 80, 1, "err", 0.1)
    dev = TwoStreamOnDevice(case)
    dev.cu_host[0] = np.asarray([0, 0, 5], dtype=np.int32)      # a sample without text tokens
    with pytest.raises(bm.BmError) as e:
        dev.forward()
    assert e.value.status == bm.BM_ERR_INVALID_ARG
    dev.cu_host[0] = np.asarray([0, 3, 5], dtype=np.int32)
    with pytest.raises(bm.BmError) as e:
        bm.mmdit_forward(dev.desc, dev.w, dev.x[0], dev.x[1], dev.cu_dev[0], dev.cu_host[0], dev.cu_dev[1],
                         dev.cu_host[1], dev.S, dev.cond, dev.y[0], dev.y[1], dev.saved, dev.scratch, 16)
    assert e.value.status == bm.BM_ERR_WORKSPACE_TOO_SMALL
