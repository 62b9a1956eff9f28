"""Parity of the HIP path against the CPU oracle, through the C-ABI (needs a GPU).

Bar: per output tensor max|gpu - ref| / max|ref| <= 1e-5 on the fp32 check
path and <= 2e-2 for bf16 storage with fp32 accumulation.
"""
import numpy as np
import pytest

from oracle import block_oracle as bo
from paper_2605_25451_amd import synth

pytestmark = pytest.mark.gpu

TOL = {synth.DTYPE_FP32: 1e-5, synth.DTYPE_BF16: 2e-2}


def rel_err(got, ref):
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def compare(case, got, ref, tol=None):
    tol = tol or TOL[case.cfg.dtype]
    y, dx, grads, dcond = got
    ry, rdx, rgrads, rdcond = ref
    errs = {"y": rel_err(y, ry), "dx": rel_err(dx, rdx)}
    for k in rgrads:
        errs["d" + k] = rel_err(grads[k], rgrads[k])
    if rdcond is not None:
        errs["dcond"] = rel_err(dcond, rdcond)
    print(case.name, {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"{case.name}: above {tol}: {bad}"
    return errs


def run_hip(case):
    from paper_2605_25451_amd.runner import CaseOnDevice
    dev = CaseOnDevice(case)
    dev.step()
    return dev.results()


def run_oracle(case):
    return bo.block_fwd_bwd(case.cfg, case.params, case.x, case.cu_seqlens, case.dy, case.cond)


def small_cases():
    f32 = synth.DTYPE_FP32
    tiny = dict(hidden=64, n_q_heads=4, n_kv_heads=4, head_dim=16, mlp_hidden=96, dtype=f32)
    out = [synth.config1()]
    out.append(synth.make_case(synth.scaled(synth.vit_tiny(f32), mask=synth.MASK_CAUSAL),
                               [1, 130, 37, 2], 30, name="vit_tiny_causal_fp32"))
    out.append(synth.make_case(synth.scaled(synth.decoder_7b(), **tiny), [17, 140, 5, 1], 31,
                               name="decoder_tiny_fp32"))
    out.append(synth.make_case(synth.scaled(synth.decoder_8b_gqa(), **{**tiny, "n_kv_heads": 2}),
                               [33, 129, 64], 32, name="gqa_tiny_fp32"))
    out.append(synth.make_case(synth.scaled(synth.dit_block(), **tiny), [16, 16, 40], 33,
                               name="dit_tiny_fp32"))
    out.append(synth.make_case(synth.scaled(synth.dit_block(), hidden=144, n_q_heads=2, n_kv_heads=2,
                                            head_dim=72, mlp_hidden=160, dtype=f32), [50, 21], 34,
                               name="dit_dh72_fp32"))
    # fp32 rows wider than four vectors per lane: the norm backward splits them over two wavefronts
    out.append(synth.make_case(synth.scaled(synth.vit_tiny(f32), hidden=1280, n_q_heads=80, n_kv_heads=80,
                                            head_dim=16, mlp_hidden=64), [9, 4], 35, name="vit_wide_d1280_fp32"))
    out.append(synth.make_case(synth.scaled(synth.dit_block(), hidden=1536, n_q_heads=96, n_kv_heads=96,
                                            head_dim=16, mlp_hidden=64, dtype=f32), [5, 6], 36,
                               name="dit_wide_d1536_fp32"))
    return out


def medium_bf16_cases():
    out = []
    out.append(synth.make_case(synth.vit_large(), [300, 257, 143, 1, 67], 40, name="vit_large_bf16_T768"))
    out.append(synth.make_case(synth.scaled(synth.vit_large(), mask=synth.MASK_CAUSAL),
                               [129, 500], 41, name="vit_large_causal_bf16"))
    out.append(synth.make_case(synth.scaled(synth.decoder_7b(), mlp_hidden=2816, hidden=1024,
                                            n_q_heads=8, n_kv_heads=8),
                               [333, 64, 515], 42, name="decoder_d1024_bf16"))
    out.append(synth.make_case(synth.scaled(synth.decoder_8b_gqa(), mlp_hidden=3584, hidden=1024,
                                            n_q_heads=8, n_kv_heads=2),
                               [700, 19, 180], 43, name="gqa_d1024_bf16"))
    out.append(synth.make_case(synth.dit_block(), [256, 256, 256], 44, name="dit_bf16_3img"))
    out.append(synth.make_case(synth.scaled(synth.vit_tiny(), dtype=synth.DTYPE_BF16), [16, 24], 45,
                               name="vit_tiny_bf16"))
    # wide rows (two wavefronts share a row in the norm backward), odd row counts
    out.append(synth.make_case(synth.scaled(synth.vit_large(), hidden=2560, n_q_heads=20, n_kv_heads=20,
                                            head_dim=128, mlp_hidden=1024), [70, 1], 46, name="vit_wide_d2560_bf16"))
    out.append(synth.make_case(synth.scaled(synth.decoder_7b(), mlp_hidden=1024), [33, 40], 47,
                               name="decoder_wide_d4096_bf16"))
    out.append(synth.make_case(synth.scaled(synth.dit_block(), hidden=3072, n_q_heads=24, n_kv_heads=24,
                                            head_dim=128, mlp_hidden=1024), [64, 7, 64], 48, name="dit_wide_d3072_bf16"))
    return out


@pytest.mark.parametrize("case", small_cases(), ids=lambda c: c.name)
def test_fp32_check_path_matches_oracle(case):
    compare(case, run_hip(case), run_oracle(case))


@pytest.mark.parametrize("case", medium_bf16_cases(), ids=lambda c: c.name)
def test_bf16_blocks_match_oracle(case):
    compare(case, run_hip(case), run_oracle(case))


def test_full_width_decoder_bf16():
    case = synth.make_case(synth.decoder_7b(), [400, 130, 70], 46, name="decoder_7b_bf16_T600")
    compare(case, run_hip(case), run_oracle(case))


def test_full_width_gqa_decoder_bf16():
    case = synth.make_case(synth.decoder_8b_gqa(), [290, 222], 47, name="decoder_8b_gqa_bf16_T512")
    compare(case, run_hip(case), run_oracle(case))


def edge_cases():
    f32 = synth.DTYPE_FP32
    tiny = dict(hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, mlp_hidden=96, dtype=f32)
    rng = np.random.default_rng(7)
    many = [int(v) for v in rng.integers(1, 8, size=150)]            # 150 sequences of 1..7 tokens
    out = []
    out.append(synth.make_case(synth.scaled(synth.decoder_8b_gqa(), **tiny), [1], 50, name="one_token_fp32"))
    out.append(synth.make_case(synth.scaled(synth.decoder_8b_gqa(), **tiny), many, 51, name="many_tiny_fp32"))
    out.append(synth.make_case(synth.vit_large(), [1], 52, name="one_token_vit_bf16"))
    out.append(synth.make_case(synth.vit_large(), many, 53, name="many_tiny_vit_bf16"))
    out.append(synth.make_case(synth.scaled(synth.decoder_8b_gqa(), mlp_hidden=1024, hidden=512,
                                            n_q_heads=4, n_kv_heads=1),
                               [2049], 54, name="one_long_gqa_bf16"))
    out.append(synth.make_case(synth.scaled(synth.decoder_7b(), mlp_hidden=1024, hidden=512,
                                            n_q_heads=4, n_kv_heads=4),
                               [77], 55, name="odd_T_decoder_bf16"))
    out.append(synth.make_case(synth.dit_block(), [1, 3, 257], 56, name="dit_ragged_bf16"))
    return out


@pytest.mark.parametrize("case", edge_cases(), ids=lambda c: c.name)
def test_edge_shapes_match_oracle(case):
    """Degenerate packs: a single token, many tiny sequences, one long sequence, odd totals."""
    compare(case, run_hip(case), run_oracle(case))


def test_gradients_accumulate_and_runs_are_bit_identical():
    from paper_2605_25451_amd.runner import CaseOnDevice
    case = synth.make_case(synth.vit_large(), [200, 120], 48, name="vit_large_accumulate")
    dev = CaseOnDevice(case)
    dev.step()
    y1, dx1, g1, _ = dev.results()
    dev.step()                                   # grads not zeroed: second contribution is added
    y2, dx2, g2, _ = dev.results()
    assert np.array_equal(y1, y2) and np.array_equal(dx1, dx2)
    for k in g1:
        assert rel_err(g2[k], 2 * g1[k]) < 1e-6, k
    dev.runner.zero_grads()
    dev.step()
    _, _, g3, _ = dev.results()
    for k in g1:
        assert np.array_equal(g1[k], g3[k]), k   # deterministic: no floating-point atomics


def test_argument_errors_launch_nothing():
    import torch
    from paper_2605_25451_amd import binding as bm
    from paper_2605_25451_amd.runner import CaseOnDevice
    case = synth.config1()
    dev = CaseOnDevice(case)
    r = dev.runner
    bad_cu = dev.cu_host.copy(); bad_cu[1] = 0                     # empty first sequence
    with pytest.raises(bm.BmError) as e:
        bm.block_forward(r.desc, r.w, dev.x, dev.cu_dev, bad_cu, 2, 40, 40, None, dev.y, dev.saved,
                         r.scratch, r.scratch_bytes)
    assert e.value.status == bm.BM_ERR_INVALID_ARG
    with pytest.raises(bm.BmError) as e:                            # max_seqlen too small
        bm.block_forward(r.desc, r.w, dev.x, dev.cu_dev, dev.cu_host, 2, 40, 8, None, dev.y,
                         dev.saved, r.scratch, r.scratch_bytes)
    assert e.value.status == bm.BM_ERR_INVALID_ARG
    with pytest.raises(bm.BmError) as e:                            # workspace too small
        bm.block_forward(r.desc, r.w, dev.x, dev.cu_dev, dev.cu_host, 2, 40, 40, None, dev.y,
                         dev.saved, r.scratch, 16)
    assert e.value.status == bm.BM_ERR_WORKSPACE_TOO_SMALL
    with pytest.raises(bm.BmError):                                 # NULL input
        bm.block_forward(r.desc, r.w, None, dev.cu_dev, dev.cu_host, 2, 40, 40, None, dev.y,
                         dev.saved, r.scratch, r.scratch_bytes)
    torch.cuda.synchronize()
