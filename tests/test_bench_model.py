"""The work model behind bench.py's TFLOP/s figure (CPU only): algorithmic flops of a block
are 3 x the forward GEMM flops + 3.5 x the forward attention flops, counting only unmasked
pairs inside the sequences."""
import numpy as np

import bench
from paper_2605_25451_amd import synth


def test_config2_flops_match_the_closed_form():
    case = synth.config2()
    cfg, cu = case.cfg, np.asarray(case.cu_seqlens)
    T = int(cu[-1])
    assert (T, cfg.hidden, cfg.n_q_heads, cfg.head_dim, cfg.mlp_hidden) == (16384, 1024, 16, 64, 4096)
    gemm, attn = bench.algorithmic_flops(cfg, cu)
    # QKV 2*T*d*3d, O 2*T*d*d, MLP 2 * 2*T*d*F
    assert gemm == 2.0 * T * 1024 * 3072 + 2.0 * T * 1024 * 1024 + 2 * 2.0 * T * 1024 * 4096
    assert abs(gemm - 412.3e9) < 0.1e9
    L = np.diff(cu).astype(np.float64)
    assert attn == 4.0 * 64 * 16 * float((L * L).sum())          # bidirectional: every pair of a sequence
    assert 3 * gemm + 3.5 * attn == case_total(case)


def case_total(case):
    gemm, attn = bench.algorithmic_flops(case.cfg, np.asarray(case.cu_seqlens))
    return 3 * gemm + 3.5 * attn


def test_causal_counts_the_lower_triangle_and_swiglu_three_matrices():
    case = synth.config3()
    cfg, cu = case.cfg, np.asarray(case.cu_seqlens)
    T = int(cu[-1])
    gemm, attn = bench.algorithmic_flops(cfg, cu)
    d, F = cfg.hidden, cfg.mlp_hidden
    assert gemm == 2.0 * T * d * 3 * d + 2.0 * T * d * d + 3 * 2.0 * T * d * F
    L = np.diff(cu).astype(np.float64)
    assert attn == 4.0 * cfg.head_dim * cfg.n_q_heads * float((L * (L + 1) / 2).sum())
