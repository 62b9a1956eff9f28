"""Single-operation parity through the C-ABI (needs a GPU): GEMM layouts and
attention against their plain definitions."""
import numpy as np
import pytest

from oracle import block_oracle as bo
from paper_2605_25451_amd import synth

pytestmark = pytest.mark.gpu


def rel_err(got, ref):
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def _dev(a, dtype):
    from paper_2605_25451_amd.runner import to_device
    return to_device(a, dtype)


GEMM_SHAPES = [
    # M, N, K  (tile multiples, ragged M, ragged K for the weight-gradient layout, tiny)
    (512, 512, 256), (300, 384, 512), (1000, 1152, 1152), (777, 3456, 1152), (256, 256, 64),
    (2048, 1024, 1000 * 8), (40, 64, 24), (515, 640, 1096),
    # skinny outputs with a long contraction (k ranges split over workgroups)
    (32, 1152, 6912), (5, 200, 3001),
    # few rows against wide weights (the per-sample modulation products): few output rows,
    # and for the weight-gradient layout also a contraction of only a few rows
    (16, 1152, 1152), (1, 64, 64), (33, 200, 136), (16, 512, 2048), (640, 384, 16), (8, 64, 64),
    (64, 64, 8), (24, 3072, 4608),
    # enough 256x256 tiles to fill the chip with a contraction of one, two, three and five k slices:
    # every entry path of the large-tile kernel's software pipeline (its first slice, the slices
    # that still fetch, the last two) plus a ragged last slice
    (4096, 4096, 64), (4096, 4096, 128), (4096, 4096, 192), (4096, 4096, 328),
]


@pytest.mark.parametrize("dtype", [synth.DTYPE_BF16, synth.DTYPE_FP32], ids=["bf16", "fp32"])
@pytest.mark.parametrize("layout", [0, 1, 2], ids=["NT", "NN", "TN"])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_matches_definition(layout, dtype, M, N, K):
    import torch
    from paper_2605_25451_amd import binding as bm
    rng = np.random.default_rng(M * 7 + N * 3 + K + layout)
    a_shape = (K, M) if layout == 2 else (M, K)
    b_shape = (N, K) if layout == 0 else (K, N)
    A = synth.to_storage(rng.standard_normal(a_shape, dtype=np.float32), dtype)
    B = synth.to_storage(rng.standard_normal(b_shape, dtype=np.float32), dtype)
    bias = synth.to_storage(rng.standard_normal(N, dtype=np.float32), dtype) if layout != 2 else None
    A64, B64 = A.astype(np.float64), B.astype(np.float64)
    if layout == 0:
        ref = A64 @ B64.T + bias
    elif layout == 1:
        ref = A64 @ B64 + bias
    else:
        C0 = rng.standard_normal((M, N), dtype=np.float32)
        ref = C0.astype(np.float64) + A64.T @ B64
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    if layout == 2:
        dC = torch.from_numpy(C0).cuda()
    else:
        dC = torch.empty((M, N), dtype=dA.dtype, device="cuda")
    dbias = _dev(bias, dtype) if bias is not None else None
    nbytes = bm.gemm_scratch_bytes(layout, M, N, K, dtype)
    scratch = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    print(f"gemm layout={layout} dtype={dtype} M={M} N={N} K={K} scratch={nbytes}", flush=True)
    bm.gemm(layout, dtype, M, N, K, dA, a_shape[1], dB, b_shape[1], dC, N, dbias, scratch, nbytes)
    torch.cuda.synchronize()
    got = dC.float().cpu().numpy().astype(np.float64)
    tol = 1e-5 if dtype == synth.DTYPE_FP32 else (2e-2 if layout != 2 else 1e-4)
    assert rel_err(got, ref) <= tol


ATTN_CASES = [
    # dtype, Hq, Hkv, dh, lens, causal
    (synth.DTYPE_FP32, 4, 4, 16, [16, 24], 0),
    (synth.DTYPE_FP32, 4, 2, 16, [1, 130, 37], 1),
    (synth.DTYPE_BF16, 4, 4, 64, [300, 257, 143, 1, 67], 0),
    (synth.DTYPE_BF16, 4, 4, 64, [129, 500, 64], 1),
    (synth.DTYPE_BF16, 8, 2, 128, [333, 64, 515, 7], 1),
    (synth.DTYPE_BF16, 4, 4, 128, [200, 1100], 0),
    (synth.DTYPE_BF16, 2, 2, 72, [256, 256, 100], 0),
    (synth.DTYPE_BF16, 4, 2, 72, [130, 77, 1], 1),
    (synth.DTYPE_BF16, 2, 1, 128, [2049], 1),
    # many sequences: the tile walk takes its order from a 64-entry table read 16 positions at a
    # time (longest sequences first without a mask, pack order under a causal one) and walks the
    # offsets themselves past 64 sequences
    (synth.DTYPE_BF16, 2, 2, 64, [40 + 13 * (i % 7) for i in range(16)], 0),
    (synth.DTYPE_BF16, 2, 1, 64, [150 - 8 * i for i in range(17)], 1),
    (synth.DTYPE_BF16, 2, 2, 64, [1 + (37 * i) % 131 for i in range(64)], 0),
    (synth.DTYPE_BF16, 2, 2, 128, [1 + (53 * i) % 140 for i in range(33)], 1),
    (synth.DTYPE_BF16, 2, 2, 64, [1 + (29 * i) % 97 for i in range(70)], 0),
    (synth.DTYPE_BF16, 2, 1, 72, [130 if i == 40 else 9 + i % 5 for i in range(65)], 1),
]


@pytest.mark.parametrize("dtype,Hq,Hkv,dh,lens,causal", ATTN_CASES)
def test_attention_matches_definition(dtype, Hq, Hkv, dh, lens, causal):
    import torch
    from paper_2605_25451_amd import binding as bm
    rng = np.random.default_rng(sum(lens) + Hq + dh)
    cu = synth.cu_from_lengths(lens)
    T, S = int(cu[-1]), len(lens)
    W = (Hq + 2 * Hkv) * dh
    qkv = synth.to_storage(rng.standard_normal((T, W), dtype=np.float32), dtype)
    d_o = synth.to_storage(rng.standard_normal((T, Hq * dh), dtype=np.float32), dtype)
    q = qkv[:, :Hq * dh].reshape(T, Hq, dh).astype(np.float64)
    k = qkv[:, Hq * dh:(Hq + Hkv) * dh].reshape(T, Hkv, dh).astype(np.float64)
    v = qkv[:, (Hq + Hkv) * dh:].reshape(T, Hkv, dh).astype(np.float64)
    ref_o = bo.attention_fwd(q, k, v, cu, bool(causal))
    dq, dk, dv = bo.attention_bwd(d_o.reshape(T, Hq, dh).astype(np.float64), q, k, v, cu, bool(causal))
    ref_d = np.concatenate([dq.reshape(T, -1), dk.reshape(T, -1), dv.reshape(T, -1)], axis=1)
    # log-sum-exp of the scaled scores, from the definition
    ref_lse = np.zeros((Hq, T))
    for s in range(S):
        lo, hi = cu[s], cu[s + 1]
        for a in range(Hq):
            sc = q[lo:hi, a] @ k[lo:hi, a // (Hq // Hkv)].T / np.sqrt(dh)
            if causal:
                sc = np.where(np.tril(np.ones_like(sc, dtype=bool)), sc, -np.inf)
            m = sc.max(-1)
            ref_lse[a, lo:hi] = m + np.log(np.exp(sc - m[:, None]).sum(-1))

    es = 2 if dtype == synth.DTYPE_BF16 else 4
    dqkv = _dev(qkv, dtype)
    ddo = _dev(d_o, dtype)
    cu_dev = torch.from_numpy(cu).cuda()
    o = torch.empty((T, Hq * dh), dtype=dqkv.dtype, device="cuda")
    lse = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
    base = dqkv.data_ptr()
    qp, kp, vp = base, base + Hq * dh * es, base + (Hq + Hkv) * dh * es
    print(f"attention dtype={dtype} Hq={Hq} Hkv={Hkv} dh={dh} lens={lens} causal={causal}", flush=True)
    bm.attention_forward(dtype, causal, Hq, Hkv, dh, qp, kp, vp, W, cu_dev, cu, S, T, max(lens), o, lse)
    torch.cuda.synchronize()
    tol = 1e-5 if dtype == synth.DTYPE_FP32 else 2e-2
    assert rel_err(o.float().cpu().numpy().reshape(T, Hq, dh), ref_o) <= tol
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= (1e-4 if dtype == synth.DTYPE_FP32 else 2e-2)
    grads = torch.empty_like(dqkv)
    gb = grads.data_ptr()
    nb = bm.attention_backward_scratch_bytes(Hq, Hkv, dh, T)
    scratch = torch.empty(nb, dtype=torch.uint8, device="cuda")
    bm.attention_backward(dtype, causal, Hq, Hkv, dh, qp, kp, vp, W, o, ddo, lse, cu_dev, cu, S, T,
                          max(lens), gb, gb + Hq * dh * es, gb + (Hq + Hkv) * dh * es, W, scratch, nb)
    torch.cuda.synchronize()
    got = grads.float().cpu().numpy().astype(np.float64)
    for name, sl in (("dq", slice(0, Hq * dh)), ("dk", slice(Hq * dh, (Hq + Hkv) * dh)),
                     ("dv", slice((Hq + Hkv) * dh, W))):
        assert rel_err(got[:, sl], ref_d[:, sl]) <= tol, name


def test_lds_and_issue_yardsticks_run_and_leave_their_buffers_alone():
    """The measuring kernels behind bench.py's `measured_peaks` launch, finish, and write nothing:
    the source buffer of the direct loads and the output word keep their contents."""
    import torch
    from paper_2605_25451_amd import binding as bm
    src = torch.full((1 << 20,), 7, dtype=torch.uint8, device="cuda")
    word = torch.full((4,), 5, dtype=torch.int32, device="cuda")
    out = torch.full((4,), 3.0, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    rates = {}
    for what, nbytes in ((1, 16384), (2, 16384), (4, 8192), (8, 8192), (5, 24576), (9, 24576)):
        print(f"probe_lds what={what}", flush=True)
        bm.probe_lds(what, 10, src, src.numel(), word)
        e0.record(); bm.probe_lds(what, 500, src, src.numel(), word); e1.record(); torch.cuda.synchronize()
        rates[what] = 2 * 4 * 500 * nbytes / (e0.elapsed_time(e1) * 1e6)
    for nv in (0, 4, 8):
        print(f"probe_issue n_valu={nv}", flush=True)
        bm.probe_issue(nv, 100, out)
    torch.cuda.synchronize()
    assert int(src.min()) == 7 and int(src.max()) == 7
    assert word.cpu().tolist() == [5, 5, 5, 5] and out.cpu().tolist() == [3.0, 3.0, 3.0, 3.0]
    # bytes per ns and CU: anything between a crawl and what 256 bytes per clock could give
    assert all(5.0 < r < 1000.0 for r in rates.values()), rates
