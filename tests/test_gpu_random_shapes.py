"""Seeded random shapes through the single-operation entry points (needs a GPU): GEMM sizes drawn
around the tile edges of the matrix-core kernel (1..700, multiples of 8 so that both back ends
are eligible, plus strides wider than the matrix), attention over random packs.  Each case is
checked against the definition in fp64; the case is printed before it runs."""
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


def gemm_cases():
    rng = np.random.default_rng(2024)
    out = []
    for i in range(36):
        layout = i % 3
        M = int(rng.choice([1, 8, 16, 24, 56, 64, 72, 120, 128, 136, 248, 256, 264, 392, 520, 696]))
        N = int(rng.choice([64, 72, 128, 136, 256, 264, 392, 640]))
        K = int(rng.choice([8, 16, 56, 64, 72, 128, 200, 512, 520, 1032, 2048]))
        if layout == 2:
            M = max(8, M - M % 8)
        pad = int(rng.choice([0, 8, 64]))          # row strides wider than the matrices
        out.append((layout, M, N, K, pad))
    return out


@pytest.mark.parametrize("layout,M,N,K,pad", gemm_cases())
def test_random_gemm_bf16(layout, M, N, K, pad):
    import torch
    from paper_2605_25451_amd import binding as bm
    dtype = synth.DTYPE_BF16
    rng = np.random.default_rng(M * 31 + N * 7 + K + layout)
    a_shape = (K, M) if layout == 2 else (M, K)
    b_shape = (N, K) if layout == 0 else (K, N)
    lda, ldb, ldc = a_shape[1] + pad, b_shape[1] + pad, N + pad
    A = synth.to_storage(rng.standard_normal((a_shape[0], lda), dtype=np.float32), dtype)
    B = synth.to_storage(rng.standard_normal((b_shape[0], ldb), dtype=np.float32), dtype)
    A64, B64 = A[:, :a_shape[1]].astype(np.float64), B[:, :b_shape[1]].astype(np.float64)
    bias = synth.to_storage(rng.standard_normal(N, dtype=np.float32), dtype) if layout != 2 else None
    print(f"random gemm layout={layout} M={M} N={N} K={K} lda={lda} ldb={ldb} ldc={ldc}", flush=True)
    dA, dB = _dev(A, dtype), _dev(B, dtype)
    if layout == 2:
        C0 = rng.standard_normal((M, ldc), dtype=np.float32)
        ref = C0[:, :N].astype(np.float64) + A64.T @ B64
        dC = torch.from_numpy(C0).cuda()
    else:
        ref = (A64 @ B64.T if layout == 0 else A64 @ B64) + bias
        C0 = np.full((M, ldc), 7.0, dtype=np.float32)
        dC = _dev(C0, dtype)
    nbytes = bm.gemm_scratch_bytes(layout, M, N, K, dtype)
    scratch = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    bm.gemm(layout, dtype, M, N, K, dA, lda, dB, ldb, dC, ldc, _dev(bias, dtype) if bias is not None else None,
            scratch, nbytes)
    torch.cuda.synchronize()
    got = dC.float().cpu().numpy().astype(np.float64)
    assert rel_err(got[:, :N], ref) <= (2e-2 if layout != 2 else 1e-4)
    if pad:                                         # columns past N belong to the caller
        assert np.array_equal(got[:, N:], C0[:, N:].astype(np.float64))


def attention_cases():
    rng = np.random.default_rng(77)
    out = []
    for i in range(10):
        dh = int(rng.choice([64, 72, 128]))
        Hkv = int(rng.choice([1, 2, 4]))
        Hq = Hkv * int(rng.choice([1, 2, 4]))
        lens = [int(v) for v in rng.integers(1, 400, size=int(rng.integers(1, 6)))]
        out.append((Hq, Hkv, dh, lens, i % 2))
    return out


@pytest.mark.parametrize("Hq,Hkv,dh,lens,causal", attention_cases())
def test_random_attention_bf16(Hq, Hkv, dh, lens, causal):
    import torch
    from paper_2605_25451_amd import binding as bm
    dtype = synth.DTYPE_BF16
    rng = np.random.default_rng(sum(lens) * 3 + Hq + dh)
    cu = synth.cu_from_lengths(lens)
    T, S = int(cu[-1]), len(lens)
    W = (Hq + 2 * Hkv) * dh
    print(f"random attention Hq={Hq} Hkv={Hkv} dh={dh} lens={lens} causal={causal}", flush=True)
    qkv = synth.to_storage(rng.standard_normal((T, W), dtype=np.float32), dtype)
    d_o = synth.to_storage(rng.standard_normal((T, Hq * dh), dtype=np.float32), dtype)
    q = qkv[:, :Hq * dh].reshape(T, Hq, dh).astype(np.float64)
    k = qkv[:, Hq * dh:(Hq + Hkv) * dh].reshape(T, Hkv, dh).astype(np.float64)
    v = qkv[:, (Hq + Hkv) * dh:].reshape(T, Hkv, dh).astype(np.float64)
    ref_o = bo.attention_fwd(q, k, v, cu, bool(causal))
    rdq, rdk, rdv = bo.attention_bwd(d_o.astype(np.float64).reshape(T, Hq, dh), q, k, v, cu, bool(causal))
    dqkv = _dev(qkv, dtype)
    qd, kd, vd = dqkv[:, :Hq * dh], dqkv[:, Hq * dh:], dqkv[:, (Hq + Hkv) * dh:]
    cu_dev = torch.from_numpy(np.asarray(cu, dtype=np.int32)).cuda()
    o = torch.empty((T, Hq * dh), dtype=dqkv.dtype, device="cuda")
    lse = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
    bm.attention_forward(dtype, causal, Hq, Hkv, dh, qd, kd, vd, W, cu_dev, cu, S, T, max(lens), o, lse)
    grad = torch.empty((T, W), dtype=dqkv.dtype, device="cuda")
    nbytes = bm.attention_backward_scratch_bytes(Hq, Hkv, dh, T)
    scratch = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    bm.attention_backward(dtype, causal, Hq, Hkv, dh, qd, kd, vd, W, o, _dev(d_o, dtype), lse, cu_dev, cu, S, T,
                          max(lens), grad[:, :Hq * dh], grad[:, Hq * dh:], grad[:, (Hq + Hkv) * dh:], W, scratch, nbytes)
    torch.cuda.synchronize()
    g = grad.float().cpu().numpy().astype(np.float64)
    assert rel_err(o.float().cpu().numpy().astype(np.float64), ref_o.reshape(T, -1)) <= 2e-2
    assert rel_err(g[:, :Hq * dh], rdq.reshape(T, -1)) <= 2e-2
    assert rel_err(g[:, Hq * dh:(Hq + Hkv) * dh], rdk.reshape(T, -1)) <= 2e-2
    assert rel_err(g[:, (Hq + Hkv) * dh:], rdv.reshape(T, -1)) <= 2e-2
