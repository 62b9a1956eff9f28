"""Attention backward with the library's built-in workspace (the entry point for callers that
cannot allocate) against the caller-workspace entry point, through the C-ABI (needs a GPU).

Both run the same kernels, so the results have to agree bit for bit, which is stronger than the
floating-point tolerance; the built-in workspace keeps the previous call's contents, so every case
is two calls in a row, the second on a smaller pack."""
import numpy as np
import pytest

from paper_2605_25451_amd import synth

pytestmark = pytest.mark.gpu


def _run_pair(dtype, Hq, Hkv, dh, lens, causal, seed):
    """forward, then backward through both entry points; returns (static, caller) gradients"""
    import torch
    from paper_2605_25451_amd import binding as bm
    from paper_2605_25451_amd.runner import to_device
    rng = np.random.default_rng(seed)
    cu = synth.cu_from_lengths(lens)
    T, S = int(cu[-1]), len(lens)
    W = (Hq + 2 * Hkv) * dh
    es = 2 if dtype == synth.DTYPE_BF16 else 4
    qkv = to_device(synth.to_storage(rng.standard_normal((T, W), dtype=np.float32), dtype), dtype)
    d_o = to_device(synth.to_storage(rng.standard_normal((T, Hq * dh), dtype=np.float32), dtype), dtype)
    cu_dev = torch.from_numpy(cu).cuda()
    o = torch.empty((T, Hq * dh), dtype=qkv.dtype, device="cuda")
    lse = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
    base = qkv.data_ptr()
    qp, kp, vp = base, base + Hq * dh * es, base + (Hq + Hkv) * dh * es
    bm.attention_forward(dtype, causal, Hq, Hkv, dh, qp, kp, vp, W, cu_dev, cu, S, T, max(lens), o, lse)

    def split(g):
        b = g.data_ptr()
        return b, b + Hq * dh * es, b + (Hq + Hkv) * dh * es

    # filled with a pattern first, so an output row a call failed to write would show
    g_static = torch.full_like(qkv, 3.0)
    g_caller = torch.full_like(qkv, -5.0)
    nb = bm.attention_backward_scratch_bytes(Hq, Hkv, dh, T)
    assert nb <= bm.attention_backward_static_capacity()
    print(f"static attention backward dtype={dtype} Hq={Hq} Hkv={Hkv} dh={dh} lens={lens} causal={causal} "
          f"workspace={nb}", flush=True)
    bm.attention_backward_static(dtype, causal, Hq, Hkv, dh, qp, kp, vp, W, o, d_o, lse, cu_dev, cu, S, T,
                                 max(lens), *split(g_static), W)
    torch.cuda.synchronize()
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    bm.attention_backward(dtype, causal, Hq, Hkv, dh, qp, kp, vp, W, o, d_o, lse, cu_dev, cu, S, T,
                          max(lens), *split(g_caller), W, ws, nb)
    torch.cuda.synchronize()
    return g_static.float().cpu().numpy(), g_caller.float().cpu().numpy()


PAIRS = [
    # dtype, Hq, Hkv, dh, causal, first pack, second (smaller) pack
    # grouped-query attention over a short pack: the q heads of a group are split over workgroups and
    # leave fp32 partials in the workspace, behind the delta plane
    (synth.DTYPE_BF16, 8, 2, 128, 1, [333, 64, 515, 7], [130, 61]),
    (synth.DTYPE_BF16, 4, 4, 64, 0, [300, 257, 143, 1, 67], [129]),
    (synth.DTYPE_BF16, 4, 2, 72, 1, [130, 77, 1], [40, 3]),
    (synth.DTYPE_FP32, 4, 2, 16, 1, [1, 130, 37], [16, 24]),
]


@pytest.mark.parametrize("dtype,Hq,Hkv,dh,causal,first,second", PAIRS)
def test_static_workspace_matches_caller_workspace(dtype, Hq, Hkv, dh, causal, first, second):
    for i, lens in enumerate((first, second)):
        got, ref = _run_pair(dtype, Hq, Hkv, dh, lens, causal, seed=11 + i)
        assert np.isfinite(ref).all()
        assert np.array_equal(got, ref), f"call {i}: max diff {np.abs(got - ref).max()}"


def test_static_workspace_rejects_oversized_packs():
    import torch
    from paper_2605_25451_amd import binding as bm
    cap = bm.attention_backward_static_capacity()
    assert cap == 64 << 20
    Hq, Hkv, dh = 32, 8, 128
    T = 8192
    assert bm.attention_backward_scratch_bytes(Hq, Hkv, dh, T) > cap
    dummy = torch.zeros(64, dtype=torch.float32, device="cuda")
    cu = np.array([0, T], dtype=np.int32)
    p = dummy.data_ptr()
    with pytest.raises(bm.BmError) as e:
        bm.attention_backward_static(synth.DTYPE_BF16, 1, Hq, Hkv, dh, p, p, p, (Hq + 2 * Hkv) * dh, dummy, dummy,
                                     dummy, dummy, cu, 1, T, T, p, p, p, (Hq + 2 * Hkv) * dh)
    assert e.value.status == -3          # BM_ERR_WORKSPACE_TOO_SMALL: nothing was launched
