"""Pins for the context-parallel attention oracle (CPU only): merged chunk results equal plain
attention (forward and backward) for every partition, closed forms of the merge."""
import numpy as np
import pytest

from oracle import block_oracle as bo
from oracle import cp_attention_oracle as co
from paper_2605_25451_amd import synth


def draw(lens, Hq, Hkv, dh, seed):
    rng = np.random.default_rng(seed)
    cu = synth.cu_from_lengths(lens)
    T = int(cu[-1])
    q = rng.standard_normal((T, Hq, dh))
    k = rng.standard_normal((T, Hkv, dh))
    v = rng.standard_normal((T, Hkv, dh))
    d_o = rng.standard_normal((T, Hq, dh))
    return cu, q, k, v, d_o


def ring_forward(cu, q, k, v, C, causal):
    chunks = synth.context_chunks(cu, C)
    parts = {c: ([], []) for c in range(C)}
    for c, j, diag in co.visible_pairs(C, causal):
        rq, cq = chunks[c]
        rk, ck = chunks[j]
        o, lse = co.chunk_forward(q[rq], k[rk], v[rk], cq, ck, diag)
        parts[c][0].append(o); parts[c][1].append(lse)
    o_full = np.zeros_like(q)
    lse_full = np.zeros((q.shape[1], q.shape[0]))
    for c in range(C):
        o, lse = co.merge(*parts[c])
        o_full[chunks[c][0]] = o
        lse_full[:, chunks[c][0]] = lse
    return o_full, lse_full


CASES = [([7, 12, 1, 30], 4, 2, 8), ([64], 2, 2, 4), ([3, 2, 5], 3, 1, 8), ([33, 17], 4, 4, 16)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("C", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("lens,Hq,Hkv,dh", CASES)
def test_merged_chunks_equal_plain_attention(lens, Hq, Hkv, dh, C, causal):
    cu, q, k, v, _ = draw(lens, Hq, Hkv, dh, 5 + C)
    o, lse = ring_forward(cu, q, k, v, C, causal)
    ref = bo.attention_fwd(q, k, v, cu, causal)
    assert np.abs(o - ref).max() <= 1e-12
    # lse against its definition on one sequence and head
    lo, hi = int(cu[-2]), int(cu[-1])
    sc = q[lo:hi, 0] @ k[lo:hi, 0].T / np.sqrt(dh)
    if causal:
        sc = np.where(np.tril(np.ones(sc.shape, dtype=bool)), sc, -np.inf)
    assert np.abs(lse[0, lo:hi] - np.log(np.exp(sc).sum(axis=1))).max() <= 1e-12


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("C", [2, 3, 4])
@pytest.mark.parametrize("lens,Hq,Hkv,dh", CASES)
def test_summed_chunk_gradients_equal_plain_attention_backward(lens, Hq, Hkv, dh, C, causal):
    cu, q, k, v, d_o = draw(lens, Hq, Hkv, dh, 9 + C)
    o, lse = ring_forward(cu, q, k, v, C, causal)
    chunks = synth.context_chunks(cu, C)
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    for c, j, diag in co.visible_pairs(C, causal):
        rq, cq = chunks[c]
        rk, ck = chunks[j]
        a, b, d = co.chunk_backward(q[rq], k[rk], v[rk], o[rq], d_o[rq], lse[:, rq], cq, ck, diag)
        dq[rq] += a; dk[rk] += b; dv[rk] += d
    rdq, rdk, rdv = bo.attention_bwd(d_o, q, k, v, cu, causal)
    for got, ref in ((dq, rdq), (dk, rdk), (dv, rdv)):
        assert np.abs(got - ref).max() <= 1e-11 * max(1.0, np.abs(ref).max())


def test_two_single_key_parts_merge_to_a_two_way_softmax():
    # one query, parts of one key each: o^c = v_c, lse^c = s_c, so the merge is softmax(s) . v
    s = np.array([0.3, -1.1])
    v = np.array([[1.0, 2.0], [-3.0, 0.5]])
    o, lse = co.merge([v[0].reshape(1, 1, 2), v[1].reshape(1, 1, 2)],
                      [np.array([[s[0]]]), np.array([[s[1]]])])
    w = np.exp(s) / np.exp(s).sum()
    assert np.allclose(o[0, 0], w[0] * v[0] + w[1] * v[1], atol=1e-15)
    assert np.isclose(lse[0, 0], np.log(np.exp(s).sum()), atol=1e-15)


def test_merge_ignores_empty_parts_and_order():
    rng = np.random.default_rng(3)
    o = [rng.standard_normal((5, 2, 4)) for _ in range(3)]
    l = [rng.standard_normal((2, 5)) for _ in range(3)]
    base_o, base_l = co.merge(o, l)
    empty_o, empty_l = np.zeros((5, 2, 4)), np.full((2, 5), -np.inf)
    o2, l2 = co.merge([o[2], empty_o, o[0], o[1]], [l[2], empty_l, l[0], l[1]])
    assert np.abs(o2 - base_o).max() <= 1e-14 and np.abs(l2 - base_l).max() <= 1e-14
    # nested merge = flat merge
    o01, l01 = co.merge(o[:2], l[:2])
    o3, l3 = co.merge([o01, o[2]], [l01, l[2]])
    assert np.abs(o3 - base_o).max() <= 1e-14 and np.abs(l3 - base_l).max() <= 1e-14
    # all parts empty: zero output, lse = -inf, nothing undefined
    oe, le = co.merge([empty_o, empty_o], [empty_l, empty_l])
    assert np.all(oe == 0.0) and np.all(np.isneginf(le))


def test_chunk_forward_empty_key_chunk():
    cu_q = synth.cu_from_lengths([3, 2])
    cu_k = synth.cu_from_lengths([0, 4])
    rng = np.random.default_rng(4)
    q = rng.standard_normal((5, 2, 4)); k = rng.standard_normal((4, 1, 4)); v = rng.standard_normal((4, 1, 4))
    o, lse = co.chunk_forward(q, k, v, cu_q, cu_k, False)
    assert np.all(o[:3] == 0.0) and np.all(np.isneginf(lse[:, :3])) and np.all(np.isfinite(lse[:, 3:]))


def test_partition_covers_every_row_once():
    cu = synth.cu_from_lengths([7, 1, 30, 2])
    for C in (1, 2, 3, 4, 8):
        chunks = synth.context_chunks(cu, C)
        rows = np.concatenate([r for r, _ in chunks])
        assert sorted(rows.tolist()) == list(range(int(cu[-1])))
        for r, c in chunks:
            assert int(c[-1]) == len(r) and len(c) == len(cu)
