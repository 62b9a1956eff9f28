"""CPU oracle for one GPU's share of context-parallel attention.

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and smoke/bench baseline
legs), never by the product path, and sharing no code with it.

Sec. 3.3 "Context parallelism": the tokens of every sequence are partitioned
over the ranks of a context-parallel group and attention is computed in
parallel (the ring-attention method the paper cites).  The paper gives no
arithmetic; what a rank computes follows from the definition of softmax
attention.  A rank holds the queries of its chunk of every sequence and is
handed, one after the other, the keys/values of the chunks; for one
(query chunk, key/value chunk) pair it produces, per query row i and head,

    s_ij  = <q_i, k_j> / sqrt(dh)              over the keys j of THAT chunk
    lse_i = log sum_j exp(s_ij)                (-inf when the chunk has no visible key)
    o_i   = sum_j exp(s_ij - lse_i) v_j        (0 then)

and the partial results of all chunks are merged by

    lse_i = log sum_c exp(lse_i^c),    o_i = sum_c exp(lse_i^c - lse_i) o_i^c ,

which equals attention over all keys (the merged softmax weights are
exp(s_ij - lse_i)).  Under a causal mask a chunk that lies wholly before the
query chunk is fully visible, the query chunk itself is visible up to the
diagonal (key position <= query position, both counted inside the chunk), and
later chunks are not visible and are skipped.

Backward of one pair, with the MERGED lse and the merged output o of the query
rows:  p_ij = exp(s_ij - lse_i),  delta_i = <do_i, o_i>,  dv_j = sum_i p_ij do_i,
ds_ij = p_ij (<do_i, v_j> - delta_i),  dq_i = sum_j ds_ij k_j / sqrt(dh),
dk_j = sum_i ds_ij q_i / sqrt(dh); dq sums over the key/value chunks, dk and dv
sum over the query chunks.

Pins: tests/test_oracle_cp_attention.py (merged chunk results equal plain
attention of the block oracle, forward and backward, for every partition;
closed form of a two-key merge; an empty part is the identity of the merge;
merge order does not matter).
"""
from __future__ import annotations

import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def chunk_forward(q, k, v, cu_q, cu_k, causal):
    """q:[Tq,Hq,dh] packed by cu_q; k,v:[Tk,Hkv,dh] packed by cu_k (same number of sequences).
    causal: the two chunks cover the same positions (cu_q == cu_k).
    Returns (o [Tq,Hq,dh], lse [Hq,Tq])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    Tq, Hq, dh = q.shape
    group = Hq // k.shape[1]
    o = np.zeros_like(q)
    lse = np.full((Hq, Tq), -np.inf)
    for s in range(len(cu_q) - 1):
        a0, a1 = int(cu_q[s]), int(cu_q[s + 1])
        b0, b1 = int(cu_k[s]), int(cu_k[s + 1])
        if a1 == a0 or b1 == b0:
            continue
        for h in range(Hq):
            sc = q[a0:a1, h] @ k[b0:b1, h // group].T / np.sqrt(dh)
            if causal:
                assert a1 - a0 == b1 - b0
                sc = np.where(np.tril(np.ones(sc.shape, dtype=bool)), sc, -np.inf)
            m = sc.max(axis=1, keepdims=True)
            e = np.exp(sc - m)
            z = e.sum(axis=1, keepdims=True)
            lse[h, a0:a1] = (m + np.log(z))[:, 0]
            o[a0:a1, h] = (e / z) @ v[b0:b1, h // group]
    return o, lse


def merge(o_parts, lse_parts):
    """o_parts: list of [Tq,Hq,dh]; lse_parts: list of [Hq,Tq].  Returns (o, lse)."""
    L = np.stack([_f64(l) for l in lse_parts])             # [C,Hq,Tq]
    m = L.max(axis=0)
    safe = np.where(np.isfinite(m), m, 0.0)
    with np.errstate(divide="ignore"):
        lse = safe + np.log(np.exp(L - safe).sum(axis=0))   # -inf where every part is empty
    o = np.zeros_like(_f64(o_parts[0]))
    for op, lp in zip(o_parts, L):
        w = np.where(np.isfinite(lp), np.exp(lp - np.where(np.isfinite(lse), lse, 0.0)), 0.0)   # [Hq,Tq]
        o += w.T[:, :, None] * _f64(op)
    return o, lse


def chunk_backward(q, k, v, o, d_o, lse, cu_q, cu_k, causal):
    """o, d_o [Tq,Hq,dh] and lse [Hq,Tq] are the MERGED output, its gradient and the merged lse of
    the query rows.  Returns this pair's (dq [Tq,Hq,dh], dk, dv [Tk,Hkv,dh])."""
    q, k, v, o, d_o, lse = _f64(q), _f64(k), _f64(v), _f64(o), _f64(d_o), _f64(lse)
    Tq, Hq, dh = q.shape
    group = Hq // k.shape[1]
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    scale = 1.0 / np.sqrt(dh)
    for s in range(len(cu_q) - 1):
        a0, a1 = int(cu_q[s]), int(cu_q[s + 1])
        b0, b1 = int(cu_k[s]), int(cu_k[s + 1])
        if a1 == a0 or b1 == b0:
            continue
        for h in range(Hq):
            g = h // group
            sc = q[a0:a1, h] @ k[b0:b1, g].T * scale
            p = np.exp(sc - lse[h, a0:a1, None])
            if causal:
                p = np.where(np.tril(np.ones(p.shape, dtype=bool)), p, 0.0)
            delta = (d_o[a0:a1, h] * o[a0:a1, h]).sum(axis=1, keepdims=True)
            dv[b0:b1, g] += p.T @ d_o[a0:a1, h]
            ds = p * (d_o[a0:a1, h] @ v[b0:b1, g].T - delta)
            dq[a0:a1, h] = ds @ k[b0:b1, g] * scale
            dk[b0:b1, g] += ds.T @ q[a0:a1, h] * scale
    return dq, dk, dv


def visible_pairs(C, causal):
    """(query chunk c, key/value chunk j, causal flag of the pair) in ring order: at step t rank c
    holds the keys/values of chunk (c - t) mod C.  Chunks are contiguous position ranges in
    ascending order, so under a causal mask chunk j is visible to chunk c iff j <= c."""
    out = []
    for t in range(C):
        for c in range(C):
            j = (c - t) % C
            if causal and j > c:
                continue
            out.append((c, j, bool(causal and j == c)))
    return out
