"""Device-memory plumbing for context-parallel attention on one GPU: the C ranks of a
context-parallel group are run one after the other, each through the C-ABI calls a rank makes
(chunk-pair attention, merge of the partial results, chunk-pair backward, sum of the gradient
parts).  What a real group moves between GPUs (the key/value chunks round the ring, the dk/dv
parts back to their owners) is here just another tensor of the same process.  No arithmetic
happens in this file."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as bm
from . import synth
from .runner import to_device, torch_dtype

MASK_BIDIRECTIONAL, MASK_CAUSAL = 0, 1


def ring_pairs(C: int, rank: int, causal: bool):
    """(key/value chunk, mask of the pair) that `rank` sees at ring steps 0..C-1: the chunk of rank
    (rank - step) mod C.  Chunks are ascending position ranges: under a causal mask an earlier
    chunk is fully visible, the own chunk up to the diagonal, later chunks are skipped."""
    out = []
    for step in range(C):
        j = (rank - step) % C
        if causal and j > rank:
            continue
        out.append((j, MASK_CAUSAL if (causal and j == rank) else MASK_BIDIRECTIONAL))
    return out


class ContextParallelGroup:
    def __init__(self, dtype, Hq, Hkv, dh, causal, cu, C, q, k, v, d_o, device="cuda:0", ranks=None):
        """q [T, Hq*dh], k, v [T, Hkv*dh], d_o [T, Hq*dh]: fp32 numpy values representable in
        `dtype`, packed by cu; they are split into the C chunks of synth.context_chunks.
        ranks: the ranks whose query side is run (default all)."""
        self.dtype, self.Hq, self.Hkv, self.dh, self.causal, self.C = dtype, Hq, Hkv, dh, bool(causal), C
        self.S = len(cu) - 1
        self.chunks = synth.context_chunks(cu, C)
        self.ranks = list(range(C)) if ranks is None else list(ranks)
        td = torch_dtype(dtype)
        self.cu_host = [np.asarray(c, dtype=np.int32) for _, c in self.chunks]
        self.cu_dev = [torch.from_numpy(c).to(device) for c in self.cu_host]
        self.T = [int(c[-1]) for c in self.cu_host]
        pick = lambda a, r: to_device(a[r], dtype, device)
        self.q = [pick(q, r) for r, _ in self.chunks]
        self.k = [pick(k, r) for r, _ in self.chunks]
        self.v = [pick(v, r) for r, _ in self.chunks]
        self.d_o = [pick(d_o, r) for r, _ in self.chunks]
        new = lambda t, w, dt=td: torch.empty((max(t, 1), w), dtype=dt, device=device)
        self.o = [new(t, Hq * dh) for t in self.T]
        self.lse = [torch.empty((Hq, max(t, 1)), dtype=torch.float32, device=device) for t in self.T]
        self.pairs = {c: ring_pairs(C, c, self.causal) for c in self.ranks}
        self.o_part = {c: [new(self.T[c], Hq * dh) for _ in self.pairs[c]] for c in self.ranks}
        self.lse_part = {c: [torch.empty((Hq, max(self.T[c], 1)), dtype=torch.float32, device=device)
                             for _ in self.pairs[c]] for c in self.ranks}
        self.dq_part = {c: [new(self.T[c], Hq * dh) for _ in self.pairs[c]] for c in self.ranks}
        self.dk_part = {(c, j): new(self.T[j], Hkv * dh) for c in self.ranks for j, _ in self.pairs[c]}
        self.dv_part = {(c, j): new(self.T[j], Hkv * dh) for c in self.ranks for j, _ in self.pairs[c]}
        self.dq = [new(t, Hq * dh) for t in self.T]
        self.dk = [new(t, Hkv * dh) for t in self.T]
        self.dv = [new(t, Hkv * dh) for t in self.T]
        tmax = max(self.T)
        self.scratch_bytes = bm.cp_attention_backward_scratch_bytes(Hq, Hkv, dh, tmax, tmax)
        self.scratch = torch.empty(max(self.scratch_bytes, 16), dtype=torch.uint8, device=device)

    def forward(self):
        a = (self.dtype,)
        for c in self.ranks:
            for n, (j, mask) in enumerate(self.pairs[c]):
                bm.cp_attention_forward(self.dtype, mask, self.Hq, self.Hkv, self.dh, self.q[c], self.Hq * self.dh,
                                        self.k[j], self.v[j], self.Hkv * self.dh, self.cu_dev[c], self.cu_host[c],
                                        self.cu_dev[j], self.cu_host[j], self.S, self.o_part[c][n],
                                        self.lse_part[c][n])
            bm.cp_attention_merge(self.dtype, self.Hq, self.dh, self.T[c], self.o_part[c], self.lse_part[c],
                                  self.o[c], self.lse[c])

    def backward(self):
        for c in self.ranks:
            for n, (j, mask) in enumerate(self.pairs[c]):
                bm.cp_attention_backward(self.dtype, mask, self.Hq, self.Hkv, self.dh, self.q[c], self.Hq * self.dh,
                                         self.k[j], self.v[j], self.Hkv * self.dh, self.o[c], self.d_o[c],
                                         self.lse[c], self.cu_dev[c], self.cu_host[c], self.cu_dev[j],
                                         self.cu_host[j], self.S, self.dq_part[c][n], self.Hq * self.dh,
                                         self.dk_part[(c, j)], self.dv_part[(c, j)], self.Hkv * self.dh,
                                         self.scratch, self.scratch_bytes)
            bm.cp_sum_parts(self.dtype, self.T[c] * self.Hq * self.dh, self.dq_part[c], self.dq[c])
        # dk, dv of chunk j: the parts of every rank that saw it, in rank order
        for j in range(self.C):
            owners = [c for c in self.ranks if (c, j) in self.dk_part]
            if owners:
                n = self.T[j] * self.Hkv * self.dh
                bm.cp_sum_parts(self.dtype, n, [self.dk_part[(c, j)] for c in owners], self.dk[j])
                bm.cp_sum_parts(self.dtype, n, [self.dv_part[(c, j)] for c in owners], self.dv[j])

    def gather(self, per_chunk, width):
        """Chunk tensors back into the full packed order, as float64 numpy."""
        torch.cuda.synchronize()
        T = sum(self.T)
        out = np.zeros((T, width), dtype=np.float64)
        for (rows, _), t, n in zip(self.chunks, per_chunk, self.T):
            out[rows] = t[:n].detach().float().cpu().numpy().astype(np.float64)
        return out

    def gather_lse(self):
        torch.cuda.synchronize()
        out = np.zeros((self.Hq, sum(self.T)), dtype=np.float64)
        for (rows, _), t, n in zip(self.chunks, self.lse, self.T):
            out[:, rows] = t[:, :n].detach().cpu().numpy().astype(np.float64)
        return out
