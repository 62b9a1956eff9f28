"""Device-memory plumbing around the C-ABI calls: holds one block's parameters,
gradient buffers and workspaces as torch device tensors and forwards pointers.
No arithmetic happens here.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import binding as bm
from . import synth


def torch_dtype(dtype: int):
    return torch.bfloat16 if dtype == synth.DTYPE_BF16 else torch.float32


def to_device(a: np.ndarray, dtype: int, device="cuda:0") -> torch.Tensor:
    """fp32 numpy values (already representable in the storage type) -> device tensor."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device).to(torch_dtype(dtype)).contiguous()


class BlockRunner:
    """One block on one GPU: parameters, fp32 gradient accumulators, workspaces."""

    def __init__(self, cfg: synth.BlockConfig, params: Dict[str, np.ndarray], max_T: int, max_S: int,
                 device="cuda:0"):
        self.cfg = cfg
        self.device = device
        self.desc = bm.make_desc(cfg)
        self.params = {k: to_device(v, cfg.dtype, device) for k, v in params.items()}
        self.grads = {k: torch.zeros(v.shape, dtype=torch.float32, device=device)
                      for k, v in self.params.items()}
        self.w = bm.make_params(self.params)
        self.g = bm.make_params(self.grads)
        self.max_T, self.max_S = max_T, max_S
        saved, scratch = bm.block_sizes(self.desc, max_T, max_S, max_T)
        self.saved_bytes, self.scratch_bytes = saved, scratch
        self.scratch = torch.empty(scratch, dtype=torch.uint8, device=device)

    def new_saved(self) -> torch.Tensor:
        return torch.empty(self.saved_bytes, dtype=torch.uint8, device=self.device)

    def zero_grads(self):
        for g in self.grads.values():
            g.zero_()

    def forward(self, x, cu_dev, cu_host, cond, y, saved):
        cu_host = np.asarray(cu_host, dtype=np.int32)
        S, T = len(cu_host) - 1, int(cu_host[-1])
        max_len = int(np.max(np.diff(cu_host)))
        bm.block_forward(self.desc, self.w, x, cu_dev, cu_host, S, T, max_len, cond, y, saved,
                         self.scratch, self.scratch_bytes)

    def backward(self, x, dy, cu_dev, cu_host, cond, saved, dx, dcond):
        cu_host = np.asarray(cu_host, dtype=np.int32)
        S, T = len(cu_host) - 1, int(cu_host[-1])
        max_len = int(np.max(np.diff(cu_host)))
        bm.block_backward(self.desc, self.w, x, dy, cu_dev, cu_host, S, T, max_len, cond, saved, dx,
                          self.g, dcond, self.scratch, self.scratch_bytes)


class CaseOnDevice:
    """A synth.BlockCase resident in HBM with output buffers."""

    def __init__(self, case: synth.BlockCase, device="cuda:0", runner: Optional[BlockRunner] = None):
        cfg = case.cfg
        self.case = case
        self.runner = runner or BlockRunner(cfg, case.params, case.T, case.S, device)
        self.cu_host = np.asarray(case.cu_seqlens, dtype=np.int32)
        self.cu_dev = torch.from_numpy(self.cu_host).to(device)
        self.x = to_device(case.x, cfg.dtype, device)
        self.dy = to_device(case.dy, cfg.dtype, device)
        self.cond = to_device(case.cond, cfg.dtype, device) if case.cond is not None else None
        self.y = torch.empty_like(self.x)
        self.dx = torch.empty_like(self.x)
        self.dcond = torch.empty_like(self.cond) if self.cond is not None else None
        self.saved = self.runner.new_saved()

    def forward(self):
        self.runner.forward(self.x, self.cu_dev, self.cu_host, self.cond, self.y, self.saved)

    def backward(self):
        self.runner.backward(self.x, self.dy, self.cu_dev, self.cu_host, self.cond, self.saved,
                             self.dx, self.dcond)

    def step(self):
        self.forward()
        self.backward()

    def moe_routing(self):
        """(experts int32 [T, top_k], gates fp32 [T, top_k]) the forward left in ``saved``, as numpy arrays."""
        torch.cuda.synchronize()
        T, S, k = self.case.T, self.case.S, self.case.cfg.top_k
        e_ptr, g_ptr = bm.block_moe_routing(self.runner.desc, T, S, self.saved)
        base = self.saved.data_ptr()
        n = T * k * 4
        experts = self.saved[e_ptr - base:e_ptr - base + n].view(torch.int32).reshape(T, k)
        gates = self.saved[g_ptr - base:g_ptr - base + n].view(torch.float32).reshape(T, k)
        return experts.cpu().numpy(), gates.cpu().numpy()

    def results(self):
        """(y, dx, grads, dcond) as float64 numpy arrays."""
        torch.cuda.synchronize()
        f = lambda t: None if t is None else t.detach().float().cpu().numpy().astype(np.float64)
        return f(self.y), f(self.dx), {k: f(v) for k, v in self.runner.grads.items()}, f(self.dcond)


class TwoStreamOnDevice:
    """A synth.TwoStreamCase resident in HBM: both streams' tokens, parameters, fp32 gradient
    accumulators, outputs and workspaces, forwarded to bm_mmdit_forward / bm_mmdit_backward."""

    def __init__(self, case: synth.TwoStreamCase, device="cuda:0", qk_norm_eps: float = 1e-6):
        cfg = case.cfg
        self.case = case
        self.desc = bm.make_mmdit_desc(cfg, case.qk_norm, qk_norm_eps)
        self.params = [{k: to_device(v, cfg.dtype, device) for k, v in p.items()} for p in case.params]
        self.grads = [{k: torch.zeros(v.shape, dtype=torch.float32, device=device) for k, v in p.items()}
                      for p in self.params]
        self.w = bm.make_mmdit_params(self.params)
        self.g = bm.make_mmdit_params(self.grads)
        self.cu_host = [np.asarray(c, dtype=np.int32) for c in case.cu]
        self.cu_dev = [torch.from_numpy(c).to(device) for c in self.cu_host]
        self.S = case.S
        self.x = [to_device(a, cfg.dtype, device) for a in case.x]
        self.dy = [to_device(a, cfg.dtype, device) for a in case.dy]
        self.cond = to_device(case.cond, cfg.dtype, device)
        self.y = [torch.empty_like(a) for a in self.x]
        self.dx = [torch.empty_like(a) for a in self.x]
        self.dcond = torch.empty_like(self.cond)
        saved, scratch = bm.mmdit_sizes(self.desc, int(self.cu_host[0][-1]), int(self.cu_host[1][-1]), self.S)
        self.saved_bytes, self.scratch_bytes = saved, scratch
        self.saved = torch.empty(saved, dtype=torch.uint8, device=device)
        self.scratch = torch.empty(scratch, dtype=torch.uint8, device=device)

    def zero_grads(self):
        for gs in self.grads:
            for g in gs.values():
                g.zero_()

    def forward(self):
        bm.mmdit_forward(self.desc, self.w, self.x[0], self.x[1], self.cu_dev[0], self.cu_host[0], self.cu_dev[1],
                         self.cu_host[1], self.S, self.cond, self.y[0], self.y[1], self.saved, self.scratch,
                         self.scratch_bytes)

    def backward(self):
        bm.mmdit_backward(self.desc, self.w, self.x[0], self.x[1], self.dy[0], self.dy[1], self.cu_dev[0],
                          self.cu_host[0], self.cu_dev[1], self.cu_host[1], self.S, self.cond, self.saved,
                          self.dx[0], self.dx[1], self.g, self.dcond, self.scratch, self.scratch_bytes)

    def step(self):
        self.forward()
        self.backward()

    def results(self):
        """([y_text, y_img], [dx_text, dx_img], [grads_text, grads_img], dcond) as float64 numpy arrays."""
        torch.cuda.synchronize()
        f = lambda t: t.detach().float().cpu().numpy().astype(np.float64)
        return ([f(t) for t in self.y], [f(t) for t in self.dx],
                [{k: f(v) for k, v in gs.items()} for gs in self.grads], f(self.dcond))
