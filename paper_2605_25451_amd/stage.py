"""Device-memory plumbing for the micro-unit executor: puts a synth.StageCase into
HBM, fills the C structs and forwards calls.  No arithmetic happens here."""
from __future__ import annotations

import ctypes as C

import numpy as np
import torch

from . import binding as bm
from . import synth
from .runner import to_device


class StageOnDevice:
    def __init__(self, stage: synth.StageCase, device="cuda:0", repeat: int = 1):
        """repeat > 1: the executor sees repeat * M microbatches (and their units), entry k being
        the stage's microbatch k mod M -- the same read-only device buffers again (a benchmark's way
        to a larger batch without drawing and uploading more inputs)."""
        self.stage = stage
        self.repeat = repeat
        dt = stage.llm_cfg.dtype
        dev = lambda a: to_device(a, dt, device)
        i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)
        self.keep = []                       # everything the executor points to stays alive here

        def blocks(plist):
            ws, gs, ps, pg = [], [], [], []
            for p in plist:
                w = {k: dev(v) for k, v in p.items()}
                g = {k: torch.zeros(v.shape, dtype=torch.float32, device=device) for k, v in w.items()}
                ws.append(w); gs.append(g)
                ps.append(bm.make_params(w)); pg.append(bm.make_params(g))
            n = max(len(plist), 1)
            arr_w = (bm.BlockParams * n)(*ps) if ps else (bm.BlockParams * 1)()
            arr_g = (bm.BlockParams * n)(*pg) if pg else (bm.BlockParams * 1)()
            return ws, gs, arr_w, arr_g

        self.enc_w, self.enc_g, enc_aw, enc_ag = blocks(stage.enc_params)
        self.llm_w, self.llm_g, llm_aw, llm_ag = blocks(stage.llm_params)
        self.gen_w, self.gen_g, gen_aw, gen_ag = blocks(stage.gen_params)
        self.proj_in = dev(stage.proj_in)
        self.g_proj_in = torch.zeros(stage.proj_in.shape, dtype=torch.float32, device=device)
        gen = stage.has_generator
        self.proj_out = dev(stage.proj_out) if gen else None
        self.g_proj_out = torch.zeros(stage.proj_out.shape, dtype=torch.float32, device=device) if gen else None
        self.w = bm.ExecutorParams(enc_aw, llm_aw, gen_aw, self.proj_in.data_ptr(),
                                   self.proj_out.data_ptr() if gen else None)
        self.g = bm.ExecutorParams(enc_ag, llm_ag, gen_ag, self.g_proj_in.data_ptr(),
                                   self.g_proj_out.data_ptr() if gen else None)
        self.keep += [enc_aw, enc_ag, llm_aw, llm_ag, gen_aw, gen_ag]

        assert repeat == 1 or stage.M % stage.unit_size == 0
        mbs = (bm.Microbatch * (stage.M * repeat))()
        for m, mb in enumerate(stage.microbatches):
            cu_h = np.ascontiguousarray(mb.cu_seqlens, dtype=np.int32)
            t = dict(cu_d=i32(cu_h), base=dev(mb.base), rows=i32(mb.image_rows),
                     last=i32(mb.image_last_row), og=dev(mb.out_grad))
            self.keep += [cu_h, t]
            mbs[m] = bm.Microbatch(mb.T, len(cu_h) - 1, t["cu_d"].data_ptr(), cu_h.ctypes.data,
                                   t["base"].data_ptr(), len(mb.image_rows), t["rows"].data_ptr(),
                                   len(mb.image_last_row), t["last"].data_ptr(), t["og"].data_ptr())
        for m in range(stage.M, stage.M * repeat):
            mbs[m] = mbs[m % stage.M]
        units = (bm.Unit * (len(stage.units) * repeat))()
        for u, un in enumerate(stage.units):
            cu_h = np.ascontiguousarray(un.cu_seqlens, dtype=np.int32)
            S = len(cu_h) - 1
            gcu_h = (np.arange(S + 1, dtype=np.int32) * stage.tokens_per_image)
            t = dict(cu_d=i32(cu_h), patches=dev(un.patches), gcu_d=i32(gcu_h))
            if gen:
                t["lat"] = dev(un.latents); t["tgt"] = dev(un.targets)
            self.keep += [cu_h, gcu_h, t]
            units[u] = bm.Unit(int(cu_h[-1]), S, t["cu_d"].data_ptr(), cu_h.ctypes.data,
                               t["patches"].data_ptr(), t["gcu_d"].data_ptr(), gcu_h.ctypes.data,
                               t["lat"].data_ptr() if gen else None, t["tgt"].data_ptr() if gen else None)
        for u in range(len(stage.units), len(stage.units) * repeat):
            units[u] = units[u % len(stage.units)]
        self.mbs, self.units = mbs, units
        self.cfg = bm.ExecutorConfig(bm.make_desc(stage.enc_cfg), bm.make_desc(stage.llm_cfg),
                                     bm.make_desc(stage.gen_cfg if gen else stage.enc_cfg),
                                     len(stage.enc_params), len(stage.llm_params),
                                     len(stage.gen_params) if gen else 0, stage.M * repeat, stage.unit_size,
                                     stage.tokens_per_image)
        self.loss = torch.zeros(stage.M * repeat, dtype=torch.float32, device=device)
        self.ex = None
        self.arena = None
        self.device = device

    def create(self, enc_slots: int, llm_slots: int, M: int = None):
        """M: run only the first M microbatches of the stage (and the units they fill)."""
        self.destroy()
        if M is not None:
            total = self.stage.M * self.repeat
            assert 1 <= M <= total and (M % self.stage.unit_size == 0 or M == total)
            self.cfg.M = M
        nbytes = bm.executor_arena_bytes(self.cfg, self.mbs, self.units, enc_slots, llm_slots)
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        off = (-self.arena.data_ptr()) % 256
        self.arena_bytes = nbytes
        self.ex = bm.executor_create(self.cfg, self.w, self.g, self.mbs, self.units,
                                     self.arena.data_ptr() + off, nbytes, enc_slots, llm_slots)
        return nbytes

    def zero_grads(self):
        for gl in (self.enc_g, self.llm_g, self.gen_g):
            for g in gl:
                for t in g.values():
                    t.zero_()
        self.g_proj_in.zero_()
        if self.g_proj_out is not None:
            self.g_proj_out.zero_()

    def run(self, ops):
        bm.executor_load_schedule(self.ex, ops)
        self.loss.zero_()
        bm.executor_execute(self.ex, self.loss)

    def run_timed(self, ops):
        """Runs the op stream with per-op timing: (ms per op, live activation bytes after each op)."""
        bm.executor_load_schedule(self.ex, ops)
        self.loss.zero_()
        return bm.executor_execute_timed(self.ex, self.loss, len(ops))

    def results(self):
        torch.cuda.synchronize()
        f = lambda t: t.detach().float().cpu().numpy().astype(np.float64)
        n = len(self.stage.units) if self.stage.has_generator else self.stage.M
        grads = {"enc": [{k: f(v) for k, v in g.items()} for g in self.enc_g],
                 "llm": [{k: f(v) for k, v in g.items()} for g in self.llm_g],
                 "gen": [{k: f(v) for k, v in g.items()} for g in self.gen_g],
                 "proj_in": f(self.g_proj_in)}
        if self.g_proj_out is not None:
            grads["proj_out"] = f(self.g_proj_out)
        return f(self.loss)[:n], grads

    def peak_bytes(self):
        return bm.executor_peak_activation_bytes(self.ex), bm.executor_peak_encoder_bytes(self.ex)

    def destroy(self):
        if self.ex is not None:
            bm.executor_destroy(self.ex)
            self.ex = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
