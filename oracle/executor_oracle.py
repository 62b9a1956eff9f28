"""CPU oracle for one pipeline stage's share (fp64, numpy): the modules of every
unit run one after the other, nothing overlapped.

TEST INFRASTRUCTURE ONLY (tests/, smoke, the cpu_baseline leg of bench.py).

What is computed follows the paper's module functions (Sec. 3.2, executor interface
figure): encoder_forward -> embed_preprocess + llm -> generator_forward, and the
reverse for gradients, with gradients of all units accumulated (Sec. 3.2 "Module
handoff": accumulation semantics are preserved).  The glue the paper leaves open
("projectors") is a stand-in: feat = enc_out proj_in^T placed at the image-token
rows of the LLM input; cond = llm_out[last row of each image] proj_out^T; per-unit
loss 0.5*mean((gen_out - target)^2); without a generator the per-microbatch loss is
<llm_out, out_grad>.  Pins: tests/test_oracle_executor.py (finite differences of the
total loss, reduction to single blocks).
"""
from __future__ import annotations

import numpy as np

from . import block_oracle as bo

F64 = np.float64


def _gen_cu(n_images, tpi):
    return np.arange(n_images + 1, dtype=np.int64) * tpi


def run_stage(stage):
    """Returns (losses, grads): losses per unit (generator) or per microbatch;
    grads = {"enc": [dict per block], "llm": [...], "gen": [...], "proj_in", "proj_out"}."""
    acc = lambda plist: [{k: np.zeros(v.shape, dtype=F64) for k, v in p.items()} for p in plist]
    g_enc, g_llm, g_gen = acc(stage.enc_params), acc(stage.llm_params), acc(stage.gen_params)
    proj_in = np.asarray(stage.proj_in, dtype=F64)
    g_proj_in = np.zeros_like(proj_in)
    has_gen = stage.has_generator
    if has_gen:
        proj_out = np.asarray(stage.proj_out, dtype=F64)
        g_proj_out = np.zeros_like(proj_out)
    losses = []
    us = stage.unit_size
    for u, unit in enumerate(stage.units):
        mbs = stage.microbatches[u * us:(u + 1) * us]
        # encoder forward
        x = np.asarray(unit.patches, dtype=F64)
        enc_caches = []
        for p in stage.enc_params:
            x, c = bo.block_forward(stage.enc_cfg, p, x, unit.cu_seqlens)
            enc_caches.append(c)
        enc_out = x
        feat = enc_out @ proj_in.T
        # LLM forward per microbatch
        llm_caches, llm_out, off = [], [], 0
        for mb in mbs:
            h = np.asarray(mb.base, dtype=F64).copy()
            n = len(mb.image_rows)
            h[mb.image_rows] = feat[off:off + n]
            off += n
            caches = []
            for p in stage.llm_params:
                h, c = bo.block_forward(stage.llm_cfg, p, h, mb.cu_seqlens)
                caches.append(c)
            llm_caches.append(caches); llm_out.append(h)
        # generator forward + backward, or the stand-in LLM loss
        d_out = []
        if has_gen:
            hsel = np.concatenate([o[mb.image_last_row] for o, mb in zip(llm_out, mbs)], axis=0)
            cond = hsel @ proj_out.T
            n_img = hsel.shape[0]
            cu_g = _gen_cu(n_img, stage.tokens_per_image)
            z = np.asarray(unit.latents, dtype=F64)
            gcaches = []
            for p in stage.gen_params:
                z, c = bo.block_forward(stage.gen_cfg, p, z, cu_g, cond)
                gcaches.append(c)
            diff = z - np.asarray(unit.targets, dtype=F64)
            losses.append(0.5 * float((diff * diff).mean()))
            dz = diff / diff.size
            dcond = np.zeros_like(cond)
            for b in reversed(range(len(stage.gen_params))):
                dz, g, dc = bo.block_backward(stage.gen_cfg, stage.gen_params[b], gcaches[b], dz)
                for k in g:
                    g_gen[b][k] += g[k]
                dcond += dc
            g_proj_out += dcond.T @ hsel
            dhsel = dcond @ proj_out
            i0 = 0
            for o, mb in zip(llm_out, mbs):
                d = np.zeros_like(o)
                d[mb.image_last_row] = dhsel[i0:i0 + len(mb.image_last_row)]
                i0 += len(mb.image_last_row)
                d_out.append(d)
        else:
            for o, mb in zip(llm_out, mbs):
                og = np.asarray(mb.out_grad, dtype=F64)
                losses.append(float((o * og).sum()))
                d_out.append(og)
        # LLM backward, gather the encoder-row gradients
        dfeat = np.zeros_like(feat)
        off = 0
        for mb, caches, d in zip(mbs, llm_caches, d_out):
            for b in reversed(range(len(stage.llm_params))):
                d, g, _ = bo.block_backward(stage.llm_cfg, stage.llm_params[b], caches[b], d)
                for k in g:
                    g_llm[b][k] += g[k]
            n = len(mb.image_rows)
            dfeat[off:off + n] = d[mb.image_rows]
            off += n
        # encoder backward
        g_proj_in += dfeat.T @ enc_out
        d = dfeat @ proj_in
        for b in reversed(range(len(stage.enc_params))):
            d, g, _ = bo.block_backward(stage.enc_cfg, stage.enc_params[b], enc_caches[b], d)
            for k in g:
                g_enc[b][k] += g[k]
    grads = {"enc": g_enc, "llm": g_llm, "gen": g_gen, "proj_in": g_proj_in}
    if has_gen:
        grads["proj_out"] = g_proj_out
    return losses, grads


def total_loss(stage):
    return float(np.sum(run_stage(stage)[0]))
