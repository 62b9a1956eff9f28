#!/usr/bin/env python3
"""Benchmark of the hot path: forward + backward of one packed variable-length
transformer block on one MI355X, through the C-ABI library.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config2|config3|config4|dit|moe|mmdit]
  python bench.py --workload config5 --batch 8|16|32 [--unit-size 1] [--steps K]
  python bench.py --workload pipeline [--steps K]
  python bench.py --workload cp [--steps K]

One step = bm_block_forward + bm_block_backward over one batch of seeded
synthetic packed tokens that is already resident in HBM.  Prints ONE JSON line:
block fwd+bwd TFLOP/s (algorithmic flops: 3 x GEMM-forward + 3.5 x
attention-forward over unmasked within-sequence pairs), the roofline figures
of the dominant kernel class measured with HIP events on the launch stream,
and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PAPER_CONTEXT = ("the paper reports 1.08x-1.9x end-to-end training speedups of its nested schedule over "
                 "prior systems on 128 H800 GPUs (Sec. 4.2) and no per-block time, TFLOP/s or bandwidth: "
                 "context only, not comparable with a single-GPU block measurement")
MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of a kernel class come from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# summarised under profiles/: each summary ends with a JSON block "traffic_bytes_per_launch"
# (fetched + written, counters scaled by what they read for a plain 1 GiB copy; the split-k
# reduction that follows a weight-gradient GEMM is part of that class's launch).  They are an
# offline measurement of the same command, not counters read in this run; workloads or classes
# without a summarised counter run report null.
PROFILE_OF = {
    "config2_vit_large_bf16": "block_fwd_bwd_config2.md",
    "config3_decoder_7b_bf16": "block_fwd_bwd_config3.md",
    "config4_decoder_8b_gqa_bf16": "block_fwd_bwd_config4.md",
}


def measured_traffic(case_name):
    """(bytes per launch by class, source) from the committed profile summary, or ({}, None)."""
    name = PROFILE_OF.get(case_name)
    if name is None:
        return {}, None
    path = os.path.join(ROOT, "profiles", name)
    try:
        text = open(path).read()
        block = text.split("```json traffic_bytes_per_launch", 1)[1].split("```", 1)[0]
        return json.loads(block), f"offline rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, profiles/{name}"
    except (OSError, IndexError, ValueError):
        return {}, None


def moe_case(seed=5, total=8192):
    """Decoder block with the mixture-of-experts FFN (128 experts of width 768, 8 per token,
    hidden 2048) over config-3-style documents."""
    import numpy as np
    from paper_2605_25451_amd import synth
    rng = np.random.default_rng(seed)
    docs = synth.documents_interleaved(rng, total)
    return synth.make_case(synth.decoder_moe(), [d.length for d in docs], seed, rng=rng, docs=docs,
                           name="moe_decoder_bf16")


def algorithmic_flops(cfg, cu):
    """(gemm_fwd, attn_fwd) flops of one block over the packed batch."""
    import numpy as np
    T = int(cu[-1])
    d, F = cfg.hidden, cfg.mlp_hidden
    qd = cfg.n_q_heads * cfg.head_dim
    gemm = 2.0 * T * d * cfg.qkv_dim + 2.0 * T * qd * d
    if getattr(cfg, "n_experts", 0) > 0:      # router + k active experts per token
        gemm += 2.0 * T * d * cfg.n_experts + cfg.top_k * (2.0 * T * d * cfg.up_dim + 2.0 * T * F * d)
    else:
        gemm += 2.0 * T * d * cfg.up_dim + 2.0 * T * F * d
    if cfg.norm == 2:
        gemm += 2.0 * (len(cu) - 1) * d * 6 * d
    L = np.diff(cu).astype(np.float64)
    pairs = (L * (L + 1) / 2).sum() if cfg.mask else (L * L).sum()
    attn = 4.0 * cfg.head_dim * cfg.n_q_heads * pairs
    return gemm, attn


def mmdit_case(seed=6, n_samples=16, image_tokens=1024):
    """Two-stream block at the shape of a 20 B-class multimodal diffusion transformer (hidden 3072,
    24 heads of 128, MLP 12288; the paper states the size only): per sample one caption of
    U[32, 256] text tokens and 1024 latent image tokens."""
    import numpy as np
    from paper_2605_25451_amd import synth
    rng = np.random.default_rng(seed)
    text = [int(v) for v in rng.integers(32, 257, size=n_samples)]
    cfg = synth.scaled(synth.dit_block(), hidden=3072, n_q_heads=24, n_kv_heads=24, head_dim=128, mlp_hidden=12288)
    return synth.make_two_stream_case(cfg, text, [image_tokens] * n_samples, seed, 1, "mmdit_20b_block_bf16")


def mmdit_flops(cfg, cu_text, cu_img):
    """(gemm_fwd, attn_fwd) flops of the two-stream block: per-stream projections, joint attention."""
    import numpy as np
    d, F, S = cfg.hidden, cfg.mlp_hidden, len(cu_text) - 1
    T = int(cu_text[-1]) + int(cu_img[-1])
    gemm = 2.0 * T * d * (3 * d + d + 2 * F) + 2 * 2.0 * S * d * 6 * d
    L = (np.diff(cu_text) + np.diff(cu_img)).astype(np.float64)
    attn = 4.0 * cfg.head_dim * cfg.n_q_heads * (L * L).sum()
    return gemm, attn


def mmdit_sub_case(case, n):
    """The first n samples of a two-stream case (same parameters)."""
    from paper_2605_25451_amd import synth
    cu = [c[:n + 1] for c in case.cu]
    return synth.TwoStreamCase(case.cfg, cu, [case.x[s][:cu[s][-1]] for s in range(2)], case.params,
                               [case.dy[s][:cu[s][-1]] for s in range(2)], case.cond[:n], case.qk_norm,
                               case.name + "_sub")


def cpu_baseline_mmdit(case, budget_flops=2.0e12):
    from oracle import mmdit_oracle as mo
    n = 1
    while n < case.S:
        g, a = mmdit_flops(case.cfg, case.cu[0][:n + 1], case.cu[1][:n + 1])
        if 3.0 * g + 3.5 * a >= budget_flops:
            break
        n += 1
    sub = mmdit_sub_case(case, n)
    t0 = time.perf_counter()
    _, cache = mo.mmdit_forward(sub.cfg, sub.params, sub.x, sub.cu, sub.cond, bool(sub.qk_norm))
    mo.mmdit_backward(sub.cfg, cache, sub.dy, bool(sub.qk_norm))
    dt = time.perf_counter() - t0
    g, a = mmdit_flops(sub.cfg, sub.cu[0], sub.cu[1])
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    T_sub, T = int(sub.cu[0][-1] + sub.cu[1][-1]), int(case.cu[0][-1] + case.cu[1][-1])
    return {"value": (3.0 * g + 3.5 * a) / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"numpy fp64 oracle fwd+bwd on the first {n} samples ({T_sub} of {T} tokens) "
                      f"of the same batch, {dt:.1f} s"}


def copy_calibration():
    """Three plain 1 GiB device copies: the yardstick for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE."""
    import torch
    src = torch.empty(1 << 29, dtype=torch.bfloat16, device="cuda").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()


def run_cp_workload(args):
    """One rank of a context-parallel group of 4 on a 32768-token causal document (the 8 B GQA
    attention shape): the last rank, whose 8192 queries see all four key/value chunks."""
    import numpy as np
    import torch
    from paper_2605_25451_amd import binding as bm, synth
    from paper_2605_25451_amd.cp import ContextParallelGroup
    Hq, Hkv, dh, C, L = 32, 8, 128, 4, 32768
    dt = synth.DTYPE_BF16
    rng = np.random.default_rng(7)
    cu = synth.cu_from_lengths([L])
    mk = lambda w: synth.to_storage(rng.standard_normal((L, w), dtype=np.float32), dt)
    q, k, v, d_o = mk(Hq * dh), mk(Hkv * dh), mk(Hkv * dh), mk(Hq * dh)
    rank = C - 1
    g = ContextParallelGroup(dt, Hq, Hkv, dh, True, cu, C, q, k, v, d_o, ranks=[rank])
    n = L // C
    pairs = (C - 1) * float(n) * n + n * (n + 1) / 2.0
    fwd_flops = 4.0 * dh * Hq * pairs
    step_flops = 3.5 * fwd_flops
    def step():
        g.forward(); g.backward()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    bm.profile_begin()
    for _ in range(args.steps):
        step()
    prof = bm.profile_end()
    torch.cuda.synchronize()
    breakdown = {c: {"ms_per_step": m / args.steps, "launches_per_step": cnt / args.steps,
                     "avg_launch_us": m / cnt * 1e3,
                     **({"tflops": w / (m * 1e-3) / 1e12} if c.startswith("attn") else {"gbs": w / (m * 1e-3) / 1e9})}
                 for c, (m, w, cnt) in prof.items() if cnt}
    dom = max(breakdown, key=lambda c: breakdown[c]["ms_per_step"])
    d_ms, d_work, d_n = prof[dom]
    ach = d_work / (d_ms * 1e-3) / 1e12
    tflops = step_flops / (ms * 1e-3) / 1e12
    out = {"metric": "context-parallel attention fwd+bwd TFLOP/s of one rank (bf16)", "value": tflops,
           "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "cp4_last_rank_causal_32k", "document_tokens": L, "cp_degree": C, "rank": rank,
                      "queries": n, "heads": f"{Hq}q/{Hkv}kv x {dh}",
                      "step": "4 chunk-pair forwards + merge, 4 chunk-pair backwards + sum of the dq parts",
                      "flops_per_step": step_flops},
           "mfma_util_pct": 100.0 * tflops / MFMA_BF16_PEAK_TFLOPS,
           "roofline": {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
                        "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS, "avg_launch_us": d_ms / d_n * 1e3,
                        "traffic": None},
           "breakdown": breakdown, "paper_context": PAPER_CONTEXT}
    if args.copy_calibration:
        copy_calibration()
    if not args.no_cpu_baseline:
        from oracle import cp_attention_oracle as co
        Ls = 12288                                   # same shape, a 12288-token document
        cus = synth.cu_from_lengths([Ls])
        ch = synth.context_chunks(cus, C)
        r3 = lambda a, w: a[:Ls].astype(np.float64).reshape(Ls, -1, dh)
        q3, k3, v3, do3 = r3(q, Hq), r3(k, Hkv), r3(v, Hkv), r3(d_o, Hq)
        t0 = time.perf_counter()
        rq, cq = ch[rank]
        parts = [co.chunk_forward(q3[rq], k3[ch[j][0]], v3[ch[j][0]], cq, ch[j][1], j == rank) for j in range(C)]
        o, lse = co.merge([p[0] for p in parts], [p[1] for p in parts])
        for j in range(C):
            co.chunk_backward(q3[rq], k3[ch[j][0]], v3[ch[j][0]], o, do3[rq], lse, cq, ch[j][1], j == rank)
        dt_s = time.perf_counter() - t0
        ns = Ls // C
        fl = 3.5 * 4.0 * dh * Hq * ((C - 1) * float(ns) * ns + ns * (ns + 1) / 2.0)
        out["cpu_baseline"] = {"value": fl / dt_s / 1e12, "unit": "TFLOP/s", "cores": os.cpu_count(), "kind": "oracle",
                               "sample": f"numpy fp64 oracle, the same rank of a {Ls}-token document, {dt_s:.1f} s"}
    print(json.dumps(out))


def measured_peaks():
    """What this chip sustains: register-resident MFMA loop and a streaming copy."""
    import torch
    from paper_2605_25451_amd import binding as bm
    out = torch.zeros(16, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    blocks, iters = 256 * 4, 4000
    bm.probe_mfma(blocks, 200, out)
    e0.record(); bm.probe_mfma(blocks, iters, out); e1.record(); torch.cuda.synchronize()
    mfma = blocks * 4 * iters * 16 * 32768.0 / (e0.elapsed_time(e1) * 1e-3) / 1e12
    # the same loop by instruction shape and operand data: the clock under matrix load depends on the data
    by_data = {}
    for shape16, sname in ((0, "32x32x16"), (1, "16x16x32")):
        for rnd, dname in ((0, "zeros"), (1, "random")):
            it = iters * 4 if shape16 == 0 else iters * 2
            bm.probe_mfma_ex(blocks, 200, shape16, rnd, out)
            e0.record(); bm.probe_mfma_ex(blocks, it, shape16, rnd, out); e1.record(); torch.cuda.synchronize()
            by_data[f"{sname}_{dname}"] = blocks * 4 * it * (2.0 ** 19 if shape16 == 0 else 2.0 ** 20) / (e0.elapsed_time(e1) * 1e-3) / 1e12
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda"); dst = torch.empty_like(src)
    src.zero_()
    bm.probe_copy(src, dst, n)
    e0.record()
    for _ in range(5):
        bm.probe_copy(src, dst, n)
    e1.record(); torch.cuda.synchronize()
    hbm = 5 * 2.0 * n / (e0.elapsed_time(e1) * 1e-3) / 1e9
    # the two legs on their own, over a handful of launch shapes (workgroups per CU x loads in flight)
    word = torch.zeros(256, dtype=torch.int32, device="cuda")
    def timed(fn):
        fn()
        e0.record()
        for _ in range(5):
            fn()
        e1.record(); torch.cuda.synchronize()
        return 5.0 * n / (e0.elapsed_time(e1) * 1e-3) / 1e9
    reads = {f"{wpc}wg_per_cu_x{u}": timed(lambda: bm.probe_read(src, n, 256 * wpc, u, word))
             for wpc, u in ((8, 1), (8, 4), (8, 8), (16, 4), (4, 8))}
    fills = {f"{wpc}wg_per_cu": timed(lambda: bm.probe_fill(dst, n, 256 * wpc)) for wpc in (4, 8, 16)}
    # LDS by instruction kind (bytes per ns and CU; two workgroups of four wavefronts per CU), and what a
    # GEMM slice's mix -- two bytes of fragment reads per byte filled -- takes with either kind of fill
    lds_iters, per_wave = 4000, {1: 16384, 2: 16384, 4: 8192, 8: 8192, 5: 24576, 9: 24576}
    names = {1: "read_b128", 2: "read_tr_b64", 4: "store_b128", 8: "direct_load_b128", 5: "reads_and_stores", 9: "reads_and_direct_loads"}
    lds = {}
    for what in (1, 2, 4, 8, 5, 9):
        bm.probe_lds(what, 100, src, n, word)
        e0.record(); bm.probe_lds(what, lds_iters, src, n, word); e1.record(); torch.cuda.synchronize()
        lds[names[what]] = 2 * 4 * lds_iters * per_wave[what] / (e0.elapsed_time(e1) * 1e6)
    # ns per group of one 32x32x16 MFMA and 0 / 4 / 8 independent vector instructions, one wavefront per SIMD
    issue = {}
    for nv in (0, 4, 8):
        bm.probe_issue(nv, 100, out)
        e0.record(); bm.probe_issue(nv, 20000, out); e1.record(); torch.cuda.synchronize()
        issue[f"mfma_plus_{nv}_valu"] = e0.elapsed_time(e1) * 1e6 / (20000 * 4)
    return {"mfma_bf16_tflops": mfma, "mfma_bf16_tflops_by_shape_and_operands": by_data, "hbm_copy_gbs": hbm, "hbm_read_gbs": max(reads.values()),
            "hbm_write_gbs": max(fills.values()), "hbm_read_sweep_gbs": reads, "hbm_write_sweep_gbs": fills,
            "lds_bytes_per_ns_per_cu": lds, "issue_ns_per_group": issue}


def make_workload(name):
    from paper_2605_25451_amd import synth
    if name == "config2":
        return synth.config2()
    if name == "config3":
        return synth.config3()
    if name == "config4":
        return synth.config4()
    if name == "dit":
        return synth.dit_case()
    if name == "moe":
        return moe_case()
    raise SystemExit(f"unknown workload {name}")


def cpu_baseline(case, budget_flops=2.0e12):
    """The oracle as it stands, timed on a bounded sample: the first sequences of
    the same pack up to about budget_flops algorithmic flops (10-30 s of fp64 BLAS)."""
    import numpy as np
    from oracle import block_oracle as bo
    from paper_2605_25451_amd import synth
    ids = []
    for s in range(case.S):
        ids.append(s)
        g, a = algorithmic_flops(case.cfg, synth.sub_case(case, ids).cu_seqlens)
        if 3.0 * g + 3.5 * a >= budget_flops:
            break
    sub = synth.sub_case(case, ids)
    t0 = time.perf_counter()
    bo.block_fwd_bwd(sub.cfg, sub.params, sub.x, sub.cu_seqlens, sub.dy, sub.cond)
    dt = time.perf_counter() - t0
    g, a = algorithmic_flops(sub.cfg, sub.cu_seqlens)
    flops = 3.0 * g + 3.5 * a
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"numpy fp64 oracle fwd+bwd on the first {len(ids)} sequences "
                      f"({sub.T} of {case.T} tokens) of the same pack, {dt:.1f} s"}


def stage_sweep(batches, unit_size, steps):
    """config 5: one pipeline stage's share -- 4 decoder blocks over M microbatches of 8192 packed
    tokens, with 6 ViT-L blocks per encoder unit and 2 DiT blocks per generator unit nested between
    them -- for every M in `batches` (8 seeded microbatches are drawn; larger batches run them
    again cyclically).  Per M and order (nested / compute-efficient): LLM tokens/s, the executor's
    activation high-water marks (all activations, and the encoder units' part) and the arena the
    slots occupy in HBM."""
    import torch
    from paper_2605_25451_amd import binding as bm
    from paper_2605_25451_amd import synth
    from paper_2605_25451_amd.stage import StageOnDevice
    Mdraw = min(max(batches), max(8, unit_size))
    stage = synth.make_stage(synth.vit_large(), synth.decoder_7b(), synth.dit_block(), 6, 4, 2, Mdraw,
                             unit_size, 8192, seed=4)
    # batches above the drawn one reuse its microbatches cyclically (same read-only inputs in HBM):
    # step time and activation memory do not depend on the values
    dev = StageOnDevice(stage, repeat=-(-max(batches) // Mdraw))
    units_all = [stage.units[u % len(stage.units)] for u in range(-(-max(batches) // unit_size))]
    depth = 3
    out = {"blocks": "6 ViT-L / 4 decoder-7B / 2 DiT", "llm_tokens_per_microbatch": 8192,
           "unit_size": unit_size, "encoder_slots_nested": 3, "llm_units_in_flight": depth,
           "steps": steps, "batches": {}}
    for M in batches:
        U = -(-M // unit_size)
        entry = {"encoder_tokens_per_unit": [int(u.cu_seqlens[-1]) for u in units_all[:U]]}
        for name, order, slots in (("nested", bm.ORDER_NESTED, min(3, U)),
                                   ("compute_efficient", bm.ORDER_COMPUTE_EFFICIENT, U)):
            arena = dev.create(slots, depth * unit_size, M=M)
            ops = bm.build_schedule(order, M, unit_size, 3, depth, 1)
            dev.zero_grads()
            dev.run(ops)                                     # warm-up step
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                dev.run(ops)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / steps
            peak, peak_enc = dev.peak_bytes()
            entry[name] = {"ms_per_step": dt * 1e3, "tokens_per_s": M * 8192 / dt,
                           "peak_activation_bytes": peak, "peak_encoder_bytes": peak_enc,
                           "arena_bytes": arena}
            dev.destroy()
        out["batches"][str(M)] = entry
    return out


def run_stage_workload(args):
    """config 5 at one batch size: python bench.py --workload config5 --batch M [--unit-size U]."""
    sweep = stage_sweep((args.batch,), args.unit_size, args.steps)
    entry = sweep["batches"][str(args.batch)]
    out = {"metric": "stage tokens/s and peak activation bytes (config 5)", "unit": "tokens/s",
           "n_gpus": 1, "dtype": "bf16", "data": "synthetic", "higher_is_better": True,
           "config": {"workload": "config5_stage", "microbatches": args.batch, "unit_size": args.unit_size,
                      "llm_tokens_per_microbatch": 8192, "blocks": sweep["blocks"],
                      "encoder_tokens": entry["encoder_tokens_per_unit"]},
           "orders": {k: entry[k] for k in ("nested", "compute_efficient")}}
    out["value"] = out["orders"]["nested"]["tokens_per_s"]
    out["ms_per_step"] = out["orders"]["nested"]["ms_per_step"]
    out["steps"] = args.steps
    print(json.dumps(out))


def run_pipeline_workload(args):
    """Replay of the paper's scheme-figure configuration (pp 4, vpp 2, batch 64, W = 3) with
    operator times measured here: 16 microbatches of the config-5 stage (6 ViT-L / 4 decoder-7B
    / 2 DiT blocks, 8192 LLM tokens each) are run one unit at a time with per-op event timing;
    their encoder / generator times (they vary with the image-token count) are reused
    cyclically for the 64 microbatches; an LLM chunk is half of the rank's 4 blocks."""
    import torch
    from paper_2605_25451_amd import binding as bm
    from paper_2605_25451_amd import synth
    from paper_2605_25451_amd.stage import StageOnDevice
    P, V, M, W = 4, 2, 64, 3
    Mm = 16
    stage = synth.make_stage(synth.vit_large(), synth.decoder_7b(), synth.dit_block(), 6, 4, 2, Mm, 1,
                             8192, seed=4)
    dev = StageOnDevice(stage)
    dev.create(1, 1)
    ops = bm.build_schedule(bm.ORDER_SEQUENTIAL, Mm, 1, 3, 3, 1)
    dev.zero_grads()
    dev.run(ops)
    torch.cuda.synchronize()
    acc = {}
    for _ in range(args.steps):
        ms, live = dev.run_timed(ops)
        prev = 0.0
        for (code, idx), t, lv in zip(ops, ms, live):
            a = acc.setdefault((code, idx), [0.0, 0.0])
            a[0] += t / args.steps
            a[1] = lv - prev
            prev = lv
    dev.destroy()
    sec = lambda code: [acc[(code, i)][0] * 1e-3 for i in range(Mm)]
    grow = lambda code: [acc[(code, i)][1] for i in range(Mm)]
    tile = lambda v: [v[i % Mm] for i in range(M)]
    llm_f = sum(sec(bm.OP_LLM_FWD)) / Mm / V
    llm_b = sum(sec(bm.OP_LLM_BWD)) / Mm / V
    act_llm = sum(grow(bm.OP_LLM_FWD)) / Mm / V
    times = dict(llm_fwd=[llm_f] * (P * V), llm_bwd=[llm_b] * (P * V),
                 enc_fwd=tile(sec(bm.OP_ENC_FWD)), enc_bwd=tile(sec(bm.OP_ENC_BWD)),
                 gen_fwd=tile(sec(bm.OP_GEN_FWD)), gen_bwd=tile(sec(bm.OP_GEN_BWD)))
    acts = dict(act_llm=act_llm, act_enc=tile(grow(bm.OP_ENC_FWD)), act_gen=tile(grow(bm.OP_GEN_FWD)))
    xgmi = 8192 * 4096 * 2 / 153e9            # one [T, d] bf16 activation over one xGMI link (estimate)
    orders = {}
    for name, order in (("nested", bm.ORDER_NESTED), ("compute_efficient", bm.ORDER_COMPUTE_EFFICIENT),
                        ("memory_efficient", bm.ORDER_MEMORY_EFFICIENT)):
        entry = {}
        for tag, lat in (("p2p_0", 0.0), ("p2p_xgmi_estimate", xgmi)):
            r = bm.pipeline_replay(order, P, V, M, W, 1, p2p=lat, **times, **acts)
            entry[tag] = {"makespan_ms": r["makespan"] * 1e3, "bubble": r["bubble"],
                          "tokens_per_s": M * 8192 / r["makespan"],
                          "peak_activation_gib": max(r["peak"]) / 2**30,
                          "peak_encoder_gib": max(r["peak_enc"]) / 2**30,
                          "peak_generator_gib": max(r["peak_gen"]) / 2**30}
        orders[name] = entry
    out = {"metric": "pipeline replay tokens/s (pp 4, vpp 2, batch 64, W 3) from operator times measured on this GPU",
           "value": orders["nested"]["p2p_0"]["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1,
           "steps": args.steps, "warmup": 1, "ms_per_step": orders["nested"]["p2p_0"]["makespan_ms"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": "pipeline_replay_pp4_vpp2_batch64", "measured_microbatches": Mm,
                      "llm_chunk_fwd_ms": llm_f * 1e3, "llm_chunk_bwd_ms": llm_b * 1e3,
                      "encoder_fwd_ms_range": [min(times["enc_fwd"]) * 1e3, max(times["enc_fwd"]) * 1e3],
                      "generator_fwd_ms_range": [min(times["gen_fwd"]) * 1e3, max(times["gen_fwd"]) * 1e3],
                      "p2p_xgmi_estimate_ms": xgmi * 1e3,
                      "note": "value is the replay's throughput of a 4-GPU pipeline group, not a measurement on 4 GPUs"},
           "orders": orders}
    if not args.no_cpu_baseline:
        from oracle import pipeline_oracle as po
        t0 = time.perf_counter()
        ref = po.replay(po.NESTED, P, V, M, W, True, times["llm_fwd"], times["llm_bwd"], times["enc_fwd"],
                        times["enc_bwd"], times["gen_fwd"], times["gen_bwd"], **acts)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 1.0 / dt, "unit": "replays/s", "cores": 1, "kind": "oracle",
                               "sample": "one nested replay of the same configuration",
                               "makespan_matches": ref["makespan"] == orders["nested"]["p2p_0"]["makespan_ms"] * 1e-3}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="headline",
                    help="headline (default: config4 as the headline, config2/config3 and the config-5 stage "
                         "sweep as extra keys) | config2 | config3 | config4 | dit | moe | mmdit | config5 | "
                         "pipeline | cp")
    ap.add_argument("--no-stage-sweep", action="store_true", help="headline run without the config-5 sweep")
    ap.add_argument("--batch", type=int, default=8, help="microbatches (config5 only)")
    ap.add_argument("--unit-size", type=int, default=1, help="microbatches per unit (config5 only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (a counter yardstick for "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_25451_amd import binding as bm
    from paper_2605_25451_amd.runner import CaseOnDevice

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    bm.lib()                                    # fail loudly if the HIP library is missing
    if args.workload == "config5":
        return run_stage_workload(args)
    if args.workload == "pipeline":
        return run_pipeline_workload(args)
    if args.workload == "cp":
        return run_cp_workload(args)
    if args.workload == "headline":
        # the default line: the largest single-GPU block configuration as the headline, the two
        # smaller block configurations and the stage sweep (peak activation memory against batch
        # size) as extra keys of the same JSON line
        out = bench_block("config4", args.steps, args.warmup, peaks=True, baseline=not args.no_cpu_baseline)
        out["other_configs"] = {}
        for name in ("config2", "config3"):
            r = bench_block(name, max(args.steps // 2, 5), args.warmup, peaks=False, baseline=False)
            out["other_configs"][r["config"]["workload"]] = {
                k: r[k] for k in ("ms_per_step", "value", "unit", "mfma_util_pct", "gemm_tflops",
                                  "attention_tflops", "tokens_per_s", "roofline", "breakdown")}
            out["other_configs"][r["config"]["workload"]]["config"] = r["config"]
        if not args.no_stage_sweep:
            out["config5_stage_sweep"] = stage_sweep((8, 16, 32), 1, steps=2)
        print(json.dumps(out))
        return
    out = bench_block(args.workload, args.steps, args.warmup, peaks=True, baseline=not args.no_cpu_baseline,
                      copy_cal=args.copy_calibration)
    print(json.dumps(out))


def bench_block(workload, steps, warmup, peaks=True, baseline=True, copy_cal=False):
    """Times `steps` forward+backward passes of one block workload and returns the result record."""
    import torch
    from paper_2605_25451_amd import binding as bm
    from paper_2605_25451_amd.runner import CaseOnDevice
    if workload == "mmdit":
        import numpy as np
        from paper_2605_25451_amd.runner import TwoStreamOnDevice
        case = mmdit_case()
        dev = TwoStreamOnDevice(case)
        gemm_f, attn_f = mmdit_flops(case.cfg, case.cu[0], case.cu[1])
        tokens, n_seq = int(case.cu[0][-1] + case.cu[1][-1]), case.S
        max_seqlen = int(np.max(np.diff(case.cu[0]) + np.diff(case.cu[1])))
        extra = {"text_tokens": int(case.cu[0][-1]), "image_tokens": int(case.cu[1][-1]),
                 "step": "one two-stream block forward + backward (joint attention over [text ; image], "
                         "q/k RMS norm, weight grads accumulated in fp32)"}
        run_baseline = lambda: cpu_baseline_mmdit(case)
    else:
        case = make_workload(workload)
        dev = CaseOnDevice(case)
        gemm_f, attn_f = algorithmic_flops(case.cfg, case.cu_seqlens)
        tokens, n_seq, max_seqlen = case.T, case.S, case.max_seqlen
        extra = {"step": "one block forward + backward (weight grads accumulated in fp32)"}
        run_baseline = lambda: cpu_baseline(case)
    step_flops = 3.0 * gemm_f + 3.5 * attn_f

    for _ in range(warmup):
        dev.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        dev.step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / steps * 1e3
    tflops = step_flops / (ms_per_step * 1e-3) / 1e12

    # per-kernel-class durations: HIP events on the launch stream, same K steps
    bm.profile_begin()
    for _ in range(steps):
        dev.step()
    prof = bm.profile_end()
    torch.cuda.synchronize()
    breakdown = {}
    for cls, (ms, work, n) in prof.items():
        if n == 0:
            continue
        per_launch_ms = ms / n
        entry = {"ms_per_step": ms / steps, "launches_per_step": n / steps,
                 "avg_launch_us": per_launch_ms * 1e3}
        if cls.startswith("gemm") or cls.startswith("attn"):
            entry["tflops"] = work / (ms * 1e-3) / 1e12 if ms > 0 else None
        elif work > 0:
            entry["gbs"] = work / (ms * 1e-3) / 1e9 if ms > 0 else None
        breakdown[cls] = entry
    dom = max(breakdown, key=lambda c: breakdown[c]["ms_per_step"])
    d_ms, d_work, d_n = prof[dom]
    traffic_by_class, traffic_source = measured_traffic(case.name)
    traffic = traffic_by_class.get(dom)
    if dom.startswith("gemm") or dom.startswith("attn"):
        achieved = d_work / (d_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                    "avg_launch_us": d_ms / d_n * 1e3, "traffic": traffic}
    else:
        achieved = d_work / (d_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                    "avg_launch_us": d_ms / d_n * 1e3, "traffic": traffic}
    if traffic is not None:
        roofline["traffic_source"] = traffic_source
        if dom.startswith("gemm"):
            # the counter sits below the eight per-XCD L2s: an operand panel is fetched once by every
            # L2 whose tiles use it, and fetches that the memory-side cache serves are counted too
            roofline["traffic_note"] = ("FETCH_SIZE counts fetches below the per-XCD L2 caches "
                                        "(operand panels re-fetched per XCD, memory-side cache hits included)")
    gemm_ms = sum(prof[c][0] for c in ("gemm_nt", "gemm_nn", "gemm_tn"))
    gemm_work = sum(prof[c][1] for c in ("gemm_nt", "gemm_nn", "gemm_tn"))
    attn_ms = prof["attn_fwd"][0] + prof["attn_bwd"][0]
    attn_work = prof["attn_fwd"][1] + prof["attn_bwd"][1]

    out = {
        "metric": "block fwd+bwd TFLOP/s + MFMA util% on packed varlen multimodal tokens (bf16)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": case.name, "tokens": tokens, "sequences": n_seq,
                   "max_seqlen": max_seqlen, "hidden": case.cfg.hidden,
                   "heads": f"{case.cfg.n_q_heads}q/{case.cfg.n_kv_heads}kv x {case.cfg.head_dim}",
                   "mlp_hidden": case.cfg.mlp_hidden, **extra,
                   "flops_per_step": step_flops},
        "mfma_util_pct": 100.0 * tflops / MFMA_BF16_PEAK_TFLOPS,
        "gemm_tflops": gemm_work / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else None,
        "attention_tflops": attn_work / (attn_ms * 1e-3) / 1e12 if attn_ms > 0 else None,
        "tokens_per_s": tokens / (ms_per_step * 1e-3),
        "roofline": roofline,
        "breakdown": breakdown,
    }
    if peaks:
        out["measured_peaks"] = measured_peaks()
        out["paper_context"] = PAPER_CONTEXT
    if copy_cal:
        copy_calibration()
    del dev
    torch.cuda.empty_cache()
    if baseline:
        out["cpu_baseline"] = run_baseline()
    return out


if __name__ == "__main__":
    main()
