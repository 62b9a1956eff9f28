"""Thin ctypes binding over the C-ABI library (argument marshalling only).

Every function has the name and argument order of its C entry point in
``include/*.h``.  Tensors are torch device tensors used purely as
device memory: the binding passes their ``data_ptr()`` and the current HIP
stream.  There is no fallback: if the shared library is missing or a call
fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbigmac_block.so")

BM_OK = 0
BM_ERR_INVALID_ARG, BM_ERR_UNSUPPORTED, BM_ERR_WORKSPACE_TOO_SMALL, BM_ERR_HIP = -1, -2, -3, -4
GEMM_NT, GEMM_NN, GEMM_TN = 0, 1, 2
OP_ENC_FWD, OP_ENC_BWD, OP_LLM_FWD, OP_LLM_BWD, OP_GEN_FWD, OP_GEN_BWD = range(6)
ORDER_NESTED, ORDER_COMPUTE_EFFICIENT, ORDER_SEQUENTIAL, ORDER_MEMORY_EFFICIENT = 0, 1, 2, 3

PARAM_FIELDS = ("norm1_g", "norm1_b", "w_qkv", "b_qkv", "w_o", "b_o", "norm2_g", "norm2_b",
                "w_up", "b_up", "w_down", "b_down", "w_ada", "b_ada", "w_router")


class BmError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"bm_status {status}: {text}")
        self.status = status


class BlockDesc(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("mlp_hidden", C.c_int32), ("norm", C.c_int32),
                ("act", C.c_int32), ("mask", C.c_int32), ("rope", C.c_int32),
                ("rope_base", C.c_float), ("norm_eps", C.c_float), ("linear_bias", C.c_int32),
                ("dtype", C.c_int32), ("deterministic", C.c_int32),
                ("n_experts", C.c_int32), ("top_k", C.c_int32)]


class BlockParams(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_FIELDS]


class MmditDesc(C.Structure):
    _fields_ = [("block", BlockDesc), ("qk_norm", C.c_int32), ("qk_norm_eps", C.c_float)]


class MmditParams(C.Structure):
    _fields_ = [("stream", BlockParams * 2), ("q_norm_g", C.c_void_p * 2), ("k_norm_g", C.c_void_p * 2)]


class ExecutorConfig(C.Structure):
    _fields_ = [("enc", BlockDesc), ("llm", BlockDesc), ("gen", BlockDesc),
                ("n_enc_blocks", C.c_int32), ("n_llm_blocks", C.c_int32), ("n_gen_blocks", C.c_int32),
                ("M", C.c_int32), ("unit_size", C.c_int32), ("gen_tokens_per_image", C.c_int32)]


class ExecutorParams(C.Structure):
    _fields_ = [("enc", C.POINTER(BlockParams)), ("llm", C.POINTER(BlockParams)),
                ("gen", C.POINTER(BlockParams)), ("proj_in", C.c_void_p), ("proj_out", C.c_void_p)]


class Microbatch(C.Structure):
    _fields_ = [("T", C.c_int32), ("S", C.c_int32), ("cu_dev", C.c_void_p), ("cu_host", C.c_void_p),
                ("base", C.c_void_p), ("n_image_rows", C.c_int32), ("image_rows", C.c_void_p),
                ("n_images", C.c_int32), ("image_last_row", C.c_void_p), ("out_grad", C.c_void_p)]


class Unit(C.Structure):
    _fields_ = [("T", C.c_int32), ("S", C.c_int32), ("cu_dev", C.c_void_p), ("cu_host", C.c_void_p),
                ("patches", C.c_void_p), ("gen_cu_dev", C.c_void_p), ("gen_cu_host", C.c_void_p),
                ("latents", C.c_void_p), ("targets", C.c_void_p)]


class PipeOp(C.Structure):
    _fields_ = [("op", C.c_int32), ("index", C.c_int32), ("chunk", C.c_int32), ("column", C.c_int32)]


class PipeXOp(C.Structure):
    _fields_ = [("op", C.c_int32), ("index", C.c_int32), ("chunk", C.c_int32), ("peer", C.c_int32),
                ("what", C.c_int32)]


class PipeCommReport(C.Structure):
    _fields_ = [("deadlock", C.c_int32), ("unmatched", C.c_int32), ("fifo", C.c_int32),
                ("max_inflight", C.c_int32), ("messages", C.c_int64)]


class PipeReplayConfig(C.Structure):
    _fields_ = [("order", C.c_int32), ("P", C.c_int32), ("V", C.c_int32), ("M", C.c_int32),
                ("W", C.c_int32), ("has_generator", C.c_int32)] + \
               [(n, C.POINTER(C.c_double)) for n in ("llm_fwd", "llm_bwd", "enc_fwd", "enc_bwd",
                                                      "gen_fwd", "gen_bwd")] + \
               [("p2p", C.c_double), ("act_llm", C.c_double),
                ("act_enc", C.POINTER(C.c_double)), ("act_gen", C.POINTER(C.c_double))]


class PipeReplayResult(C.Structure):
    _fields_ = [("makespan", C.c_double), ("bubble", C.c_double)] + \
               [(n, C.POINTER(C.c_double)) for n in ("busy", "peak", "peak_enc", "peak_gen", "peak_llm")]



_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2605_25451_amd.build` "
                "(there is no fallback path)")
        # torch ships its own HIP runtime: load it first so that this library binds to the same
        # one (two runtimes in one process do not share devices, streams or allocations)
        import torch  # noqa: F401
        l = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        pi32 = C.POINTER(C.c_int32)
        l.bm_last_error.restype = C.c_char_p
        l.bm_block_sizes.argtypes = [C.POINTER(BlockDesc), i32, i32, i32, C.POINTER(sz), C.POINTER(sz)]
        l.bm_block_forward.argtypes = [C.POINTER(BlockDesc), C.POINTER(BlockParams), vp, vp, vp, i32,
                                       i32, i32, vp, vp, vp, vp, sz, vp]
        l.bm_block_backward.argtypes = [C.POINTER(BlockDesc), C.POINTER(BlockParams), vp, vp, vp, vp,
                                        i32, i32, i32, vp, vp, vp, C.POINTER(BlockParams), vp, vp, sz, vp]
        l.bm_block_moe_routing.argtypes = [C.POINTER(BlockDesc), i32, i32, vp, C.POINTER(vp), C.POINTER(vp)]
        l.bm_block_moe_routing.restype = C.c_int
        l.bm_gemm_scratch_bytes.argtypes = [i32] * 5
        l.bm_gemm_scratch_bytes.restype = sz
        l.bm_gemm.argtypes = [i32, i32, i32, i32, i32, vp, i32, vp, i32, vp, i32, vp, vp, sz, vp]
        l.bm_attention_forward.argtypes = [i32] * 5 + [vp, vp, vp, i32, vp, vp, i32, i32, i32, vp, vp, vp]
        l.bm_attention_backward_scratch_bytes.argtypes = [i32] * 4
        l.bm_attention_backward_scratch_bytes.restype = sz
        l.bm_attention_backward.argtypes = ([i32] * 5 + [vp, vp, vp, i32, vp, vp, vp, vp, vp, i32, i32,
                                                          i32, vp, vp, vp, i32, vp, sz, vp])
        l.bm_attention_backward_static_capacity.argtypes = []
        l.bm_attention_backward_static_capacity.restype = sz
        l.bm_attention_backward_static.argtypes = ([i32] * 5 + [vp, vp, vp, i32, vp, vp, vp, vp, vp, i32, i32,
                                                                i32, vp, vp, vp, i32, vp])
        l.bm_attention_backward_static.restype = C.c_int
        l.bm_profile_begin.argtypes = []
        l.bm_profile_end.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        l.bm_probe_mfma.argtypes = [i32, i32, vp, vp]
        l.bm_probe_copy.argtypes = [vp, vp, sz, vp]
        l.bm_probe_mfma_ex.argtypes = [i32, i32, i32, i32, vp, vp]
        l.bm_probe_mfma_ex.restype = C.c_int
        l.bm_probe_read.argtypes = [vp, sz, i32, i32, vp, vp]
        l.bm_probe_fill.argtypes = [vp, sz, i32, vp]
        l.bm_probe_lds.argtypes = [i32, i32, vp, sz, vp, vp]
        l.bm_probe_lds.restype = C.c_int
        l.bm_probe_issue.argtypes = [i32, i32, vp, vp]
        l.bm_probe_issue.restype = C.c_int
        l.bm_probe_read.restype = C.c_int
        l.bm_probe_fill.restype = C.c_int
        l.bm_probe_mfma.restype = C.c_int
        l.bm_probe_copy.restype = C.c_int
        l.bm_build_schedule.argtypes = [i32] * 6 + [pi32, pi32]
        l.bm_check_schedule.argtypes = [pi32, i32, i32, i32, i32, pi32]
        pcfg, ppar = C.POINTER(ExecutorConfig), C.POINTER(ExecutorParams)
        pmb, pun = C.POINTER(Microbatch), C.POINTER(Unit)
        l.bm_executor_arena_bytes.argtypes = [pcfg, pmb, pun, i32, i32, C.POINTER(sz)]
        l.bm_executor_create.argtypes = [pcfg, ppar, ppar, pmb, pun, vp, sz, i32, i32, C.POINTER(vp)]
        l.bm_executor_load_schedule.argtypes = [vp, pi32, i32]
        l.bm_executor_execute.argtypes = [vp, vp, vp]
        l.bm_executor_execute_timed.argtypes = [vp, vp, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
        l.bm_executor_execute_timed.restype = C.c_int
        l.bm_executor_peak_activation_bytes.argtypes = [vp]
        l.bm_executor_peak_activation_bytes.restype = sz
        l.bm_executor_peak_encoder_bytes.argtypes = [vp]
        l.bm_executor_peak_encoder_bytes.restype = sz
        l.bm_executor_destroy.argtypes = [vp]
        l.bm_executor_destroy.restype = None
        for name in ("bm_executor_arena_bytes", "bm_executor_create", "bm_executor_load_schedule",
                     "bm_executor_execute"):
            getattr(l, name).restype = C.c_int
        for name in ("bm_block_sizes", "bm_block_forward", "bm_block_backward", "bm_gemm",
                     "bm_attention_forward", "bm_attention_backward", "bm_build_schedule",
                     "bm_check_schedule", "bm_profile_begin", "bm_profile_end"):
            getattr(l, name).restype = C.c_int
        ppo = C.POINTER(PipeOp)
        l.bm_pipeline_llm_schedule.argtypes = [i32] * 4 + [ppo, pi32]
        l.bm_pipeline_build_schedule.argtypes = [i32] * 7 + [ppo, pi32]
        l.bm_pipeline_replay.argtypes = [C.POINTER(PipeReplayConfig), C.POINTER(PipeReplayResult)]
        l.bm_pipeline_comm_schedule.argtypes = [i32] * 7 + [C.POINTER(PipeXOp), pi32]
        l.bm_pipeline_check_comm.argtypes = [i32] * 6 + [C.POINTER(PipeCommReport)]
        for name in ("bm_pipeline_llm_schedule", "bm_pipeline_build_schedule", "bm_pipeline_replay",
                     "bm_pipeline_comm_schedule", "bm_pipeline_check_comm"):
            getattr(l, name).restype = C.c_int
        pmd, pmp = C.POINTER(MmditDesc), C.POINTER(MmditParams)
        l.bm_mmdit_sizes.argtypes = [pmd, i32, i32, i32, C.POINTER(sz), C.POINTER(sz)]
        l.bm_mmdit_forward.argtypes = [pmd, pmp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
        l.bm_mmdit_backward.argtypes = [pmd, pmp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, pmp,
                                        vp, vp, sz, vp]
        for name in ("bm_mmdit_sizes", "bm_mmdit_forward", "bm_mmdit_backward"):
            getattr(l, name).restype = C.c_int
        i64 = C.c_int64
        l.bm_cp_attention_forward.argtypes = [i32] * 5 + [vp, i32, vp, vp, i32, vp, vp, vp, vp, i32, vp, vp, vp]
        l.bm_cp_attention_merge.argtypes = [i32] * 5 + [C.POINTER(vp), C.POINTER(vp), vp, vp, vp]
        l.bm_cp_attention_backward_scratch_bytes.argtypes = [i32] * 5
        l.bm_cp_attention_backward_scratch_bytes.restype = sz
        l.bm_cp_attention_backward.argtypes = ([i32] * 5 + [vp, i32, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, i32,
                                                            vp, i32, vp, vp, i32, vp, sz, vp])
        l.bm_cp_sum_parts.argtypes = [i32, i64, i32, C.POINTER(vp), vp, vp]
        for name in ("bm_cp_attention_forward", "bm_cp_attention_merge", "bm_cp_attention_backward",
                     "bm_cp_sum_parts"):
            getattr(l, name).restype = C.c_int
        l.bm_cp_conversion_plan.argtypes = [i32, i32, i32, pi32, pi32, i32, pi32, pi32, pi32, pi32]
        l.bm_cp_encoder_unit_size.argtypes = [i32, i32, i32, pi32]
        l.bm_row_gather.argtypes = [i32, vp, vp, vp, i32, i32, vp]
        l.bm_row_scatter.argtypes = [i32, vp, vp, vp, i32, i32, vp]
        for name in ("bm_cp_conversion_plan", "bm_cp_encoder_unit_size", "bm_row_gather", "bm_row_scatter"):
            getattr(l, name).restype = C.c_int
        _lib = l
    return _lib


def _check(status: int):
    if status != BM_OK:
        raise BmError(status, lib().bm_last_error().decode())


def last_error() -> str:
    return lib().bm_last_error().decode()


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    return t.data_ptr() if hasattr(t, "data_ptr") else int(t)


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def make_desc(cfg) -> BlockDesc:
    """From any object with the BlockDesc field names (e.g. synth.BlockConfig)."""
    return BlockDesc(cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.mlp_hidden,
                     cfg.norm, cfg.act, cfg.mask, cfg.rope, cfg.rope_base, cfg.norm_eps,
                     cfg.linear_bias, cfg.dtype, getattr(cfg, "deterministic", 1),
                     getattr(cfg, "n_experts", 0), getattr(cfg, "top_k", 0))


def make_params(tensors: Dict[str, object]) -> BlockParams:
    p = BlockParams()
    for n in PARAM_FIELDS:
        setattr(p, n, _ptr(tensors.get(n)))
    return p


def _host_cu(cu_host) -> np.ndarray:
    a = np.ascontiguousarray(cu_host, dtype=np.int32)
    return a


# ---------------------------------------------------------------- entry points

def block_sizes(desc: BlockDesc, T: int, S: int, max_seqlen: int):
    saved, scratch = C.c_size_t(0), C.c_size_t(0)
    _check(lib().bm_block_sizes(C.byref(desc), T, S, max_seqlen, C.byref(saved), C.byref(scratch)))
    return saved.value, scratch.value


def block_forward(desc, w: BlockParams, x, cu_seqlens_dev, cu_seqlens_host, S, T, max_seqlen, cond,
                  y, saved, scratch, scratch_bytes, stream=None):
    cu_h = _host_cu(cu_seqlens_host)
    _check(lib().bm_block_forward(C.byref(desc), C.byref(w), _ptr(x), _ptr(cu_seqlens_dev),
                                  cu_h.ctypes.data, S, T, max_seqlen, _ptr(cond), _ptr(y),
                                  _ptr(saved), _ptr(scratch), scratch_bytes,
                                  _stream() if stream is None else stream))


def block_backward(desc, w: BlockParams, x, dy, cu_seqlens_dev, cu_seqlens_host, S, T, max_seqlen,
                   cond, saved, dx, grads: BlockParams, dcond, scratch, scratch_bytes, stream=None):
    cu_h = _host_cu(cu_seqlens_host)
    _check(lib().bm_block_backward(C.byref(desc), C.byref(w), _ptr(x), _ptr(dy),
                                   _ptr(cu_seqlens_dev), cu_h.ctypes.data, S, T, max_seqlen,
                                   _ptr(cond), _ptr(saved), _ptr(dx), C.byref(grads), _ptr(dcond),
                                   _ptr(scratch), scratch_bytes,
                                   _stream() if stream is None else stream))


def block_moe_routing(desc, T, S, saved):
    """Device addresses (inside ``saved``) of the expert choice int32 [T, top_k] and the gates fp32 [T, top_k]."""
    e, g = C.c_void_p(), C.c_void_p()
    _check(lib().bm_block_moe_routing(C.byref(desc), T, S, _ptr(saved), C.byref(e), C.byref(g)))
    return e.value, g.value


def make_mmdit_desc(cfg, qk_norm: int, qk_norm_eps: float = 1e-6) -> MmditDesc:
    return MmditDesc(make_desc(cfg), int(qk_norm), float(qk_norm_eps))


def make_mmdit_params(streams) -> MmditParams:
    """streams: two dicts of tensors (text, image), block parameter names plus q_norm_g / k_norm_g."""
    p = MmditParams()
    for s in range(2):
        p.stream[s] = make_params(streams[s])
        p.q_norm_g[s] = _ptr(streams[s].get("q_norm_g"))
        p.k_norm_g[s] = _ptr(streams[s].get("k_norm_g"))
    return p


def mmdit_sizes(desc: MmditDesc, T_text: int, T_img: int, S: int):
    saved, scratch = C.c_size_t(0), C.c_size_t(0)
    _check(lib().bm_mmdit_sizes(C.byref(desc), T_text, T_img, S, C.byref(saved), C.byref(scratch)))
    return saved.value, scratch.value


def mmdit_forward(desc, w: MmditParams, x_text, x_img, cu_text_dev, cu_text_host, cu_img_dev, cu_img_host, S,
                  cond, y_text, y_img, saved, scratch, scratch_bytes, stream=None):
    ct, ci = _host_cu(cu_text_host), _host_cu(cu_img_host)
    _check(lib().bm_mmdit_forward(C.byref(desc), C.byref(w), _ptr(x_text), _ptr(x_img), _ptr(cu_text_dev),
                                  ct.ctypes.data, _ptr(cu_img_dev), ci.ctypes.data, S, _ptr(cond),
                                  _ptr(y_text), _ptr(y_img), _ptr(saved), _ptr(scratch), scratch_bytes,
                                  _stream() if stream is None else stream))


def mmdit_backward(desc, w: MmditParams, x_text, x_img, dy_text, dy_img, cu_text_dev, cu_text_host,
                   cu_img_dev, cu_img_host, S, cond, saved, dx_text, dx_img, grads: MmditParams, dcond,
                   scratch, scratch_bytes, stream=None):
    ct, ci = _host_cu(cu_text_host), _host_cu(cu_img_host)
    _check(lib().bm_mmdit_backward(C.byref(desc), C.byref(w), _ptr(x_text), _ptr(x_img), _ptr(dy_text),
                                   _ptr(dy_img), _ptr(cu_text_dev), ct.ctypes.data, _ptr(cu_img_dev),
                                   ci.ctypes.data, S, _ptr(cond), _ptr(saved), _ptr(dx_text), _ptr(dx_img),
                                   C.byref(grads), _ptr(dcond), _ptr(scratch), scratch_bytes,
                                   _stream() if stream is None else stream))


def gemm_scratch_bytes(layout, M, N, K, dtype) -> int:
    return lib().bm_gemm_scratch_bytes(layout, M, N, K, dtype)


def gemm(layout, dtype, M, N, K, A, lda, B, ldb, Cmat, ldc, bias=None, scratch=None,
         scratch_bytes=0, stream=None):
    _check(lib().bm_gemm(layout, dtype, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(Cmat), ldc,
                         _ptr(bias), _ptr(scratch), scratch_bytes,
                         _stream() if stream is None else stream))


def attention_forward(dtype, mask, Hq, Hkv, dh, q, k, v, ld_qkv, cu_seqlens_dev, cu_seqlens_host,
                      S, T, max_seqlen, o, lse, stream=None):
    cu_h = _host_cu(cu_seqlens_host)
    _check(lib().bm_attention_forward(dtype, mask, Hq, Hkv, dh, _ptr(q), _ptr(k), _ptr(v), ld_qkv,
                                      _ptr(cu_seqlens_dev), cu_h.ctypes.data, S, T, max_seqlen,
                                      _ptr(o), _ptr(lse), _stream() if stream is None else stream))


def attention_backward_scratch_bytes(Hq, Hkv, dh, T) -> int:
    return lib().bm_attention_backward_scratch_bytes(Hq, Hkv, dh, T)


def attention_backward(dtype, mask, Hq, Hkv, dh, q, k, v, ld_qkv, o, d_o, lse, cu_seqlens_dev,
                       cu_seqlens_host, S, T, max_seqlen, dq, dk, dv, ld_dqkv, scratch,
                       scratch_bytes, stream=None):
    cu_h = _host_cu(cu_seqlens_host)
    _check(lib().bm_attention_backward(dtype, mask, Hq, Hkv, dh, _ptr(q), _ptr(k), _ptr(v), ld_qkv,
                                       _ptr(o), _ptr(d_o), _ptr(lse), _ptr(cu_seqlens_dev),
                                       cu_h.ctypes.data, S, T, max_seqlen, _ptr(dq), _ptr(dk),
                                       _ptr(dv), ld_dqkv, _ptr(scratch), scratch_bytes,
                                       _stream() if stream is None else stream))


def attention_backward_static_capacity() -> int:
    return lib().bm_attention_backward_static_capacity()


def attention_backward_static(dtype, mask, Hq, Hkv, dh, q, k, v, ld_qkv, o, d_o, lse, cu_seqlens_dev,
                              cu_seqlens_host, S, T, max_seqlen, dq, dk, dv, ld_dqkv, stream=None):
    cu_h = _host_cu(cu_seqlens_host)
    _check(lib().bm_attention_backward_static(dtype, mask, Hq, Hkv, dh, _ptr(q), _ptr(k), _ptr(v), ld_qkv,
                                              _ptr(o), _ptr(d_o), _ptr(lse), _ptr(cu_seqlens_dev),
                                              cu_h.ctypes.data, S, T, max_seqlen, _ptr(dq), _ptr(dk),
                                              _ptr(dv), ld_dqkv, _stream() if stream is None else stream))


def _ptr_array(tensors):
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = _ptr(t)
    return arr


def cp_attention_forward(dtype, mask, Hq, Hkv, dh, q, ld_q, k, v, ld_kv, cu_q_dev, cu_q_host, cu_k_dev,
                         cu_k_host, S, o_part, lse_part, stream=None):
    cq, ck = _host_cu(cu_q_host), _host_cu(cu_k_host)
    _check(lib().bm_cp_attention_forward(dtype, mask, Hq, Hkv, dh, _ptr(q), ld_q, _ptr(k), _ptr(v), ld_kv,
                                         _ptr(cu_q_dev), cq.ctypes.data, _ptr(cu_k_dev), ck.ctypes.data, S,
                                         _ptr(o_part), _ptr(lse_part),
                                         _stream() if stream is None else stream))


def cp_attention_merge(dtype, Hq, dh, Tq, o_parts, lse_parts, o, lse, stream=None):
    _check(lib().bm_cp_attention_merge(dtype, Hq, dh, Tq, len(o_parts), _ptr_array(o_parts),
                                       _ptr_array(lse_parts), _ptr(o), _ptr(lse),
                                       _stream() if stream is None else stream))


def cp_attention_backward_scratch_bytes(Hq, Hkv, dh, Tq, Tk) -> int:
    return lib().bm_cp_attention_backward_scratch_bytes(Hq, Hkv, dh, Tq, Tk)


def cp_attention_backward(dtype, mask, Hq, Hkv, dh, q, ld_q, k, v, ld_kv, o, d_o, lse, cu_q_dev, cu_q_host,
                          cu_k_dev, cu_k_host, S, dq_part, ld_dq, dk_part, dv_part, ld_dkv, scratch,
                          scratch_bytes, stream=None):
    cq, ck = _host_cu(cu_q_host), _host_cu(cu_k_host)
    _check(lib().bm_cp_attention_backward(dtype, mask, Hq, Hkv, dh, _ptr(q), ld_q, _ptr(k), _ptr(v), ld_kv,
                                          _ptr(o), _ptr(d_o), _ptr(lse), _ptr(cu_q_dev), cq.ctypes.data,
                                          _ptr(cu_k_dev), ck.ctypes.data, S, _ptr(dq_part), ld_dq,
                                          _ptr(dk_part), _ptr(dv_part), ld_dkv, _ptr(scratch), scratch_bytes,
                                          _stream() if stream is None else stream))


def cp_sum_parts(dtype, n, parts, out, stream=None):
    _check(lib().bm_cp_sum_parts(dtype, n, len(parts), _ptr_array(parts), _ptr(out),
                                 _stream() if stream is None else stream))


def cp_conversion_plan(enc_cp, llm_cp, image_lens, image_rows, cu_docs):
    """(counts [enc_cp, llm_cp], src_rows, dst_rows) as int32 numpy arrays (host planning)."""
    il = np.ascontiguousarray(image_lens, dtype=np.int32)
    ir = np.ascontiguousarray(image_rows, dtype=np.int32)
    cd = np.ascontiguousarray(cu_docs, dtype=np.int32)
    n = int(il.sum()) if len(il) else 0
    counts = np.zeros(enc_cp * llm_cp, dtype=np.int32)
    src, dst = np.zeros(max(n, 1), dtype=np.int32), np.zeros(max(n, 1), dtype=np.int32)
    p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    _check(lib().bm_cp_conversion_plan(enc_cp, llm_cp, len(il), p(il), p(ir), len(cd) - 1, p(cd), p(counts),
                                       p(src), p(dst)))
    return counts.reshape(enc_cp, llm_cp), src[:n], dst[:n]


def cp_encoder_unit_size(pp_size, llm_cp, enc_cp) -> int:
    out = C.c_int32(0)
    _check(lib().bm_cp_encoder_unit_size(pp_size, llm_cp, enc_cp, C.byref(out)))
    return out.value


def row_gather(dtype, src, rows_dev, dst, n, width, stream=None):
    _check(lib().bm_row_gather(dtype, _ptr(src), _ptr(rows_dev), _ptr(dst), n, width,
                               _stream() if stream is None else stream))


def row_scatter(dtype, src, rows_dev, dst, n, width, stream=None):
    _check(lib().bm_row_scatter(dtype, _ptr(src), _ptr(rows_dev), _ptr(dst), n, width,
                                _stream() if stream is None else stream))


def probe_mfma(blocks, iters, out, stream=None):
    _check(lib().bm_probe_mfma(blocks, iters, _ptr(out), _stream() if stream is None else stream))


def probe_mfma_ex(blocks, iters, shape16, random_operands, out, stream=None):
    _check(lib().bm_probe_mfma_ex(blocks, iters, shape16, random_operands, _ptr(out), _stream() if stream is None else stream))


def probe_copy(src, dst, nbytes, stream=None):
    _check(lib().bm_probe_copy(_ptr(src), _ptr(dst), nbytes, _stream() if stream is None else stream))


PROF_CLASSES = ("gemm_nt", "gemm_nn", "gemm_tn", "attn_fwd", "attn_bwd", "norm", "elementwise")


def probe_read(src, nbytes, blocks, unroll, out, stream=None):
    _check(lib().bm_probe_read(_ptr(src), nbytes, blocks, unroll, _ptr(out), _stream() if stream is None else stream))


def probe_fill(dst, nbytes, blocks, stream=None):
    _check(lib().bm_probe_fill(_ptr(dst), nbytes, blocks, _stream() if stream is None else stream))


def probe_lds(what, iters, src, src_bytes, out, stream=None):
    _check(lib().bm_probe_lds(what, iters, _ptr(src), src_bytes, _ptr(out), _stream() if stream is None else stream))


def probe_issue(n_valu, iters, out, stream=None):
    _check(lib().bm_probe_issue(n_valu, iters, _ptr(out), _stream() if stream is None else stream))


def profile_begin():
    _check(lib().bm_profile_begin())


def profile_end():
    """{class: (milliseconds, work, launches)}; work = flops (gemm/attn) or bytes."""
    n = len(PROF_CLASSES)
    ms, work, cnt = (C.c_double * n)(), (C.c_double * n)(), (C.c_int64 * n)()
    _check(lib().bm_profile_end(ms, work, cnt))
    return {PROF_CLASSES[i]: (ms[i], work[i], cnt[i]) for i in range(n)}


def build_schedule(order, M, unit_size, W, llm_depth, has_generator):
    """Returns a list of (opcode, index)."""
    n = C.c_int32(0)
    lib().bm_build_schedule(order, M, unit_size, W, llm_depth, int(has_generator), None, C.byref(n))
    if n.value <= 0:
        _check(BM_ERR_INVALID_ARG)
    buf = (C.c_int32 * (2 * n.value))()
    _check(lib().bm_build_schedule(order, M, unit_size, W, llm_depth, int(has_generator), buf, C.byref(n)))
    return [(buf[2 * i], buf[2 * i + 1]) for i in range(n.value)]


def check_schedule(ops, M, unit_size, has_generator):
    """Raises BmError if the op stream is not dependency safe; returns the peak
    live (encoder units, generator units, LLM microbatches)."""
    flat = (C.c_int32 * (2 * len(ops)))(*[v for op in ops for v in op])
    peak = (C.c_int32 * 3)()
    _check(lib().bm_check_schedule(flat, len(ops), M, unit_size, int(has_generator), peak))
    return tuple(peak)


# ---------------------------------------------------------------- multi-rank schedule and replay

def _pipe_ops(fn, *args):
    n = C.c_int32(0)
    fn(*args, None, C.byref(n))
    if n.value <= 0:
        _check(BM_ERR_INVALID_ARG)
    buf = (PipeOp * n.value)()
    _check(fn(*args, buf, C.byref(n)))
    return [(o.op, o.index, o.chunk, o.column) for o in buf[:n.value]]


def pipeline_llm_schedule(P, V, M, rank):
    """LLM ops of one rank: list of (opcode, microbatch, chunk, column)."""
    return _pipe_ops(lib().bm_pipeline_llm_schedule, P, V, M, rank)


def pipeline_build_schedule(order, P, V, M, W, has_generator, rank):
    """Program of one rank: list of (opcode, index, chunk, column)."""
    return _pipe_ops(lib().bm_pipeline_build_schedule, order, P, V, M, W, int(has_generator), rank)


OP_SEND, OP_RECV = 6, 7
MSG_NAMES = ("ACT", "GRAD", "FEAT", "FGRAD", "OUT", "OGRAD")


def pipeline_comm_schedule(order, P, V, M, W, has_generator, rank):
    """Program of one rank with communication operators: list of (opcode, index, chunk, peer, what);
    peer and what are -1 for compute ops."""
    fn = lib().bm_pipeline_comm_schedule
    n = C.c_int32(0)
    fn(order, P, V, M, W, int(has_generator), rank, None, C.byref(n))
    if n.value <= 0:
        _check(BM_ERR_INVALID_ARG)
    buf = (PipeXOp * n.value)()
    _check(fn(order, P, V, M, W, int(has_generator), rank, buf, C.byref(n)))
    return [(o.op, o.index, o.chunk, o.peer, o.what) for o in buf[:n.value]]


def pipeline_check_comm(order, P, V, M, W, has_generator):
    """Deadlock / matching report of the P rank programs (see bm_pipeline_check_comm)."""
    rep = PipeCommReport()
    _check(lib().bm_pipeline_check_comm(order, P, V, M, W, int(has_generator), C.byref(rep)))
    return {"deadlock": bool(rep.deadlock), "unmatched": rep.unmatched, "fifo": bool(rep.fifo),
            "max_inflight": rep.max_inflight, "messages": rep.messages}


def pipeline_replay(order, P, V, M, W, has_generator, llm_fwd, llm_bwd, enc_fwd, enc_bwd,
                    gen_fwd=None, gen_bwd=None, p2p=0.0, act_llm=0.0, act_enc=None, act_gen=None):
    """Replays the rank programs with the given operator seconds; returns a dict with makespan,
    bubble and per-rank busy / peak / peak_enc / peak_gen / peak_llm lists."""
    def arr(v, n):
        if v is None:
            return None
        if len(v) != n:
            raise ValueError(f"expected {n} values, got {len(v)}")
        return (C.c_double * n)(*[float(x) for x in v])
    keep = [arr(llm_fwd, P * V), arr(llm_bwd, P * V), arr(enc_fwd, M), arr(enc_bwd, M), arr(gen_fwd, M),
            arr(gen_bwd, M), arr(act_enc, M), arr(act_gen, M)]
    cast = lambda a: C.cast(a, C.POINTER(C.c_double)) if a is not None else None
    cfg = PipeReplayConfig(order, P, V, M, W, int(has_generator), cast(keep[0]), cast(keep[1]),
                           cast(keep[2]), cast(keep[3]), cast(keep[4]), cast(keep[5]), float(p2p),
                           float(act_llm), cast(keep[6]), cast(keep[7]))
    outs = [(C.c_double * P)() for _ in range(5)]
    res = PipeReplayResult(0.0, 0.0, *[cast(o) for o in outs])
    _check(lib().bm_pipeline_replay(C.byref(cfg), C.byref(res)))
    names = ("busy", "peak", "peak_enc", "peak_gen", "peak_llm")
    out = {"makespan": res.makespan, "bubble": res.bubble}
    out.update({n: list(o) for n, o in zip(names, outs)})
    return out


# ---------------------------------------------------------------- executor

def executor_arena_bytes(cfg: ExecutorConfig, mbs, units, enc_slots: int, llm_slots: int) -> int:
    n = C.c_size_t(0)
    _check(lib().bm_executor_arena_bytes(C.byref(cfg), mbs, units, enc_slots, llm_slots, C.byref(n)))
    return n.value


def executor_create(cfg, w: ExecutorParams, grads: ExecutorParams, mbs, units, arena, arena_bytes,
                    enc_slots, llm_slots):
    h = C.c_void_p()
    _check(lib().bm_executor_create(C.byref(cfg), C.byref(w), C.byref(grads), mbs, units, _ptr(arena),
                                    arena_bytes, enc_slots, llm_slots, C.byref(h)))
    return h


def executor_load_schedule(ex, ops):
    flat = (C.c_int32 * (2 * len(ops)))(*[v for op in ops for v in op])
    _check(lib().bm_executor_load_schedule(ex, flat, len(ops)))


def executor_execute(ex, loss, stream=None):
    _check(lib().bm_executor_execute(ex, _ptr(loss), _stream() if stream is None else stream))


def executor_execute_timed(h, loss, n_ops, stream=None):
    """Runs the loaded op stream with per-op event timing; returns (ms per op, live bytes after each op)."""
    ms = (C.c_double * n_ops)()
    live = (C.c_double * n_ops)()
    _check(lib().bm_executor_execute_timed(h, _ptr(loss), ms, live, _stream() if stream is None else stream))
    return list(ms), list(live)


def executor_peak_activation_bytes(ex) -> int:
    return lib().bm_executor_peak_activation_bytes(ex)


def executor_peak_encoder_bytes(ex) -> int:
    return lib().bm_executor_peak_encoder_bytes(ex)


def executor_destroy(ex):
    lib().bm_executor_destroy(ex)
