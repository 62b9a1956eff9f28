"""Seeded synthetic inputs for packed variable-length transformer blocks.

This module only *draws* data: block configurations, packed sequence lengths,
activations, parameters and upstream gradients.  It holds none of the block
arithmetic, so both the CPU oracle's tests and the HIP path's tests may use it
to obtain bit-identical inputs.

The workloads stand in for the multimodal mixtures the paper trains on
(packed sequences whose image-token counts are skewed per sample; Sec. 2.1
"Data heterogeneity", Sec. 4.1 "8K sequence length"): none of the paper's
datasets are reproduced, only their structure (length mix, image fraction).

Draw order for one case, all from ``numpy.random.default_rng(seed)``:
lengths, x, parameters in ``PARAM_NAMES`` order, dy, cond.
Values are drawn in fp32, rounded to the storage dtype (bf16 or fp32) and
returned as fp32 arrays that are exactly representable in that dtype.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np

PARAM_NAMES = (
    "norm1_g", "norm1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "norm2_g", "norm2_b", "w_up", "b_up", "w_down", "b_down",
    "w_ada", "b_ada",
    "w_router",
)

NORM_LAYERNORM, NORM_RMSNORM, NORM_ADALN = 0, 1, 2
ACT_GELU, ACT_SWIGLU = 0, 1
MASK_BIDIRECTIONAL, MASK_CAUSAL = 0, 1
DTYPE_BF16, DTYPE_FP32 = 0, 1


@dataclass(frozen=True)
class BlockConfig:
    """Shape and variant of one pre-norm transformer block."""
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp_hidden: int
    norm: int = NORM_LAYERNORM
    act: int = ACT_GELU
    mask: int = MASK_BIDIRECTIONAL
    rope: int = 0
    rope_base: float = 10000.0
    norm_eps: float = 1e-5
    linear_bias: int = 1
    dtype: int = DTYPE_BF16
    n_experts: int = 0          # > 0: mixture-of-experts FFN, mlp_hidden is the width of ONE expert
    top_k: int = 0
    router_std: float = 0.02    # std of the router matrix (drawn apart from the other weights)

    @property
    def qkv_dim(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def up_dim(self) -> int:
        return self.mlp_hidden * (2 if self.act == ACT_SWIGLU else 1)

    def param_shapes(self) -> Dict[str, tuple]:
        """Shapes of the parameters this variant owns (others are absent)."""
        d, f = self.hidden, self.mlp_hidden
        qd = self.n_q_heads * self.head_dim
        s: Dict[str, tuple] = {}
        if self.norm == NORM_LAYERNORM:
            s["norm1_g"] = (d,); s["norm1_b"] = (d,)
            s["norm2_g"] = (d,); s["norm2_b"] = (d,)
        elif self.norm == NORM_RMSNORM:
            s["norm1_g"] = (d,); s["norm2_g"] = (d,)
        s["w_qkv"] = (self.qkv_dim, d)
        s["w_o"] = (d, qd)
        e = max(self.n_experts, 1)
        s["w_up"] = (e * self.up_dim, d)        # expert-major; per expert gate rows first, then linear rows
        s["w_down"] = (e * d, f)                # expert-major; per expert a [d, f] matrix
        if self.n_experts > 0:
            s["w_router"] = (self.n_experts, d)
        if self.linear_bias:
            s["b_qkv"] = (self.qkv_dim,); s["b_o"] = (d,)
            s["b_up"] = (self.up_dim,); s["b_down"] = (d,)
        if self.norm == NORM_ADALN:
            s["w_ada"] = (6 * d, d); s["b_ada"] = (6 * d,)
        return {k: s[k] for k in PARAM_NAMES if k in s}


def vit_tiny(dtype: int = DTYPE_FP32) -> BlockConfig:
    return BlockConfig(hidden=64, n_q_heads=4, n_kv_heads=4, head_dim=16, mlp_hidden=256,
                       norm=NORM_LAYERNORM, act=ACT_GELU, mask=MASK_BIDIRECTIONAL,
                       rope=0, norm_eps=1e-5, linear_bias=1, dtype=dtype)


def vit_large(dtype: int = DTYPE_BF16) -> BlockConfig:
    return BlockConfig(hidden=1024, n_q_heads=16, n_kv_heads=16, head_dim=64, mlp_hidden=4096,
                       norm=NORM_LAYERNORM, act=ACT_GELU, mask=MASK_BIDIRECTIONAL,
                       rope=0, norm_eps=1e-5, linear_bias=1, dtype=dtype)


def decoder_7b(dtype: int = DTYPE_BF16) -> BlockConfig:
    return BlockConfig(hidden=4096, n_q_heads=32, n_kv_heads=32, head_dim=128, mlp_hidden=11008,
                       norm=NORM_RMSNORM, act=ACT_SWIGLU, mask=MASK_CAUSAL,
                       rope=1, rope_base=10000.0, norm_eps=1e-6, linear_bias=0, dtype=dtype)


def decoder_8b_gqa(dtype: int = DTYPE_BF16) -> BlockConfig:
    return BlockConfig(hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, mlp_hidden=14336,
                       norm=NORM_RMSNORM, act=ACT_SWIGLU, mask=MASK_CAUSAL,
                       rope=1, rope_base=500000.0, norm_eps=1e-6, linear_bias=0, dtype=dtype)


def decoder_moe(dtype: int = DTYPE_BF16) -> BlockConfig:
    """Decoder block with a mixture-of-experts FFN in the shape of the paper's backbone family
    (Sec. 4.1 names a 30B-A3B model): hidden 2048, 16 q / 4 kv heads of 128 (the library keeps
    hidden = heads x head size), 128 experts of width 768, 8 active per token, normalised
    top-k gates."""
    return BlockConfig(hidden=2048, n_q_heads=16, n_kv_heads=4, head_dim=128, mlp_hidden=768,
                       norm=NORM_RMSNORM, act=ACT_SWIGLU, mask=MASK_CAUSAL,
                       rope=1, rope_base=1000000.0, norm_eps=1e-6, linear_bias=0, dtype=dtype,
                       n_experts=128, top_k=8, router_std=0.02)


def dit_block(dtype: int = DTYPE_BF16) -> BlockConfig:
    return BlockConfig(hidden=1152, n_q_heads=16, n_kv_heads=16, head_dim=72, mlp_hidden=4608,
                       norm=NORM_ADALN, act=ACT_GELU, mask=MASK_BIDIRECTIONAL,
                       rope=0, norm_eps=1e-6, linear_bias=1, dtype=dtype)


def scaled(cfg: BlockConfig, **kw) -> BlockConfig:
    """A copy of ``cfg`` with some fields replaced (small variants for tests)."""
    return replace(cfg, **kw)


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------

def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def to_storage(a: np.ndarray, dtype: int) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return round_to_bf16(a) if dtype == DTYPE_BF16 else a


# --------------------------------------------------------------------------
# packed sequence lengths
# --------------------------------------------------------------------------

def _pack_to_total(draw, total: int) -> List[int]:
    """Draw lengths until their sum reaches ``total``; clip the last one so the
    sum is exact; a remainder shorter than 16 tokens joins the previous one."""
    lens: List[int] = []
    left = total
    while left > 0:
        n = int(draw())
        n = max(1, min(n, left))
        lens.append(n)
        left -= n
    if len(lens) > 1 and lens[-1] < 16:
        last = lens.pop()
        lens[-1] += last
    return lens


def lengths_images(rng, total: int, lo: int = 256, hi: int = 1024) -> List[int]:
    """One sequence per image, patch counts uniform in [lo, hi]."""
    return _pack_to_total(lambda: rng.integers(lo, hi + 1), total)


@dataclass
class Document:
    length: int
    spans: List[tuple] = field(default_factory=list)   # (kind, start, length), kind in {"image","text"}


def documents_interleaved(rng, total: int, image_range=(256, 1024), text_range=(32, 512)) -> List[Document]:
    """Documents of 1..3 (image span, text span) pairs, image first.
    Image spans uniform [256,1024] tokens, text spans uniform [32,512] by default."""
    docs: List[Document] = []
    left = total
    while left > 0:
        n_pairs = int(rng.integers(1, 4))
        spans, pos = [], 0
        for _ in range(n_pairs):
            li = int(rng.integers(image_range[0], image_range[1] + 1))
            lt = int(rng.integers(text_range[0], text_range[1] + 1))
            spans.append(("image", pos, li)); pos += li
            spans.append(("text", pos, lt)); pos += lt
        if pos > left:                      # clip the document to what is left
            clipped, pos2 = [], 0
            for kind, st, ln in spans:
                if st >= left:
                    break
                ln = min(ln, left - st)
                clipped.append((kind, st, ln)); pos2 = st + ln
            spans, pos = clipped, pos2
        docs.append(Document(pos, spans)); left -= pos
    if len(docs) > 1 and docs[-1].length < 16:
        last = docs.pop()
        base = docs[-1].length
        docs[-1].spans += [(k, base + s, l) for k, s, l in last.spans]
        docs[-1].length += last.length
    return docs


def documents_lognormal(rng, total: int, median: float = 1024.0, sigma: float = 1.0,
                        lo: int = 64, hi: int = 16384) -> List[Document]:
    """Heavy-tailed document lengths, each with an image-token fraction U[0.3,0.7]
    (one leading image span, then text; the split is metadata only)."""
    def draw():
        return int(np.clip(np.rint(np.exp(rng.normal(np.log(median), sigma))), lo, hi))
    lens = _pack_to_total(draw, total)
    docs = []
    for n in lens:
        frac = float(rng.uniform(0.3, 0.7))
        ni = int(round(frac * n))
        spans = [("image", 0, ni), ("text", ni, n - ni)] if 0 < ni < n else [("text", 0, n)]
        docs.append(Document(n, spans))
    return docs


def cu_from_lengths(lens) -> np.ndarray:
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lens, dtype=np.int64))
    return cu


def context_chunks(cu, C: int):
    """Partition of every packed sequence into C contiguous position ranges (the token layout of a
    context-parallel group of C ranks): chunk c of a sequence of length L holds its positions
    [c*L // C, (c+1)*L // C).  Returns, per chunk, (rows, cu_c): the rows of the full pack that
    the chunk holds, in order, and the offsets of the chunk's own packed layout (one entry per
    sequence; a short sequence leaves some chunks empty)."""
    cu = np.asarray(cu, dtype=np.int64)
    out = []
    for c in range(C):
        rows, lens = [], []
        for s in range(len(cu) - 1):
            L = int(cu[s + 1] - cu[s])
            a, b = c * L // C, (c + 1) * L // C
            rows.append(np.arange(cu[s] + a, cu[s] + b, dtype=np.int64))
            lens.append(b - a)
        out.append((np.concatenate(rows) if rows else np.zeros(0, dtype=np.int64), cu_from_lengths(lens)))
    return out


# --------------------------------------------------------------------------
# one block's inputs
# --------------------------------------------------------------------------

@dataclass
class BlockCase:
    cfg: BlockConfig
    cu_seqlens: np.ndarray                 # int32 [S+1]
    x: np.ndarray                          # fp32 [T, hidden], storage-representable
    params: Dict[str, np.ndarray]          # fp32, storage-representable
    dy: np.ndarray                         # fp32 [T, hidden]
    cond: Optional[np.ndarray] = None      # fp32 [S, hidden] (adaLN only)
    docs: Optional[List[Document]] = None
    name: str = ""

    @property
    def T(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def S(self) -> int:
        return len(self.cu_seqlens) - 1

    @property
    def max_seqlen(self) -> int:
        return int(np.max(np.diff(self.cu_seqlens)))


def _normal(rng, shape, std=1.0, mean=0.0):
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return a


def draw_params(rng, cfg: BlockConfig, std: float = 0.02) -> Dict[str, np.ndarray]:
    """Matrices, biases and beta ~ N(0, std); gamma = 1 + N(0, std)."""
    out = {}
    for name, shape in cfg.param_shapes().items():
        mean = 1.0 if name in ("norm1_g", "norm2_g") else 0.0
        sd = cfg.router_std if name == "w_router" else std
        out[name] = to_storage(_normal(rng, shape, sd, mean), cfg.dtype)
    return out


def make_case(cfg: BlockConfig, lens, seed: int, rng=None, docs=None, name: str = "",
              weight_std: float = 0.02) -> BlockCase:
    """Draw x, parameters, dy (and cond) for sequences of the given lengths."""
    if rng is None:
        rng = np.random.default_rng(seed)
    cu = cu_from_lengths(lens)
    T, S = int(cu[-1]), len(lens)
    x = to_storage(_normal(rng, (T, cfg.hidden)), cfg.dtype)
    params = draw_params(rng, cfg, weight_std)
    dy = to_storage(_normal(rng, (T, cfg.hidden)), cfg.dtype)
    cond = to_storage(_normal(rng, (S, cfg.hidden)), cfg.dtype) if cfg.norm == NORM_ADALN else None
    return BlockCase(cfg, cu, x, params, dy, cond, docs, name)


@dataclass
class TwoStreamCase:
    """Inputs of a two-stream (text / image) adaLN block: per stream the packed tokens, the
    per-sample offsets, the parameters and the upstream gradient; one conditioning row per
    sample.  Stream 0 is text, stream 1 is image."""
    cfg: BlockConfig
    cu: List[np.ndarray]
    x: List[np.ndarray]
    params: List[Dict[str, np.ndarray]]
    dy: List[np.ndarray]
    cond: np.ndarray
    qk_norm: int = 1
    name: str = ""

    @property
    def S(self) -> int:
        return len(self.cu[0]) - 1


def make_two_stream_case(cfg: BlockConfig, text_lens, image_lens, seed: int, qk_norm: int = 1,
                         name: str = "", weight_std: float = 0.02) -> TwoStreamCase:
    """Draw order: per stream (text, image) x, parameters (block parameters, then the q and k
    normalisation weights 1 + N(0, std) of length head_dim), dy; then cond."""
    assert cfg.norm == NORM_ADALN and len(text_lens) == len(image_lens)
    rng = np.random.default_rng(seed)
    cu, x, params, dy = [], [], [], []
    for lens in (text_lens, image_lens):
        c = cu_from_lengths(lens)
        T = int(c[-1])
        cu.append(c)
        x.append(to_storage(_normal(rng, (T, cfg.hidden)), cfg.dtype))
        p = draw_params(rng, cfg, weight_std)
        p["q_norm_g"] = to_storage(_normal(rng, (cfg.head_dim,), weight_std, 1.0), cfg.dtype)
        p["k_norm_g"] = to_storage(_normal(rng, (cfg.head_dim,), weight_std, 1.0), cfg.dtype)
        params.append(p)
        dy.append(to_storage(_normal(rng, (T, cfg.hidden)), cfg.dtype))
    cond = to_storage(_normal(rng, (len(text_lens), cfg.hidden)), cfg.dtype)
    return TwoStreamCase(cfg, cu, x, params, dy, cond, qk_norm, name)


def config1(seed: int = 0) -> BlockCase:
    """Tiny fp32 ViT block: two images of 16 and 24 patch tokens in one 40-token pack."""
    return make_case(vit_tiny(DTYPE_FP32), [16, 24], seed, name="config1_vit_tiny_fp32")


def config2(seed: int = 1, total: int = 16384) -> BlockCase:
    """ViT-L block over a pack of images with U[256,1024] patch tokens each."""
    rng = np.random.default_rng(seed)
    lens = lengths_images(rng, total)
    return make_case(vit_large(), lens, seed, rng=rng, name="config2_vit_large_bf16")


def config3(seed: int = 2, total: int = 8192) -> BlockCase:
    """7B-shaped decoder block over documents of alternating image/text spans."""
    rng = np.random.default_rng(seed)
    docs = documents_interleaved(rng, total)
    return make_case(decoder_7b(), [d.length for d in docs], seed, rng=rng, docs=docs,
                     name="config3_decoder_7b_bf16")


def config4(seed: int = 3, total: int = 32768) -> BlockCase:
    """8B-shaped GQA decoder block over heavy-tailed documents."""
    rng = np.random.default_rng(seed)
    docs = documents_lognormal(rng, total)
    return make_case(decoder_8b_gqa(), [d.length for d in docs], seed, rng=rng, docs=docs,
                     name="config4_decoder_8b_gqa_bf16")


def dit_case(seed: int = 4, n_images: int = 32, tokens_per_image: int = 256,
             cfg: Optional[BlockConfig] = None) -> BlockCase:
    """DiT-style generator block: one sequence of latent tokens per image."""
    cfg = cfg or dit_block()
    return make_case(cfg, [tokens_per_image] * n_images, seed, name="dit_block_bf16")


def sub_case(case: BlockCase, seq_ids) -> BlockCase:
    """The same case restricted to some of its sequences (same parameters)."""
    cu = case.cu_seqlens
    rows = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in seq_ids])
    lens = [int(cu[s + 1] - cu[s]) for s in seq_ids]
    cond = case.cond[list(seq_ids)] if case.cond is not None else None
    return BlockCase(case.cfg, cu_from_lengths(lens), case.x[rows], case.params, case.dy[rows],
                     cond, None, case.name + "_sub")


# --------------------------------------------------------------------------
# one pipeline stage's share: LLM microbatches with nested encoder / generator units
# --------------------------------------------------------------------------

@dataclass
class MicrobatchCase:
    cu_seqlens: np.ndarray            # documents
    base: np.ndarray                  # fp32 [T, llm.hidden] text-token activations (image rows get overwritten)
    image_rows: np.ndarray            # int32: LLM row of every encoder token of this microbatch, image by image
    image_lens: List[int]             # patch tokens per image
    image_last_row: np.ndarray        # int32 [n_images]: LLM row of the last token of each image span
    out_grad: np.ndarray              # fp32 [T, llm.hidden] (loss = <out, out_grad> when there is no generator)

    @property
    def T(self) -> int:
        return int(self.cu_seqlens[-1])


@dataclass
class UnitCase:
    cu_seqlens: np.ndarray            # one sequence per image
    patches: np.ndarray               # fp32 [T_enc, enc.hidden]
    latents: Optional[np.ndarray]     # fp32 [S*tokens_per_image, gen.hidden]
    targets: Optional[np.ndarray]


@dataclass
class StageCase:
    enc_cfg: BlockConfig
    llm_cfg: BlockConfig
    gen_cfg: Optional[BlockConfig]
    enc_params: List[Dict[str, np.ndarray]]
    llm_params: List[Dict[str, np.ndarray]]
    gen_params: List[Dict[str, np.ndarray]]
    proj_in: np.ndarray               # [llm.hidden, enc.hidden]
    proj_out: Optional[np.ndarray]    # [gen.hidden, llm.hidden]
    microbatches: List[MicrobatchCase]
    units: List[UnitCase]
    unit_size: int
    tokens_per_image: int

    @property
    def M(self) -> int:
        return len(self.microbatches)

    @property
    def has_generator(self) -> bool:
        return self.gen_cfg is not None and len(self.gen_params) > 0


def make_stage(enc_cfg: BlockConfig, llm_cfg: BlockConfig, gen_cfg: Optional[BlockConfig], n_enc: int,
               n_llm: int, n_gen: int, M: int, unit_size: int, llm_tokens: int, seed: int,
               image_range=(256, 1024), text_range=(32, 512), tokens_per_image: int = 256,
               proj_std: float = 0.02) -> StageCase:
    """Draw order: per-block parameters (encoder, LLM, generator), projectors, then per microbatch
    (documents, base, out_grad), then per unit (patches, latents, targets)."""
    rng = np.random.default_rng(seed)
    dt = llm_cfg.dtype
    enc_p = [draw_params(rng, enc_cfg) for _ in range(n_enc)]
    llm_p = [draw_params(rng, llm_cfg) for _ in range(n_llm)]
    gen_p = [draw_params(rng, gen_cfg) for _ in range(n_gen)] if gen_cfg is not None else []
    proj_in = to_storage(_normal(rng, (llm_cfg.hidden, enc_cfg.hidden), proj_std), dt)
    proj_out = (to_storage(_normal(rng, (gen_cfg.hidden, llm_cfg.hidden), proj_std), dt)
                if gen_cfg is not None and n_gen > 0 else None)
    mbs = []
    for _ in range(M):
        docs = documents_interleaved(rng, llm_tokens, image_range, text_range)
        cu = cu_from_lengths([d.length for d in docs])
        rows, lens, last = [], [], []
        for di, d in enumerate(docs):
            for kind, st, ln in d.spans:
                if kind == "image" and ln > 0:
                    r0 = int(cu[di]) + st
                    rows.extend(range(r0, r0 + ln)); lens.append(ln); last.append(r0 + ln - 1)
        base = to_storage(_normal(rng, (llm_tokens, llm_cfg.hidden)), dt)
        og = to_storage(_normal(rng, (llm_tokens, llm_cfg.hidden)), dt)
        mbs.append(MicrobatchCase(cu, base, np.asarray(rows, dtype=np.int32), lens,
                                  np.asarray(last, dtype=np.int32), og))
    units = []
    for u0 in range(0, M, unit_size):
        lens = [l for m in mbs[u0:u0 + unit_size] for l in m.image_lens]
        cu = cu_from_lengths(lens)
        patches = to_storage(_normal(rng, (int(cu[-1]), enc_cfg.hidden)), dt)
        lat = tgt = None
        if proj_out is not None:
            lat = to_storage(_normal(rng, (len(lens) * tokens_per_image, gen_cfg.hidden)), dt)
            tgt = to_storage(_normal(rng, (len(lens) * tokens_per_image, gen_cfg.hidden)), dt)
        units.append(UnitCase(cu, patches, lat, tgt))
    return StageCase(enc_cfg, llm_cfg, gen_cfg if proj_out is not None else None, enc_p, llm_p, gen_p,
                     proj_in, proj_out, mbs, units, unit_size, tokens_per_image)
