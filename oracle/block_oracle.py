"""CPU oracle for one packed variable-length transformer block (fp64, numpy).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
HIP path is compared against.  It is imported by ``tests/``, by
``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of ``bench.py``;
the product path never calls it and shares no code with it.

What it computes.  The paper (Sec. 2.1 "Multimodal LLMs" / "Model
heterogeneity", Sec. 4.1 "Models") names the three module kinds that every
pipeline unit executes -- ViT encoder blocks, LLM decoder blocks, diffusion
transformer generator blocks -- but gives no arithmetic for them.  The block
is therefore the standard pre-norm residual transformer block of each kind,
over *packed* sequences (Sec. 3.3 "sequence packing"): attention never
crosses a ``cu_seqlens`` boundary.

    h   = N1(x)                      LayerNorm | RMSNorm | LN0 + adaLN modulate
    qkv = h Wqkv^T + bqkv            q:[T,Hq,dh]  k,v:[T,Hkv,dh]
    q,k = RoPE(q,k)                  (decoder) positions restart per sequence
    o   = softmax(q k^T / sqrt(dh) + mask) v      per sequence, per head
    x1  = x + [gate1 *] (o Wo^T + bo)
    h2  = N2(x1)
    m   = gelu(h2 W1^T + b1) W2^T + b2     |  (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T
    y   = x1 + [gate2 *] m

Attention materialises the full L x L score matrix of each sequence: no
blocking, no online softmax.  The backward is written out by hand and is
pinned by finite differences and by a torch-CPU-float64 autograd cross-check
in the tests.  Pins: every function here is pinned by ``tests/test_oracle_*``.
The *choices* the paper leaves open (exact-erf GELU, rotate-half RoPE pairing,
biases, adaLN form) are conventions: parity unpinned against the paper itself,
which prints no worked numerical example.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
from scipy.special import erf

# Attention evaluates the kv heads of a sequence independently of each other, so a test that has
# to get through a 16384-token document in minutes may spread them over a few threads
# (BM_ORACLE_THREADS, default 1 = the plain loop).  Nothing about the arithmetic changes: every
# (sequence, head) matrix is computed by the same statements and the q heads of a group are
# added to their kv head's gradient in the same order, so the result is bit-identical to the
# serial loop (pinned in tests/test_oracle_block.py).
KV_HEAD_THREADS = max(1, int(os.environ.get("BM_ORACLE_THREADS", "1")))
KV_HEAD_DONE = None      # optional callable(kv_head): a long test prints its progress from here


def _each_kv_head(n, fn):
    def run(b):
        fn(b)
        if KV_HEAD_DONE is not None:
            KV_HEAD_DONE(b)

    w = min(KV_HEAD_THREADS, n)
    if w <= 1:
        for b in range(n):
            run(b)
    else:
        with ThreadPoolExecutor(max_workers=w) as ex:
            list(ex.map(run, range(n)))

F64 = np.float64


def _f64(a):
    return None if a is None else np.asarray(a, dtype=F64)


# ---------------------------------------------------------------- norms

def layernorm_fwd(x, gamma, beta, eps):
    """Biased-variance LayerNorm over the last axis; gamma/beta may be None."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = xc * rstd
    h = xhat
    if gamma is not None:
        h = h * gamma
    if beta is not None:
        h = h + beta
    return h, (xhat, rstd)


def layernorm_bwd(dh, gamma, cache):
    xhat, rstd = cache
    g = dh * gamma if gamma is not None else dh
    dx = rstd * (g - g.mean(axis=-1, keepdims=True)
                 - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    dgamma = (dh * xhat).sum(axis=0)
    dbeta = dh.sum(axis=0)
    return dx, dgamma, dbeta


def rmsnorm_fwd(x, gamma, eps):
    r = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps)
    return x * r * gamma, (x, r)


def rmsnorm_bwd(dh, gamma, cache):
    x, r = cache
    g = dh * gamma
    dx = r * g - x * (r ** 3) * (g * x).mean(axis=-1, keepdims=True)
    dgamma = (dh * x * r).sum(axis=0)
    return dx, dgamma


# ---------------------------------------------------------------- activations

def gelu(z):
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def gelu_grad(z):
    cdf = 0.5 * (1.0 + erf(z / np.sqrt(2.0)))
    pdf = np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)
    return cdf + z * pdf


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def silu(z):
    return z * sigmoid(z)


def silu_grad(z):
    s = sigmoid(z)
    return s * (1.0 + z * (1.0 - s))


# ---------------------------------------------------------------- RoPE

def rope_angles(positions, head_dim, base):
    """theta[p, i] = p * base^(-2i/dh), i in [0, dh/2)."""
    i = np.arange(head_dim // 2, dtype=F64)
    inv_freq = base ** (-2.0 * i / head_dim)
    return positions[:, None].astype(F64) * inv_freq[None, :]


def rope_apply(t, theta, sign=1.0):
    """Rotate-half pairing (i, i+dh/2) of t[T, H, dh] by sign*theta[T, dh/2]."""
    half = t.shape[-1] // 2
    c = np.cos(theta)[:, None, :]
    s = sign * np.sin(theta)[:, None, :]
    a, b = t[..., :half], t[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def positions_in_sequence(cu):
    """Token position counted from the start of its own sequence."""
    T = int(cu[-1])
    pos = np.zeros(T, dtype=np.int64)
    for s in range(len(cu) - 1):
        pos[cu[s]:cu[s + 1]] = np.arange(cu[s + 1] - cu[s])
    return pos


# ---------------------------------------------------------------- attention

def attention_probs(q, k, causal):
    """softmax(q k^T / sqrt(dh)) of one head of one sequence; q,k: [L, dh]."""
    L, dh = q.shape
    sc = (q @ k.T) / np.sqrt(dh)
    if causal:
        sc = np.where(np.tril(np.ones((L, L), dtype=bool)), sc, -np.inf)
    sc = sc - sc.max(axis=-1, keepdims=True)
    e = np.exp(sc)
    return e / e.sum(axis=-1, keepdims=True)


def attention_fwd(q, k, v, cu, causal):
    """q:[T,Hq,dh] k,v:[T,Hkv,dh] -> o:[T,Hq,dh].  q head a uses kv head
    a // (Hq/Hkv)."""
    T, Hq, dh = q.shape
    group = Hq // k.shape[1]
    o = np.zeros_like(q)
    for s in range(len(cu) - 1):
        lo, hi = int(cu[s]), int(cu[s + 1])

        def kv_head(b):
            for a in range(b * group, (b + 1) * group):
                p = attention_probs(q[lo:hi, a], k[lo:hi, b], causal)
                o[lo:hi, a] = p @ v[lo:hi, b]

        _each_kv_head(k.shape[1], kv_head)
    return o


def attention_bwd(do, q, k, v, cu, causal):
    T, Hq, dh = q.shape
    group = Hq // k.shape[1]
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    scale = 1.0 / np.sqrt(dh)
    for s in range(len(cu) - 1):
        lo, hi = int(cu[s]), int(cu[s + 1])

        def kv_head(b):
            for a in range(b * group, (b + 1) * group):
                p = attention_probs(q[lo:hi, a], k[lo:hi, b], causal)
                d_o = do[lo:hi, a]
                dv[lo:hi, b] += p.T @ d_o
                dp = d_o @ v[lo:hi, b].T
                dsc = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
                dq[lo:hi, a] = dsc @ k[lo:hi, b] * scale
                dk[lo:hi, b] += dsc.T @ q[lo:hi, a] * scale

        _each_kv_head(k.shape[1], kv_head)
    return dq, dk, dv


# ---------------------------------------------------------------- adaLN helpers

def _seq_of_token(cu):
    T = int(cu[-1])
    sid = np.zeros(T, dtype=np.int64)
    for s in range(len(cu) - 1):
        sid[cu[s]:cu[s + 1]] = s
    return sid


def _segment_sum(a, cu):
    return np.stack([a[cu[s]:cu[s + 1]].sum(axis=0) for s in range(len(cu) - 1)])


# ---------------------------------------------------------------- the block

NORM_LAYERNORM, NORM_RMSNORM, NORM_ADALN = 0, 1, 2
ACT_GELU, ACT_SWIGLU = 0, 1


# ---------------------------------------------------------------------------
# mixture-of-experts FFN (the paper's LLM backbone is a mixture-of-experts model,
# Sec. 4.1, and Sec. 3.3 names expert imbalance as a source of uneven operator
# times; it gives no arithmetic).  Reading: router logits = h W_r^T (no bias),
# probabilities = softmax over the experts, the k most probable experts are
# chosen (ties: lower expert index), their probabilities renormalised to sum 1
# are the gates, every expert is a SwiGLU FFN, no token is dropped, no
# auxiliary loss.
# ---------------------------------------------------------------------------

def moe_route(logits, k, expert_choice=None):
    """(idx [T,k] by descending probability, gate [T,k], probs [T,E]).

    ``expert_choice`` (int [T,k], distinct experts per token) replaces the top-k decision: the
    choice is an integer taken from floating-point logits, so where two logits are closer than
    the rounding of an implementation's own arithmetic several choices are correct; a test
    hands that implementation's (admissible) choice in and compares everything else, which is
    then unique.  Probabilities, gates and every gradient formula are unchanged."""
    z = logits - logits.max(axis=1, keepdims=True)
    e = np.exp(z)
    probs = e / e.sum(axis=1, keepdims=True)
    T, E = probs.shape
    if expert_choice is not None:
        idx = np.asarray(expert_choice, dtype=np.int64)
        assert idx.shape == (T, k) and idx.min() >= 0 and idx.max() < E
        assert all(len(set(row)) == k for row in idx.tolist()), "an expert is chosen twice for one token"
    else:
        # descending probability, ties to the lower expert index (stable sort of the negated row)
        idx = np.argsort(-probs, axis=1, kind="stable")[:, :k]
    sel = np.take_along_axis(probs, idx, axis=1)
    gate = sel / sel.sum(axis=1, keepdims=True)
    return idx, gate, probs


def moe_ffn_fwd(h, p, E, k, F, expert_choice=None):
    """out[t] = sum_j gate[t,j] * FFN_{idx[t,j]}(h[t]);  returns (out, cache).
    Expert by expert: the tokens (and their choice slot j) that picked expert e."""
    T, d = h.shape
    logits = h @ p["w_router"].T
    idx, gate, probs = moe_route(logits, k, expert_choice)
    w_up = p["w_up"].reshape(E, 2 * F, d)
    w_down = p["w_down"].reshape(E, d, F)
    ys = np.zeros((T, k, d))
    ups = np.zeros((T, k, 2 * F))
    acts = np.zeros((T, k, F))
    for e in range(E):
        t, j = np.nonzero(idx == e)
        if t.size == 0:
            continue
        up = h[t] @ w_up[e].T
        a = silu(up[:, :F]) * up[:, F:]
        ups[t, j], acts[t, j] = up, a
        ys[t, j] = a @ w_down[e].T
    out = (gate[:, :, None] * ys).sum(axis=1)
    return out, dict(idx=idx, gate=gate, probs=probs, ys=ys, ups=ups, acts=acts)


def moe_ffn_bwd(dm, h, p, mc, E, k, F):
    """Gradients of moe_ffn_fwd: (dh, {"w_router", "w_up", "w_down"})."""
    T, d = h.shape
    idx, gate, probs, ys, ups, acts = (mc[n] for n in ("idx", "gate", "probs", "ys", "ups", "acts"))
    w_up = p["w_up"].reshape(E, 2 * F, d)
    w_down = p["w_down"].reshape(E, d, F)
    g_up = np.zeros_like(w_up); g_down = np.zeros_like(w_down)
    dh = np.zeros_like(h)
    dgate = np.einsum("td,tkd->tk", dm, ys)
    for e in range(E):
        t, j = np.nonzero(idx == e)
        if t.size == 0:
            continue
        dy = gate[t, j][:, None] * dm[t]
        g_down[e] = dy.T @ acts[t, j]
        da = dy @ w_down[e]
        gt, lin = ups[t, j, :F], ups[t, j, F:]
        dup = np.concatenate([da * lin * silu_grad(gt), da * silu(gt)], axis=1)
        g_up[e] = dup.T @ h[t]
        np.add.at(dh, t, dup @ w_up[e])
    # gates = selected probabilities / their sum; probabilities = softmax(logits)
    sel = np.take_along_axis(probs, idx, axis=1)
    ssum = sel.sum(axis=1, keepdims=True)
    dsel = (dgate - (dgate * gate).sum(axis=1, keepdims=True)) / ssum
    dprobs = np.zeros_like(probs)
    np.put_along_axis(dprobs, idx, dsel, axis=1)
    dlogits = probs * (dprobs - (probs * dprobs).sum(axis=1, keepdims=True))
    g_router = dlogits.T @ h
    dh += dlogits @ p["w_router"]
    return dh, {"w_router": g_router, "w_up": g_up.reshape(E * 2 * F, d), "w_down": g_down.reshape(E * d, F)}


def block_forward(cfg, params, x, cu_seqlens, cond=None, expert_choice=None):
    """Forward of one block.  ``cfg`` needs the fields hidden, n_q_heads,
    n_kv_heads, head_dim, mlp_hidden, norm, act, mask, rope, rope_base,
    norm_eps.  ``expert_choice``: see moe_route.  Returns (y, cache)."""
    p = {k: _f64(v) for k, v in params.items()}
    x = _f64(x); cu = np.asarray(cu_seqlens, dtype=np.int64)
    T, d = x.shape
    Hq, Hkv, dh, F = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.mlp_hidden
    causal = bool(cfg.mask)
    c = {"cu": cu}

    if cfg.norm == NORM_ADALN:
        cond = _f64(cond)
        sid = _seq_of_token(cu)
        mod = silu(cond) @ p["w_ada"].T + p["b_ada"]           # [S, 6d]
        sh1, sc1, g1, sh2, sc2, g2 = [mod[:, i * d:(i + 1) * d] for i in range(6)]
        c.update(cond=cond, sid=sid, mod=mod)

    # --- attention half
    if cfg.norm == NORM_LAYERNORM:
        h, c["n1"] = layernorm_fwd(x, p["norm1_g"], p["norm1_b"], cfg.norm_eps)
    elif cfg.norm == NORM_RMSNORM:
        h, c["n1"] = rmsnorm_fwd(x, p["norm1_g"], cfg.norm_eps)
    else:
        xhat, c["n1"] = layernorm_fwd(x, None, None, cfg.norm_eps)
        h = xhat * (1.0 + sc1[sid]) + sh1[sid]
    qkv = h @ p["w_qkv"].T
    if "b_qkv" in p:
        qkv = qkv + p["b_qkv"]
    q = qkv[:, :Hq * dh].reshape(T, Hq, dh)
    k = qkv[:, Hq * dh:(Hq + Hkv) * dh].reshape(T, Hkv, dh)
    v = qkv[:, (Hq + Hkv) * dh:].reshape(T, Hkv, dh)
    if cfg.rope:
        theta = rope_angles(positions_in_sequence(cu), dh, cfg.rope_base)
        q = rope_apply(q, theta); k = rope_apply(k, theta)
        c["theta"] = theta
    o = attention_fwd(q, k, v, cu, causal)
    attn = o.reshape(T, Hq * dh) @ p["w_o"].T
    if "b_o" in p:
        attn = attn + p["b_o"]
    x1 = x + (g1[sid] * attn if cfg.norm == NORM_ADALN else attn)

    # --- MLP half
    if cfg.norm == NORM_LAYERNORM:
        h2, c["n2"] = layernorm_fwd(x1, p["norm2_g"], p["norm2_b"], cfg.norm_eps)
    elif cfg.norm == NORM_RMSNORM:
        h2, c["n2"] = rmsnorm_fwd(x1, p["norm2_g"], cfg.norm_eps)
    else:
        xhat2, c["n2"] = layernorm_fwd(x1, None, None, cfg.norm_eps)
        h2 = xhat2 * (1.0 + sc2[sid]) + sh2[sid]
    E = getattr(cfg, "n_experts", 0)
    if E > 0:
        m, c["moe"] = moe_ffn_fwd(h2, p, E, cfg.top_k, F, expert_choice)
        up = a = None
    else:
        up = h2 @ p["w_up"].T
        if "b_up" in p:
            up = up + p["b_up"]
        if cfg.act == ACT_GELU:
            a = gelu(up)
        else:
            a = silu(up[:, :F]) * up[:, F:]
        m = a @ p["w_down"].T
        if "b_down" in p:
            m = m + p["b_down"]
    y = x1 + (g2[sid] * m if cfg.norm == NORM_ADALN else m)

    c.update(x=x, h=h, q=q, k=k, v=v, o=o, attn=attn, x1=x1, h2=h2, up=up, a=a, m=m)
    return y, c


def block_backward(cfg, params, cache, dy):
    """Backward of one block.  Returns (dx, grads, dcond); ``grads`` has one
    entry per parameter the variant owns."""
    p = {k: _f64(v) for k, v in params.items()}
    c = cache; dy = _f64(dy); cu = c["cu"]
    T, d = dy.shape
    Hq, Hkv, dh, F = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.mlp_hidden
    causal = bool(cfg.mask)
    ada = cfg.norm == NORM_ADALN
    g = {}
    if ada:
        sid, mod = c["sid"], c["mod"]
        sh1, sc1, g1, sh2, sc2, g2 = [mod[:, i * d:(i + 1) * d] for i in range(6)]
        dmod = np.zeros_like(mod)

    # --- y = x1 + [g2 *] m
    dx1 = dy.copy()
    if ada:
        dmod[:, 5 * d:6 * d] = _segment_sum(dy * c["m"], cu)
        dm = dy * g2[sid]
    else:
        dm = dy
    E = getattr(cfg, "n_experts", 0)
    if E > 0:
        dh2, gm = moe_ffn_bwd(dm, c["h2"], p, c["moe"], E, cfg.top_k, F)
        g.update(gm)
    else:
        g["w_down"] = dm.T @ c["a"]
        if "b_down" in p:
            g["b_down"] = dm.sum(axis=0)
        da = dm @ p["w_down"]
        up = c["up"]
        if cfg.act == ACT_GELU:
            dup = da * gelu_grad(up)
        else:
            gate, lin = up[:, :F], up[:, F:]
            dup = np.concatenate([da * lin * silu_grad(gate), da * silu(gate)], axis=1)
        g["w_up"] = dup.T @ c["h2"]
        if "b_up" in p:
            g["b_up"] = dup.sum(axis=0)
        dh2 = dup @ p["w_up"]
    if cfg.norm == NORM_LAYERNORM:
        dxn, g["norm2_g"], g["norm2_b"] = layernorm_bwd(dh2, p["norm2_g"], c["n2"])
    elif cfg.norm == NORM_RMSNORM:
        dxn, g["norm2_g"] = rmsnorm_bwd(dh2, p["norm2_g"], c["n2"])
    else:
        xhat2 = c["n2"][0]
        dmod[:, 4 * d:5 * d] = _segment_sum(dh2 * xhat2, cu)     # dscale2
        dmod[:, 3 * d:4 * d] = _segment_sum(dh2, cu)             # dshift2
        dxn, _, _ = layernorm_bwd(dh2 * (1.0 + sc2[sid]), None, c["n2"])
    dx1 = dx1 + dxn

    # --- x1 = x + [g1 *] attn
    dx = dx1.copy()
    if ada:
        dmod[:, 2 * d:3 * d] = _segment_sum(dx1 * c["attn"], cu)
        dattn = dx1 * g1[sid]
    else:
        dattn = dx1
    o2 = c["o"].reshape(T, Hq * dh)
    g["w_o"] = dattn.T @ o2
    if "b_o" in p:
        g["b_o"] = dattn.sum(axis=0)
    do = (dattn @ p["w_o"]).reshape(T, Hq, dh)
    dq, dk, dv = attention_bwd(do, c["q"], c["k"], c["v"], cu, causal)
    if cfg.rope:
        dq = rope_apply(dq, c["theta"], sign=-1.0)
        dk = rope_apply(dk, c["theta"], sign=-1.0)
    dqkv = np.concatenate([dq.reshape(T, -1), dk.reshape(T, -1), dv.reshape(T, -1)], axis=1)
    g["w_qkv"] = dqkv.T @ c["h"]
    if "b_qkv" in p:
        g["b_qkv"] = dqkv.sum(axis=0)
    dh1 = dqkv @ p["w_qkv"]
    if cfg.norm == NORM_LAYERNORM:
        dxn, g["norm1_g"], g["norm1_b"] = layernorm_bwd(dh1, p["norm1_g"], c["n1"])
    elif cfg.norm == NORM_RMSNORM:
        dxn, g["norm1_g"] = rmsnorm_bwd(dh1, p["norm1_g"], c["n1"])
    else:
        xhat1 = c["n1"][0]
        dmod[:, 1 * d:2 * d] = _segment_sum(dh1 * xhat1, cu)     # dscale1
        dmod[:, 0 * d:1 * d] = _segment_sum(dh1, cu)             # dshift1
        dxn, _, _ = layernorm_bwd(dh1 * (1.0 + sc1[sid]), None, c["n1"])
    dx = dx + dxn

    dcond = None
    if ada:
        cond = c["cond"]
        g["w_ada"] = dmod.T @ silu(cond)
        g["b_ada"] = dmod.sum(axis=0)
        dcond = (dmod @ p["w_ada"]) * silu_grad(cond)
    return dx, g, dcond


def block_fwd_bwd(cfg, params, x, cu_seqlens, dy, cond=None, expert_choice=None):
    y, cache = block_forward(cfg, params, x, cu_seqlens, cond, expert_choice)
    dx, grads, dcond = block_backward(cfg, params, cache, dy)
    return y, dx, grads, dcond
