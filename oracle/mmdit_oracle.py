"""CPU oracle for a two-stream (text / image) adaLN transformer block with joint attention.

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and smoke/bench baseline
legs), never by the product path, and sharing no code with it.

The paper names its generator only as a "20 B MMDiT" built from attention
operators (Sec. 4.1) and gives no arithmetic.  Reading: the two-stream block
of the multimodal diffusion transformer literature.  Each sample has a text
token sequence and an image token sequence; every per-token operator (adaLN
modulation from a shared per-sample conditioning vector, QKV / output / MLP
projections, the optional RMS normalisation of q and k over the head
dimension) has its own parameters per stream, and attention runs once,
bidirectionally, over the concatenation [text tokens ; image tokens] of a
sample.  Per stream s (pre-norm, adaLN-Zero style, GELU(erf) MLP):

  mod_s = silu(c) W_ada_s^T + b_ada_s = [sh1, sc1, g1, sh2, sc2, g2]
  h     = LN0(x_s) (1 + sc1) + sh1
  q,k,v = h W_qkv_s^T + b_qkv_s ;  q <- rms_dh(q) gq_s,  k <- rms_dh(k) gk_s   (if qk_norm)
  o     = joint softmax attention of the sample, rows of stream s
  x1    = x_s + g1 (o W_o_s^T + b_o_s)
  y_s   = x1 + g2 (gelu(LN0(x1)(1 + sc2) + sh2) W_up_s^T + b_up_s) W_down_s^T + b_down_s)

Streams are packed separately: x[s] is [T_s, d] with cu[s] the per-sample
offsets of stream s (a sample may have zero text tokens).

Pins: tests/test_oracle_mmdit.py (finite differences; with an empty text
stream and qk_norm off the block is the single-stream adaLN block of
block_oracle; joint attention against a brute-force loop; stream exchange).
"""
from __future__ import annotations

import numpy as np

from oracle import block_oracle as bo

STREAM_PARAMS = ("w_qkv", "b_qkv", "w_o", "b_o", "w_up", "b_up", "w_down", "b_down", "w_ada", "b_ada",
                 "q_norm_g", "k_norm_g")


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def _rms_heads_fwd(t, g, eps):
    """t [T,H,dh]: t / sqrt(mean_dh t^2 + eps) * g[dh]."""
    r = 1.0 / np.sqrt((t * t).mean(axis=2, keepdims=True) + eps)
    return t * r * g, r


def _rms_heads_bwd(dout, t, g, r):
    gh = dout * g
    dt = r * gh - t * (r ** 3) * (gh * t).mean(axis=2, keepdims=True)
    dg = (dout * t * r).sum(axis=(0, 1))
    return dt, dg


def joint_layout(cu_text, cu_img):
    """Joint sequences [text ; image] per sample: (joint cu, index of every joint row as
    (stream, row in that stream))."""
    cu_t = np.asarray(cu_text, dtype=np.int64); cu_i = np.asarray(cu_img, dtype=np.int64)
    S = len(cu_t) - 1
    stream, row, cu = [], [], [0]
    for s in range(S):
        for r in range(cu_t[s], cu_t[s + 1]):
            stream.append(0); row.append(r)
        for r in range(cu_i[s], cu_i[s + 1]):
            stream.append(1); row.append(r)
        cu.append(len(stream))
    return np.asarray(cu, dtype=np.int64), np.asarray(stream, dtype=np.int64), np.asarray(row, dtype=np.int64)


def mmdit_forward(cfg, params, x, cu, cond, qk_norm=True, qk_eps=1e-6):
    """cfg: hidden, n_q_heads (= n_kv_heads), head_dim, mlp_hidden, norm_eps.
    params[s], x[s], cu[s] for stream s in (0 text, 1 image); cond [S, d].
    Returns ([y_text, y_img], cache)."""
    d, H, dh, F = cfg.hidden, cfg.n_q_heads, cfg.head_dim, cfg.mlp_hidden
    cond = _f64(cond)
    c = {"cond": cond, "st": []}
    jcu, jstream, jrow = joint_layout(cu[0], cu[1])
    Tj = len(jstream)
    q_j = np.zeros((Tj, H, dh)); k_j = np.zeros((Tj, H, dh)); v_j = np.zeros((Tj, H, dh))
    for s in range(2):
        p = {n: _f64(v) for n, v in params[s].items()}
        xs = _f64(x[s]); cus = np.asarray(cu[s], dtype=np.int64)
        T = xs.shape[0]
        sid = bo._seq_of_token(cus) if T else np.zeros(0, dtype=np.int64)
        mod = bo.silu(cond) @ p["w_ada"].T + p["b_ada"]
        sh1, sc1, g1, sh2, sc2, g2 = [mod[:, i * d:(i + 1) * d] for i in range(6)]
        xhat, n1 = bo.layernorm_fwd(xs, None, None, cfg.norm_eps)
        h = xhat * (1.0 + sc1[sid]) + sh1[sid]
        qkv = h @ p["w_qkv"].T + p["b_qkv"]
        q = qkv[:, :H * dh].reshape(T, H, dh)
        k = qkv[:, H * dh:2 * H * dh].reshape(T, H, dh)
        v = qkv[:, 2 * H * dh:].reshape(T, H, dh)
        st = dict(p=p, x=xs, cu=cus, sid=sid, mod=mod, n1=n1, h=h, q_raw=q, k_raw=k)
        if qk_norm:
            q, st["rq"] = _rms_heads_fwd(q, p["q_norm_g"], qk_eps)
            k, st["rk"] = _rms_heads_fwd(k, p["k_norm_g"], qk_eps)
        sel = jstream == s
        q_j[sel], k_j[sel], v_j[sel] = q[jrow[sel]], k[jrow[sel]], v[jrow[sel]]
        c["st"].append(st)
    o_j = bo.attention_fwd(q_j, k_j, v_j, jcu, False)
    c.update(jcu=jcu, jstream=jstream, jrow=jrow, q=q_j, k=k_j, v=v_j, o=o_j, qk_norm=qk_norm)
    ys = []
    for s in range(2):
        st = c["st"][s]; p = st["p"]; sid = st["sid"]; mod = st["mod"]
        sh1, sc1, g1, sh2, sc2, g2 = [mod[:, i * d:(i + 1) * d] for i in range(6)]
        T = st["x"].shape[0]
        o = np.zeros((T, H, dh))
        sel = jstream == s
        o[jrow[sel]] = o_j[sel]
        attn = o.reshape(T, H * dh) @ p["w_o"].T + p["b_o"]
        x1 = st["x"] + g1[sid] * attn
        xhat2, n2 = bo.layernorm_fwd(x1, None, None, cfg.norm_eps)
        h2 = xhat2 * (1.0 + sc2[sid]) + sh2[sid]
        up = h2 @ p["w_up"].T + p["b_up"]
        a = bo.gelu(up)
        m = a @ p["w_down"].T + p["b_down"]
        ys.append(x1 + g2[sid] * m)
        st.update(o=o, attn=attn, x1=x1, n2=n2, h2=h2, up=up, a=a, m=m)
    return ys, c


def mmdit_backward(cfg, cache, dy, qk_norm=True):
    """Returns ([dx_text, dx_img], [grads_text, grads_img], dcond)."""
    d, H, dh, F = cfg.hidden, cfg.n_q_heads, cfg.head_dim, cfg.mlp_hidden
    c = cache
    jstream, jrow, jcu = c["jstream"], c["jrow"], c["jcu"]
    Tj = len(jstream)
    do_j = np.zeros((Tj, H, dh))
    part = []
    for s in range(2):
        st = c["st"][s]; p = st["p"]; sid = st["sid"]; mod = st["mod"]; cus = st["cu"]
        sh1, sc1, g1, sh2, sc2, g2 = [mod[:, i * d:(i + 1) * d] for i in range(6)]
        dys = _f64(dy[s]); T = dys.shape[0]
        g = {}
        dmod = np.zeros_like(mod)
        dmod[:, 5 * d:6 * d] = bo._segment_sum(dys * st["m"], cus)
        dm = dys * g2[sid]
        g["w_down"] = dm.T @ st["a"]; g["b_down"] = dm.sum(axis=0)
        dup = (dm @ p["w_down"]) * bo.gelu_grad(st["up"])
        g["w_up"] = dup.T @ st["h2"]; g["b_up"] = dup.sum(axis=0)
        dh2 = dup @ p["w_up"]
        xhat2 = st["n2"][0]
        dmod[:, 4 * d:5 * d] = bo._segment_sum(dh2 * xhat2, cus)
        dmod[:, 3 * d:4 * d] = bo._segment_sum(dh2, cus)
        dxn, _, _ = bo.layernorm_bwd(dh2 * (1.0 + sc2[sid]), None, st["n2"])
        dx1 = dys + dxn
        dmod[:, 2 * d:3 * d] = bo._segment_sum(dx1 * st["attn"], cus)
        dattn = dx1 * g1[sid]
        g["w_o"] = dattn.T @ st["o"].reshape(T, H * dh); g["b_o"] = dattn.sum(axis=0)
        do = (dattn @ p["w_o"]).reshape(T, H, dh)
        sel = jstream == s
        do_j[sel] = do[jrow[sel]]
        part.append(dict(g=g, dmod=dmod, dx1=dx1))
    dq_j, dk_j, dv_j = bo.attention_bwd(do_j, c["q"], c["k"], c["v"], jcu, False)
    dxs, grads = [], []
    dcond = np.zeros_like(c["cond"])
    for s in range(2):
        st = c["st"][s]; p = st["p"]; sid = st["sid"]; mod = st["mod"]; cus = st["cu"]
        sh1, sc1 = mod[:, 0:d], mod[:, d:2 * d]
        g, dmod, dx1 = part[s]["g"], part[s]["dmod"], part[s]["dx1"]
        T = st["x"].shape[0]
        dq = np.zeros((T, H, dh)); dk = np.zeros((T, H, dh)); dv = np.zeros((T, H, dh))
        sel = jstream == s
        dq[jrow[sel]], dk[jrow[sel]], dv[jrow[sel]] = dq_j[sel], dk_j[sel], dv_j[sel]
        if qk_norm:
            dq, g["q_norm_g"] = _rms_heads_bwd(dq, st["q_raw"], p["q_norm_g"], st["rq"])
            dk, g["k_norm_g"] = _rms_heads_bwd(dk, st["k_raw"], p["k_norm_g"], st["rk"])
        dqkv = np.concatenate([dq.reshape(T, H * dh), dk.reshape(T, H * dh), dv.reshape(T, H * dh)], axis=1)
        g["w_qkv"] = dqkv.T @ st["h"]; g["b_qkv"] = dqkv.sum(axis=0)
        dh1 = dqkv @ p["w_qkv"]
        xhat1 = st["n1"][0]
        dmod[:, d:2 * d] = bo._segment_sum(dh1 * xhat1, cus)
        dmod[:, 0:d] = bo._segment_sum(dh1, cus)
        dxn, _, _ = bo.layernorm_bwd(dh1 * (1.0 + sc1[sid]), None, st["n1"])
        dxs.append(dx1 + dxn)
        g["w_ada"] = dmod.T @ bo.silu(c["cond"]); g["b_ada"] = dmod.sum(axis=0)
        dcond += (dmod @ p["w_ada"]) * bo.silu_grad(c["cond"])
        grads.append(g)
    return dxs, grads, dcond
