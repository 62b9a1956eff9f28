"""Pins for the two-stream adaLN block oracle (CPU only): finite differences, reduction to the
single-stream adaLN block, joint attention against a brute-force loop, stream exchange."""
import numpy as np
import pytest

from oracle import block_oracle as bo
from oracle import mmdit_oracle as mo
from paper_2605_25451_amd import synth

TINY = dict(hidden=16, n_q_heads=4, n_kv_heads=4, head_dim=4, mlp_hidden=24, dtype=synth.DTYPE_FP32)


def tiny(text_lens=(3, 2), image_lens=(4, 5), seed=30, qk_norm=1):
    cfg = synth.scaled(synth.dit_block(), **TINY)
    return synth.make_two_stream_case(cfg, list(text_lens), list(image_lens), seed, qk_norm, weight_std=0.3)


def fwd(case, x=None, params=None, cond=None):
    return mo.mmdit_forward(case.cfg, case.params if params is None else params,
                            case.x if x is None else x, case.cu,
                            case.cond if cond is None else cond, bool(case.qk_norm))


@pytest.mark.parametrize("qk_norm", [1, 0])
def test_backward_matches_central_differences(qk_norm):
    case = tiny(qk_norm=qk_norm)
    G = [g.astype(np.float64) for g in case.dy]
    ys, cache = fwd(case)
    dxs, grads, dcond = mo.mmdit_backward(case.cfg, cache, G, bool(qk_norm))
    eps = 1e-6

    def loss(**kw):
        y, _ = fwd(case, **kw)
        return float((y[0] * G[0]).sum() + (y[1] * G[1]).sum())

    def check(analytic, make):
        flat = analytic.reshape(-1)
        num = np.zeros_like(flat)
        for i in range(flat.size):
            num[i] = (loss(**make(i, +eps)) - loss(**make(i, -eps))) / (2 * eps)
        assert np.abs(num - flat).max() <= 1e-6 * max(1.0, np.abs(flat).max()), np.abs(num - flat).max()

    for s in range(2):
        def mk_x(i, e, s=s):
            x = [a.astype(np.float64).copy() for a in case.x]
            x[s].reshape(-1)[i] += e
            return {"x": x}
        check(dxs[s], mk_x)
        for name in grads[s]:
            if not qk_norm and name in ("q_norm_g", "k_norm_g"):
                continue
            def mk_p(i, e, s=s, name=name):
                ps = [dict(p) for p in case.params]
                a = ps[s][name].astype(np.float64).copy()
                a.reshape(-1)[i] += e
                ps[s][name] = a
                return {"params": ps}
            check(grads[s][name], mk_p)

    def mk_c(i, e):
        c = case.cond.astype(np.float64).copy()
        c.reshape(-1)[i] += e
        return {"cond": c}
    check(dcond, mk_c)


def test_empty_text_stream_without_qk_norm_is_the_single_stream_adaln_block():
    case = tiny(text_lens=(0, 0, 0), image_lens=(4, 3, 5), seed=31, qk_norm=0)
    ys, cache = fwd(case)
    dxs, grads, dcond = mo.mmdit_backward(case.cfg, cache, case.dy, False)
    p = {n: v for n, v in case.params[1].items() if n not in ("q_norm_g", "k_norm_g")}
    y, c1 = bo.block_forward(case.cfg, p, case.x[1], case.cu[1], case.cond)
    dx, g, dc = bo.block_backward(case.cfg, p, c1, case.dy[1])
    assert ys[0].shape == (0, case.cfg.hidden)
    assert np.allclose(ys[1], y, rtol=1e-12, atol=1e-13)
    assert np.allclose(dxs[1], dx, rtol=1e-11, atol=1e-13)
    for n in g:
        assert np.allclose(grads[1][n], g[n], rtol=1e-11, atol=1e-13), n
    # the text stream's conditioning path sees no token: its share of dcond comes from the image stream only
    assert np.allclose(dcond, dc, rtol=1e-11, atol=1e-13)


def test_joint_attention_matches_brute_force():
    case = tiny(text_lens=(2, 3), image_lens=(3, 1), seed=32)
    _, c = fwd(case)
    H, dh = case.cfg.n_q_heads, case.cfg.head_dim
    jcu = c["jcu"]
    assert jcu.tolist() == [0, 5, 9]
    assert c["jstream"].tolist() == [0, 0, 1, 1, 1, 0, 0, 0, 1]
    for s in range(2):
        lo, hi = jcu[s], jcu[s + 1]
        for a in range(H):
            for i in range(lo, hi):
                sc = np.array([sum(c["q"][i, a, e] * c["k"][j, a, e] for e in range(dh)) / np.sqrt(dh)
                               for j in range(lo, hi)])
                w = np.exp(sc - sc.max()); w /= w.sum()
                ref = sum(w[j - lo] * c["v"][j, a] for j in range(lo, hi))
                assert np.allclose(c["o"][i, a], ref, rtol=1e-12, atol=1e-14)


def test_q_and_k_rows_have_unit_rms_before_their_gain():
    case = tiny(seed=33)
    _, c = fwd(case)
    for s in range(2):
        st = c["st"][s]
        qn = st["q_raw"] * st["rq"]
        assert np.allclose((qn * qn).mean(axis=2), 1.0, atol=1e-4)       # eps = 1e-6


def test_exchanging_the_streams_exchanges_the_outputs():
    # attention is bidirectional over the joint sequence, so which stream comes first does not matter
    case = tiny(text_lens=(3, 2), image_lens=(4, 5), seed=34)
    ys, _ = fwd(case)
    sw = synth.TwoStreamCase(case.cfg, case.cu[::-1], case.x[::-1], case.params[::-1], case.dy[::-1],
                             case.cond, case.qk_norm)
    ys2, _ = fwd(sw)
    assert np.allclose(ys[0], ys2[1], rtol=1e-12, atol=1e-13)
    assert np.allclose(ys[1], ys2[0], rtol=1e-12, atol=1e-13)


def test_zero_modulation_weights_give_the_identity():
    case = tiny(seed=35)
    ps = [dict(p) for p in case.params]
    for p in ps:
        p["w_ada"] = np.zeros_like(p["w_ada"]); p["b_ada"] = np.zeros_like(p["b_ada"])
    ys, cache = fwd(case, params=ps)
    assert np.array_equal(ys[0], case.x[0].astype(np.float64))
    assert np.array_equal(ys[1], case.x[1].astype(np.float64))
