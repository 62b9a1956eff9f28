"""Pins for the mixture-of-experts FFN of the block oracle (CPU only): reductions to the
dense SwiGLU block, brute force over all experts, routing invariants, expert permutation,
and a torch float64 autograd composition of library routines (softmax, topk)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

from oracle import block_oracle as bo
from paper_2605_25451_amd import synth

TINY = dict(hidden=16, n_q_heads=4, n_kv_heads=2, head_dim=4, mlp_hidden=12, dtype=synth.DTYPE_FP32)


def moe_case(E=4, k=2, seed=20, lens=(6, 5), router_std=0.6):
    cfg = synth.scaled(synth.decoder_moe(), **TINY, n_experts=E, top_k=k, router_std=router_std)
    return synth.make_case(cfg, list(lens), seed, weight_std=0.3)


def margins(case):
    """Smallest gap between the k-th and (k+1)-th router probability over the tokens."""
    _, cache = bo.block_forward(case.cfg, case.params, case.x, case.cu_seqlens)
    p = np.sort(cache["moe"]["probs"], axis=1)[:, ::-1]
    k = case.cfg.top_k
    return float((p[:, k - 1] - p[:, k]).min()) if k < p.shape[1] else 1.0


def test_fd_case_has_a_routing_margin():
    # the finite-difference pin in test_oracle_block.py perturbs by 1e-6: no choice may flip
    from tests.test_oracle_block import CASES
    assert margins(CASES["moe"]) > 1e-4


def test_one_expert_is_the_dense_swiglu_block():
    moe = moe_case(E=1, k=1, seed=21)
    dense_cfg = synth.scaled(moe.cfg, n_experts=0, top_k=0)
    dense_params = {n: v for n, v in moe.params.items() if n != "w_router"}
    y0, c0 = bo.block_forward(dense_cfg, dense_params, moe.x, moe.cu_seqlens)
    y1, c1 = bo.block_forward(moe.cfg, moe.params, moe.x, moe.cu_seqlens)
    assert np.allclose(y0, y1, rtol=1e-13, atol=1e-13)
    dx0, g0, _ = bo.block_backward(dense_cfg, dense_params, c0, moe.dy)
    dx1, g1, _ = bo.block_backward(moe.cfg, moe.params, c1, moe.dy)
    assert np.allclose(dx0, dx1, rtol=1e-12, atol=1e-13)
    for n in g0:
        assert np.allclose(g0[n], g1[n], rtol=1e-12, atol=1e-13), n
    assert np.abs(g1["w_router"]).max() < 1e-14          # a single gate is the constant 1


def test_all_experts_active_is_the_probability_weighted_sum():
    case = moe_case(E=3, k=3, seed=22)
    cfg, p = case.cfg, {n: v.astype(np.float64) for n, v in case.params.items()}
    rng = np.random.default_rng(0)
    h = rng.standard_normal((7, cfg.hidden))
    out, mc = bo.moe_ffn_fwd(h, p, 3, 3, cfg.mlp_hidden)
    F, d = cfg.mlp_hidden, cfg.hidden
    ref = np.zeros_like(h)
    for t in range(h.shape[0]):
        logits = [sum(p["w_router"][e, c] * h[t, c] for c in range(d)) for e in range(3)]
        mx = max(logits)
        ex = [np.exp(v - mx) for v in logits]
        probs = [v / sum(ex) for v in ex]
        for e in range(3):
            wu = p["w_up"][e * 2 * F:(e + 1) * 2 * F]
            wd = p["w_down"][e * d:(e + 1) * d]
            up = wu @ h[t]
            a = up[:F] / (1.0 + np.exp(-up[:F])) * up[F:]
            ref[t] += probs[e] * (wd @ a)
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)
    assert np.allclose(np.sort(mc["gate"], axis=1), np.sort(mc["probs"], axis=1), rtol=1e-13)


def test_routing_invariants_and_tie_rule():
    logits = np.array([[0.1, 2.0, 2.0, -1.0, 0.5], [3.0, 3.0, 3.0, 3.0, 3.0], [-1.0, -2.0, 0.0, 5.0, 4.0]])
    idx, gate, probs = bo.moe_route(logits, 2)
    assert idx.tolist() == [[1, 2], [0, 1], [3, 4]]                 # ties go to the lower index
    assert np.allclose(gate.sum(axis=1), 1.0, atol=1e-15)
    assert np.allclose(probs.sum(axis=1), 1.0, atol=1e-15)
    assert np.allclose(gate[1], [0.5, 0.5])
    assert np.allclose(gate[2], np.exp([5.0, 4.0]) / np.exp([5.0, 4.0]).sum())
    # adding a constant to a row of logits changes nothing
    idx2, gate2, _ = bo.moe_route(logits + 7.0, 2)
    assert np.array_equal(idx, idx2) and np.allclose(gate, gate2, rtol=1e-13)


def test_permuting_experts_permutes_their_gradients_only():
    case = moe_case(E=4, k=2, seed=23)
    cfg = case.cfg
    assert margins(case) > 1e-6
    F, d, E = cfg.mlp_hidden, cfg.hidden, 4
    perm = np.array([2, 0, 3, 1])
    p2 = dict(case.params)
    p2["w_router"] = case.params["w_router"][perm]
    p2["w_up"] = case.params["w_up"].reshape(E, 2 * F, d)[perm].reshape(E * 2 * F, d)
    p2["w_down"] = case.params["w_down"].reshape(E, d, F)[perm].reshape(E * d, F)
    y1, c1 = bo.block_forward(cfg, case.params, case.x, case.cu_seqlens)
    y2, c2 = bo.block_forward(cfg, p2, case.x, case.cu_seqlens)
    assert np.allclose(y1, y2, rtol=1e-12, atol=1e-13)
    dx1, g1, _ = bo.block_backward(cfg, case.params, c1, case.dy)
    dx2, g2, _ = bo.block_backward(cfg, p2, c2, case.dy)
    assert np.allclose(dx1, dx2, rtol=1e-11, atol=1e-13)
    assert np.allclose(g1["w_router"][perm], g2["w_router"], rtol=1e-11, atol=1e-13)
    assert np.allclose(g1["w_up"].reshape(E, 2 * F, d)[perm], g2["w_up"].reshape(E, 2 * F, d), rtol=1e-11, atol=1e-13)
    assert np.allclose(g1["w_down"].reshape(E, d, F)[perm], g2["w_down"].reshape(E, d, F), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("E,k", [(4, 2), (6, 3), (5, 1)])
def test_ffn_matches_torch_autograd(E, k):
    case = moe_case(E=E, k=k, seed=24 + E)
    cfg = case.cfg
    F, d = cfg.mlp_hidden, cfg.hidden
    p = {n: v.astype(np.float64) for n, v in case.params.items()}
    rng = np.random.default_rng(E)
    h = rng.standard_normal((9, d))
    dm = rng.standard_normal((9, d))
    out, mc = bo.moe_ffn_fwd(h, p, E, k, F)
    dh, g = bo.moe_ffn_bwd(dm, h, p, mc, E, k, F)

    th = torch.tensor(h, requires_grad=True)
    wr = torch.tensor(p["w_router"], requires_grad=True)
    wu = torch.tensor(p["w_up"].reshape(E, 2 * F, d), requires_grad=True)
    wd = torch.tensor(p["w_down"].reshape(E, d, F), requires_grad=True)
    probs = Fn.softmax(th @ wr.T, dim=1)
    sel, idx = torch.topk(probs, k, dim=1)
    gate = sel / sel.sum(dim=1, keepdim=True)
    tout = torch.zeros_like(th)
    for j in range(k):
        up = torch.einsum("tfd,td->tf", wu[idx[:, j]], th)
        a = Fn.silu(up[:, :F]) * up[:, F:]
        tout = tout + gate[:, j:j + 1] * torch.einsum("tdf,tf->td", wd[idx[:, j]], a)
    (tout * torch.tensor(dm)).sum().backward()
    assert np.allclose(out, tout.detach().numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(dh, th.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(g["w_router"], wr.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(g["w_up"], wu.grad.numpy().reshape(E * 2 * F, d), rtol=1e-10, atol=1e-12)
    assert np.allclose(g["w_down"], wd.grad.numpy().reshape(E * d, F), rtol=1e-10, atol=1e-12)


# ---- a given expert choice (the integer decision handed in) --------------------------------

def test_given_own_choice_reproduces_the_result_bit_for_bit():
    case = moe_case(E=6, k=3, seed=40)
    y0, dx0, g0, _ = bo.block_fwd_bwd(case.cfg, case.params, case.x, case.cu_seqlens, case.dy)
    _, cache = bo.block_forward(case.cfg, case.params, case.x, case.cu_seqlens)
    y1, dx1, g1, _ = bo.block_fwd_bwd(case.cfg, case.params, case.x, case.cu_seqlens, case.dy,
                                      expert_choice=cache["moe"]["idx"])
    assert np.array_equal(y0, y1) and np.array_equal(dx0, dx1)
    for n in g0:
        assert np.array_equal(g0[n], g1[n]), n


def test_order_of_a_given_choice_does_not_matter():
    case = moe_case(E=6, k=3, seed=41)
    _, cache = bo.block_forward(case.cfg, case.params, case.x, case.cu_seqlens)
    idx = cache["moe"]["idx"]
    y0, dx0, g0, _ = bo.block_fwd_bwd(case.cfg, case.params, case.x, case.cu_seqlens, case.dy, expert_choice=idx)
    y1, dx1, g1, _ = bo.block_fwd_bwd(case.cfg, case.params, case.x, case.cu_seqlens, case.dy,
                                      expert_choice=idx[:, ::-1])
    assert np.allclose(y0, y1, rtol=1e-13, atol=1e-14) and np.allclose(dx0, dx1, rtol=1e-12, atol=1e-14)
    for n in g0:
        assert np.allclose(g0[n], g1[n], rtol=1e-12, atol=1e-14), n


@pytest.mark.parametrize("E,k", [(5, 2), (6, 3)])
def test_given_choice_matches_torch_autograd_with_that_choice(E, k):
    """A choice that is NOT the top-k one: gates are the chosen probabilities renormalised, and the
    gradients are those of that fixed selection (torch gathers with the same indices)."""
    case = moe_case(E=E, k=k, seed=50 + E)
    cfg = case.cfg
    F, d = cfg.mlp_hidden, cfg.hidden
    p = {n: v.astype(np.float64) for n, v in case.params.items()}
    rng = np.random.default_rng(E + 100)
    T = 8
    h = rng.standard_normal((T, d))
    dm = rng.standard_normal((T, d))
    choice = np.stack([rng.permutation(E)[:k] for _ in range(T)])
    own = bo.moe_route(h @ p["w_router"].T, k)[0]
    assert any(set(a) != set(b) for a, b in zip(choice.tolist(), own.tolist()))
    out, mc = bo.moe_ffn_fwd(h, p, E, k, F, expert_choice=choice)
    dh, g = bo.moe_ffn_bwd(dm, h, p, mc, E, k, F)

    th = torch.tensor(h, requires_grad=True)
    wr = torch.tensor(p["w_router"], requires_grad=True)
    wu = torch.tensor(p["w_up"].reshape(E, 2 * F, d), requires_grad=True)
    wd = torch.tensor(p["w_down"].reshape(E, d, F), requires_grad=True)
    probs = Fn.softmax(th @ wr.T, dim=1)
    idx = torch.tensor(choice)
    sel = torch.gather(probs, 1, idx)
    gate = sel / sel.sum(dim=1, keepdim=True)
    tout = torch.zeros_like(th)
    for j in range(k):
        up = torch.einsum("tfd,td->tf", wu[idx[:, j]], th)
        a = Fn.silu(up[:, :F]) * up[:, F:]
        tout = tout + gate[:, j:j + 1] * torch.einsum("tdf,tf->td", wd[idx[:, j]], a)
    (tout * torch.tensor(dm)).sum().backward()
    assert np.allclose(out, tout.detach().numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(dh, th.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(g["w_router"], wr.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(g["w_up"], wu.grad.numpy().reshape(E * 2 * F, d), rtol=1e-10, atol=1e-12)
    assert np.allclose(g["w_down"], wd.grad.numpy().reshape(E * d, F), rtol=1e-10, atol=1e-12)
