"""Pins for the stage oracle (CPU only): the gradients of the total loss match
central finite differences on sampled entries of every parameter group, with and
without a generator, for unit sizes 1 and 2."""
import copy

import numpy as np
import pytest

from oracle import executor_oracle as eo
from paper_2605_25451_amd import synth

f32 = synth.DTYPE_FP32
ENC = synth.scaled(synth.vit_tiny(f32), hidden=16, n_q_heads=2, n_kv_heads=2, head_dim=8, mlp_hidden=24)
LLM = synth.scaled(synth.decoder_7b(f32), hidden=24, n_q_heads=2, n_kv_heads=1, head_dim=12, mlp_hidden=32)
GEN = synth.scaled(synth.dit_block(f32), hidden=16, n_q_heads=2, n_kv_heads=2, head_dim=8, mlp_hidden=24)


def tiny_stage(gen, unit_size, seed):
    return synth.make_stage(ENC, LLM, GEN if gen else None, n_enc=2, n_llm=2, n_gen=2 if gen else 0, M=3,
                            unit_size=unit_size, llm_tokens=40, seed=seed, image_range=(3, 7),
                            text_range=(2, 6), tokens_per_image=4, proj_std=0.3)


@pytest.mark.parametrize("gen,unit_size", [(True, 1), (True, 2), (False, 1), (False, 2)])
def test_stage_gradients_match_finite_differences(gen, unit_size):
    stage = tiny_stage(gen, unit_size, 50 + unit_size)
    for plist in (stage.enc_params, stage.llm_params, stage.gen_params):      # larger weights: visible grads
        for p in plist:
            for k in p:
                if k.startswith("w_"):
                    p[k] = (p[k] * 10).astype(np.float32)
    losses, grads = eo.run_stage(stage)
    assert len(losses) == (len(stage.units) if gen else stage.M)
    rng = np.random.default_rng(0)
    eps = 1e-6

    def fd(get, n=4):
        arr = get(stage)
        out = []
        for _ in range(n):
            idx = tuple(int(rng.integers(0, s)) for s in arr.shape)
            vals = []
            for sgn in (+1, -1):
                st2 = copy.deepcopy(stage)
                a = get(st2).astype(np.float64); a[idx] += sgn * eps
                _set(st2, get, a)
                vals.append(eo.total_loss(st2))
            out.append((idx, (vals[0] - vals[1]) / (2 * eps)))
        return out

    def _set(st, get, a):
        tgt = get(st)
        holder, key = _locate(st, tgt)
        holder[key] = a

    def _locate(st, tgt):
        for name in ("proj_in", "proj_out"):
            if getattr(st, name) is tgt:
                return st.__dict__, name
        for plist in (st.enc_params, st.llm_params, st.gen_params):
            for p in plist:
                for k, v in p.items():
                    if v is tgt:
                        return p, k
        raise AssertionError

    checks = [(lambda s: s.proj_in, grads["proj_in"]),
              (lambda s: s.enc_params[0]["w_qkv"], grads["enc"][0]["w_qkv"]),
              (lambda s: s.enc_params[1]["norm2_g"], grads["enc"][1]["norm2_g"]),
              (lambda s: s.llm_params[0]["w_up"], grads["llm"][0]["w_up"]),
              (lambda s: s.llm_params[1]["w_o"], grads["llm"][1]["w_o"])]
    if gen:
        checks += [(lambda s: s.proj_out, grads["proj_out"]),
                   (lambda s: s.gen_params[0]["w_ada"], grads["gen"][0]["w_ada"]),
                   (lambda s: s.gen_params[1]["w_down"], grads["gen"][1]["w_down"])]
    scale_all = max(float(np.abs(g).max()) for _, g in checks)
    for get, g in checks:
        for idx, num in fd(get):
            assert abs(g[idx] - num) <= 2e-5 * max(abs(num), float(np.abs(g).max()), 1e-3 * scale_all), (idx, g[idx], num)


def test_unit_size_does_not_change_the_result():
    """Same microbatches grouped into units of 1 or of 3: the no-generator loss and
    gradients are sums over microbatches, so they agree."""
    a = tiny_stage(False, 1, 60)
    b = tiny_stage(False, 1, 60)
    # regroup b's microbatches into one unit of three
    lens = [l for m in b.microbatches for l in m.image_lens]
    patches = np.concatenate([u.patches for u in b.units])
    b.units = [synth.UnitCase(synth.cu_from_lengths(lens), patches, None, None)]
    b.unit_size = 3
    la, ga = eo.run_stage(a)
    lb, gb = eo.run_stage(b)
    assert np.allclose(la, lb, rtol=1e-12)
    assert np.allclose(ga["proj_in"], gb["proj_in"], rtol=1e-10, atol=1e-14)
    for x, y in zip(ga["llm"], gb["llm"]):
        for k in x:
            assert np.allclose(x[k], y[k], rtol=1e-10, atol=1e-14)
