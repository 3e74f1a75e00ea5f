"""Pins for the oracle's transformer: invariants, closed forms, brute force, library pieces.

None of these compares the oracle with itself through the same formula: each
either uses a separately written brute force, a closed form, a property that
holds for any correct implementation, or a torch library routine.
"""
import copy
import math

import numpy as np
import pytest
import torch

from oracle import transformer as T
from oracle.generate import generate, score
from oracle.sampling import Sampling
from paper_2312_11819_amd import synth
from tests import naive_ref


@pytest.fixture(scope="module")
def tiny():
    wl = synth.WORKLOADS["tiny"]
    w = synth.make_weights(wl.shape, wl.weight_seed)
    synth.randomize_norm_gains(w, 7)
    return wl.shape, w


@pytest.fixture(scope="module")
def tiny_gqa():
    w = synth.make_weights(synth.TINY_GQA, 99)
    synth.randomize_norm_gains(w, 8)
    return synth.TINY_GQA, w


def _queries(shape, B, lo, hi, seed):
    q, l = synth.make_queries(shape.vocab, B, lo, hi, seed)
    return [q[b, : l[b]].tolist() for b in range(B)]


# P1: cached incremental decode equals full recomputation, every step.
@pytest.mark.parametrize("fix", ["tiny", "tiny_gqa"])
def test_cached_equals_full(fix, request):
    shape, w = request.getfixturevalue(fix)
    qs = _queries(shape, 3, 5, 19, 3)
    a = generate(w, shape, qs, 9, Sampling(greedy=True), method="cached")
    b = generate(w, shape, qs, 9, Sampling(greedy=True), method="full")
    assert torch.equal(a["tokens"], b["tokens"])
    assert (a["logits"] - b["logits"]).abs().max() < 1e-10
    assert (a["logprobs"] - b["logprobs"]).abs().max() < 1e-10


# P3: brute force with scalar loops on a few prefixes.
@pytest.mark.parametrize("fix", ["tiny", "tiny_gqa"])
def test_against_scalar_brute_force(fix, request):
    shape, w = request.getfixturevalue(fix)
    toks = _queries(shape, 1, 7, 7, 11)[0]
    full = T.forward_full(w, shape, toks)
    for n in (1, 4, 7):
        ref = naive_ref.last_logits(w, shape, toks[:n])
        assert np.abs(full[n - 1].numpy() - ref).max() < 1e-10
    dec = T.CachedDecoder(w, shape)
    got = dec.extend(toks[:4])
    assert np.abs(got.numpy() - naive_ref.last_logits(w, shape, toks[:4])).max() < 1e-10
    got = dec.extend(toks[4:5])
    assert np.abs(got.numpy() - naive_ref.last_logits(w, shape, toks[:5])).max() < 1e-10


# P4: closed forms.
def test_zero_lm_head_gives_uniform(tiny):
    shape, w = tiny
    w2 = copy.deepcopy(w)
    w2["lm_head"].zero_()
    out = generate(w2, shape, _queries(shape, 2, 4, 6, 5), 3, Sampling(greedy=True))
    assert (out["tokens"] == 0).all()
    assert (out["logprobs"] + math.log(shape.vocab)).abs().max() < 1e-12
    assert abs(-math.log(512) - (-6.238325)) < 1e-6 and abs(-math.log(32000) - (-10.373491)) < 1e-6


def test_zero_output_projections_make_logits_context_free(tiny):
    shape, w = tiny
    w2 = copy.deepcopy(w)
    for lw in w2["layers"]:
        lw["wo"].zero_()
        lw["w_down"].zero_()
    toks = _queries(shape, 1, 9, 9, 6)[0]
    got = T.forward_full(w2, shape, toks)
    E, g, Wl = w2["tok_emb"].double(), w2["final_norm"].double(), w2["lm_head"].double()
    for i, t in enumerate(toks):
        e = E[t]
        want = (e / torch.sqrt((e * e).mean() + shape.rms_eps) * g) @ Wl.T
        assert (got[i] - want).abs().max() < 1e-12


def test_zero_query_weights_give_mean_of_values(tiny):
    # With W_q = 0 every score is 0, so attention is the plain mean of the visible values.
    shape, w = tiny
    w2 = copy.deepcopy(w)
    w2["layers"] = w2["layers"][:1]
    shape1 = synth.with_layers(shape, 1)
    lw = w2["layers"][0]
    Hq, h = shape.n_heads, shape.head_dim
    lw["wqkv"][: Hq * h].zero_()
    lw["w_down"].zero_()
    toks = _queries(shape, 1, 6, 6, 8)[0]
    got = T.forward_full(w2, shape1, toks)
    E = w2["tok_emb"].double()
    X = E[torch.tensor(toks)]
    Y = X / torch.sqrt((X * X).mean(-1, keepdim=True) + shape.rms_eps) * lw["attn_norm"].double()
    Vv = Y @ lw["wqkv"].double()[(Hq + shape.n_kv_heads) * h:].T        # [n, Hkv*h]; V is not rotated
    for i in range(len(toks)):
        a = Vv[: i + 1].mean(0)
        x1 = X[i] + lw["wo"].double() @ a
        want = (x1 / torch.sqrt((x1 * x1).mean() + shape.rms_eps) * w2["final_norm"].double()) @ w2["lm_head"].double().T
        assert (got[i] - want).abs().max() < 1e-12


# P5: causality, batch independence, pad independence.
def test_causality(tiny):
    shape, w = tiny
    toks = _queries(shape, 1, 12, 12, 9)[0]
    base = T.forward_full(w, shape, toks)
    toks2 = list(toks)
    toks2[7] = (toks2[7] + 1) % shape.vocab
    pert = T.forward_full(w, shape, toks2)
    assert torch.equal(base[:7], pert[:7])
    assert (base[7:] - pert[7:]).abs().max() > 1e-6


def test_batch_independence_and_row_selection(tiny):
    shape, w = tiny
    qs = _queries(shape, 4, 3, 14, 10)
    s = Sampling(temperature=0.9, top_p=0.8, seed=5)
    full = generate(w, shape, qs, 5, s)
    sub = generate(w, shape, qs, 5, s, rows=[2, 0])
    assert torch.equal(sub["tokens"][0], full["tokens"][2]) and torch.equal(sub["tokens"][1], full["tokens"][0])
    assert torch.equal(sub["logprobs"][0], full["logprobs"][2])


# P6: RoPE properties.
def test_rope_properties():
    g = torch.Generator().manual_seed(0)
    x = torch.randn(5, 3, 32, generator=g, dtype=torch.float64)
    pos = torch.tensor([0, 1, 7, 100, 1000])
    r = T.rope(x, pos, 10000.0)
    assert torch.equal(r[0], x[0])                                         # position 0 is the identity
    assert (r.norm(dim=-1) - x.norm(dim=-1)).abs().max() < 1e-12           # rotations preserve length
    # explicit value for one pair: dimension i=3 pairs with 3 + 16
    ang = 7 * 10000.0 ** (-2 * 3 / 32)
    a, b = float(x[2, 1, 3]), float(x[2, 1, 19])
    assert abs(float(r[2, 1, 3]) - (a * math.cos(ang) - b * math.sin(ang))) < 1e-12
    assert abs(float(r[2, 1, 19]) - (b * math.cos(ang) + a * math.sin(ang))) < 1e-12
    # scores depend on relative position only
    q = torch.randn(1, 1, 32, generator=g, dtype=torch.float64)
    k = torch.randn(1, 1, 32, generator=g, dtype=torch.float64)
    s1 = (T.rope(q, torch.tensor([9]), 1e4) * T.rope(k, torch.tensor([4]), 1e4)).sum()
    s2 = (T.rope(q, torch.tensor([59]), 1e4) * T.rope(k, torch.tensor([54]), 1e4)).sum()
    assert abs(float(s1 - s2)) < 1e-12


def test_position_offset_invariance(tiny):
    shape, w = tiny
    toks = _queries(shape, 1, 10, 10, 12)[0]
    a = T.forward_full(w, shape, toks)
    b = T.forward_full(w, shape, toks, position_offset=37)
    assert (a - b).abs().max() < 1e-9


# P7: grouped KV heads equal full multi-head attention with replicated KV weights.
def test_gqa_equals_mha_with_replicated_kv(tiny_gqa):
    shape, w = tiny_gqa
    Hq, Hkv, h = shape.n_heads, shape.n_kv_heads, shape.head_dim
    rep = Hq // Hkv
    mha_shape = synth.ModelShape(shape.n_layers, shape.d_model, Hq, Hq, h, shape.d_ffn, shape.vocab)
    w2 = copy.deepcopy(w)
    for lw in w2["layers"]:
        q = lw["wqkv"][: Hq * h]
        k = lw["wqkv"][Hq * h: (Hq + Hkv) * h].reshape(Hkv, h, -1)
        v = lw["wqkv"][(Hq + Hkv) * h:].reshape(Hkv, h, -1)
        k = k.repeat_interleave(rep, dim=0).reshape(Hq * h, -1)
        v = v.repeat_interleave(rep, dim=0).reshape(Hq * h, -1)
        lw["wqkv"] = torch.cat([q, k, v], dim=0)
    toks = _queries(shape, 1, 9, 9, 13)[0]
    assert (T.forward_full(w, shape, toks) - T.forward_full(w2, mha_shape, toks)).abs().max() < 1e-12


# P8: pieces against torch library routines.
def test_pieces_against_library():
    g = torch.Generator().manual_seed(1)
    z = torch.randn(4, 50, generator=g, dtype=torch.float64) * 3
    assert (T.softmax_rows(z) - torch.softmax(z, -1)).abs().max() < 1e-14
    assert (T.silu(z) - torch.nn.functional.silu(z)).abs().max() < 1e-14
    x = torch.randn(3, 64, generator=g, dtype=torch.float64)
    gain = torch.rand(64, generator=g, dtype=torch.float64)
    want = torch.nn.functional.rms_norm(x, (64,), gain, 1e-5)
    assert (T.rmsnorm(x, gain, 1e-5) - want).abs().max() < 1e-13


def test_attention_block_against_sdpa(tiny_gqa):
    # One layer with the MLP and LM head neutralised: compare the attention output
    # with torch's scaled_dot_product_attention fed with the same q, k, v.
    shape, w = tiny_gqa
    lw = w["layers"][0]
    Hq, Hkv, h = shape.n_heads, shape.n_kv_heads, shape.head_dim
    toks = _queries(shape, 1, 11, 11, 14)[0]
    X = w["tok_emb"].double()[torch.tensor(toks)]
    Y = T.rmsnorm(X, lw["attn_norm"].double(), shape.rms_eps)
    q, k, v = T._split_qkv(Y @ lw["wqkv"].double().T, shape)
    pos = torch.arange(len(toks))
    q, k = T.rope(q, pos, shape.rope_theta), T.rope(k, pos, shape.rope_theta)
    kk = k.repeat_interleave(Hq // Hkv, dim=1).transpose(0, 1)
    vv = v.repeat_interleave(Hq // Hkv, dim=1).transpose(0, 1)
    att = torch.nn.functional.scaled_dot_product_attention(q.transpose(0, 1), kk, vv, is_causal=True)
    att = att.transpose(0, 1).reshape(len(toks), Hq * h)
    x1 = X + att @ lw["wo"].double().T
    w1 = {"tok_emb": w["tok_emb"], "lm_head": torch.eye(shape.d_model, dtype=torch.float64),
          "final_norm": torch.ones(shape.d_model, dtype=torch.float64), "layers": [copy.deepcopy(lw)]}
    w1["layers"][0]["w_down"].zero_()
    s1 = synth.ModelShape(1, shape.d_model, Hq, Hkv, h, shape.d_ffn, shape.d_model)
    got = T.forward_full(w1, s1, toks)
    want = T.rmsnorm(x1, torch.ones(shape.d_model, dtype=torch.float64), shape.rms_eps)
    assert (got - want).abs().max() < 1e-12


# P9: generation log-probs equal a teacher-forced scoring pass (Actor.forward).
def test_generation_logprobs_equal_scoring_pass(tiny):
    shape, w = tiny
    qs = _queries(shape, 2, 6, 10, 15)
    out = generate(w, shape, qs, 7, Sampling(temperature=1.0, top_p=1.0, seed=3))
    for b in range(2):
        sc = score(w, shape, qs[b], out["tokens"][b].tolist())
        assert (sc - out["logprobs"][b]).abs().max() < 1e-10
    assert (out["logprobs"] <= 0).all()


# fp32 mode agrees with fp64 mode to fp32 accuracy.
def test_float32_mode_close(tiny):
    shape, w = tiny
    toks = _queries(shape, 1, 16, 16, 16)[0]
    a = T.forward_full(w, shape, toks)
    b = T.forward_full(w, shape, toks, dtype=torch.float32).double()
    assert (a - b).abs().max() < 2e-5


# P11: determinism.
def test_determinism(tiny):
    shape, w = tiny
    qs = _queries(shape, 2, 5, 8, 17)
    s = Sampling(temperature=0.7, top_p=0.9, seed=11)
    a, b = generate(w, shape, qs, 6, s), generate(w, shape, qs, 6, s)
    assert torch.equal(a["tokens"], b["tokens"]) and torch.equal(a["logprobs"], b["logprobs"])
