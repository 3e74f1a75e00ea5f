"""Why the 16-bit path computes in fp16 (with four tensors carried as fp16 pairs) and not in bf16: a float64 forward of
the decoder at the 7B width in which chosen activation tensors are rounded the way a 16-bit kernel would store them.
The rollout's tolerance is max |dlogit| <= 3e-2 against the unrounded forward.  Measured here, 4 layers deep:

  * every activation rounded to bf16 (8 significant bits): the tolerance is exceeded several times over;
  * every activation rounded to fp16 (11 bits): within the tolerance at 4 layers, but with no margin left for the
    8x deeper real stack (the error grows roughly with the square root of the depth);
  * fp16 everywhere, with the QKV-projection input, the rotated queries, the attention probabilities and the
    output-projection input carried as two-term fp16 pairs hi + lo: 0.64 of the fp16 error (those four tensors carry
    60 % of its variance), which is the margin the 32-layer stack needs; taking the pair away from the QKV-projection
    input alone raises the rms error by a third, from the output-projection input alone by a tenth.

  * the same with the low halves of the QKV- and output-projection inputs quantised to 4 bits (e2m1, a power-of-two
    scale per 128 columns) and multiplied with a 4-bit copy of the weights (a scale per row), which is how the prefill
    GEMMs contract them: within a few per cent of the pair form's error - the low half is 2^-11 of the value, so a
    product that is good to 20 % still removes 96 % of the rounding error's variance.

This file has its own forward and rounding helpers: it pins a design decision of the HIP path, not the oracle, and
imports neither."""
import math

import pytest
import torch

from paper_2312_11819_amd import synth

TENSORS = ["y1", "q", "k", "v", "p", "a", "y2", "h", "yf"]   # every tensor a 16-bit kernel writes or feeds to an MFMA
PAIRS = ("y1", "q", "p", "a")                                # the four that travel as fp16 pairs in the HIP path


def _round(x, mode):
    if mode == "exact":
        return x
    if mode == "bf16":
        return x.to(torch.bfloat16).to(x.dtype)
    hi = x.to(torch.float16).to(x.dtype)
    if mode == "fp16":
        return hi
    assert mode == "pair"
    return hi + (x - hi).to(torch.float16).to(x.dtype)


_E2M1 = torch.tensor([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=torch.float64)
_E2M1_EDGES = (0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0)


def _q4(x, group):
    """Nearest e2m1 value after dividing each group of `group` consecutive columns by the smallest power of two that
    brings its largest magnitude to 6 or below."""
    g = x.reshape(-1, group)
    s = torch.exp2(torch.ceil(torch.log2(g.abs().amax(-1, keepdim=True).clamp_min(1e-300) / 6.0)))
    v = (g / s).abs()
    code = sum((v > e).to(torch.int64) for e in _E2M1_EDGES)
    return (torch.sign(g) * _E2M1[code] * s).reshape(x.shape)


def _project(x, W, mode):
    """x W^T with x rounded as `mode` says; "pair4": fp16 high half against W, 4-bit low half against a 4-bit copy of W."""
    if mode != "pair4":
        return _round(x, mode) @ W.T
    hi = x.to(torch.float16).to(x.dtype)
    return hi @ W.T + _q4(x - hi, 128) @ _q4(W, W.shape[1]).T


def _forward(w, shape, toks, modes):
    """Logits of the last 8 positions; modes[name] in {"exact", "bf16", "fp16", "pair"} per rounded tensor."""
    d = torch.float64
    Hq, Hkv, h, F = shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn
    n = len(toks)
    x = w["tok_emb"].to(d)[torch.tensor(toks)]
    inv = shape.rope_theta ** (-2.0 * torch.arange(h // 2, dtype=d) / h)
    ang = torch.arange(n, dtype=d)[:, None] * inv[None, :]
    c, s_ = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]

    def rope(t):
        lo, hi = t[..., : h // 2], t[..., h // 2:]
        return torch.cat([lo * c - hi * s_, hi * c + lo * s_], -1)

    def norm(t):
        return t / torch.sqrt((t * t).mean(-1, keepdim=True) + shape.rms_eps)

    mask = torch.tril(torch.ones(n, n, dtype=torch.bool))
    for lw in w["layers"]:
        qkv = _project(norm(x), lw["wqkv"].to(d), modes["y1"])
        q = _round(rope(qkv[:, : Hq * h].reshape(n, Hq, h)), modes["q"])
        k = _round(rope(qkv[:, Hq * h: (Hq + Hkv) * h].reshape(n, Hkv, h)), modes["k"])
        v = _round(qkv[:, (Hq + Hkv) * h:].reshape(n, Hkv, h), modes["v"])
        k, v = k.repeat_interleave(Hq // Hkv, dim=1), v.repeat_interleave(Hq // Hkv, dim=1)   # grouped KV heads
        sc = (torch.einsum("ihd,jhd->hij", q, k) / math.sqrt(h)).masked_fill(~mask, float("-inf"))
        p = _round(torch.softmax(sc, -1), modes["p"])
        a = torch.einsum("hij,jhd->ihd", p, v).reshape(n, Hq * h)
        x = x + _project(a, lw["wo"].to(d), modes["a"])
        y = _round(norm(x), modes["y2"])
        gu = y @ lw["w_gate_up"].to(d).T
        g, u = gu[:, :F], gu[:, F:]
        x = x + _round(g / (1.0 + torch.exp(-g)) * u, modes["h"]) @ lw["w_down"].to(d).T
    y = _round(norm(x[-8:]), modes["yf"])
    return y @ w["lm_head"].to(d).T


def test_bf16_activations_miss_the_tolerance_fp16_pairs_meet_it():
    # the 7B layer shape (d_model 4096, 32 heads of 128, FFN 11008), 4 layers; a 4096-entry vocabulary keeps the test short
    shape = synth.ModelShape(4, 4096, 32, 32, 128, 11008, 4096)
    w = synth.make_weights(shape, 2, "bf16")
    toks = torch.randint(0, shape.vocab, (64,), generator=torch.Generator().manual_seed(1)).tolist()
    base = _forward(w, shape, toks, {k: "exact" for k in TENSORS})
    err = {}
    for name, modes in (("bf16", {k: "bf16" for k in TENSORS}),
                        ("fp16", {k: "fp16" for k in TENSORS}),
                        ("design", {k: ("pair" if k in PAIRS else "fp16") for k in TENSORS}),
                        ("design, 4-bit low halves", {k: ("pair4" if k in ("y1", "a") else "pair" if k in PAIRS else "fp16") for k in TENSORS}),
                        ("design without the y1 pair", {k: ("pair" if k in PAIRS and k != "y1" else "fp16") for k in TENSORS}),
                        ("design without the a pair", {k: ("pair" if k in PAIRS and k != "a" else "fp16") for k in TENSORS})):
        e = _forward(w, shape, toks, modes) - base
        err[name] = (float(e.abs().max()), float(e.pow(2).mean().sqrt()))
    print("\nmax / rms logit error after 4 layers:", {k: (round(a, 5), round(b, 5)) for k, (a, b) in err.items()})
    assert err["bf16"][0] > 3e-2                        # bf16 activations: beyond the tolerance after 4 of 32 layers
    assert err["fp16"][0] < 3e-2
    assert err["bf16"][1] > 6 * err["fp16"][1]          # 3 fewer significant bits: ~8x the rms error
    assert err["design"][1] < 0.7 * err["fp16"][1]      # the four pair tensors remove more than half of the error variance
    assert err["design, 4-bit low halves"][1] < 1.1 * err["design"][1]   # the prefill form of two of them costs a few per cent
    # neither projection input can go back to a single fp16 value: the QKV input alone gives back a third of the rms
    # error, the output projection's input a tenth - more than the margin the 32-layer stack has
    assert err["design without the y1 pair"][1] > 1.25 * err["design"][1]
    assert err["design without the a pair"][1] > 1.05 * err["design"][1]
    # extrapolated to 32 layers (rms grows ~ sqrt(depth); the maximum over a step's 32000 logits sits ~4.5 sigma out):
    # plain fp16 lands at the tolerance with nothing to spare, the pair design stays inside it - which the full-depth
    # GPU tests confirm on the real stack
    scale = math.sqrt(32 / 4) * 4.5
    assert err["fp16"][1] * scale > 0.9 * 3e-2
    assert err["design"][1] * scale < 0.7 * 3e-2


def test_rounding_noise_grows_with_width_and_depth_beyond_the_tolerance_at_70b_shape():
    """The same experiment at the 70B layer shape (d_model 8192, 64 query / 8 KV heads, FFN 28672), 2 layers: with
    N(0, 0.02^2) matrices a wider layer writes a larger update into the residual stream and amplifies perturbations
    more, so the same fp16-pair design leaves ~1.7x the logit error of the 7B shape at equal depth - and the stack is
    2.5x deeper.  Extrapolated with the square root of the depth (the full-depth GPU runs grow slightly faster), the
    80-layer stack ends near rms 0.011: its maximum over a step's 32000 logits, ~4.4 sigma, is beyond 3e-2 whatever
    the kernels do, short of carrying every activation and the KV cache as pairs.  This is the reason the full-depth
    GPU tests of the 13B and 70B shapes assert the log-prob tolerance and an rms bound, and report the logit maximum
    as an expected failure."""
    def design_rms(shape, seed):
        w = synth.make_weights(shape, seed, "bf16")
        toks = torch.randint(0, shape.vocab, (32,), generator=torch.Generator().manual_seed(1)).tolist()
        base = _forward(w, shape, toks, {k: "exact" for k in TENSORS})
        e = _forward(w, shape, toks, {k: ("pair" if k in PAIRS else "fp16") for k in TENSORS}) - base
        return float(e.pow(2).mean().sqrt()), float(base.std())
    r7, s7 = design_rms(synth.ModelShape(2, 4096, 32, 32, 128, 11008, 2048), 2)
    r70, s70 = design_rms(synth.ModelShape(2, 8192, 64, 8, 128, 28672, 2048), 5)
    print(f"\n2 layers: 7B shape rms {r7:.5f} (logit std {s7:.2f}), 70B shape rms {r70:.5f} (logit std {s70:.2f})")
    assert r70 > 1.4 * r7
    assert r70 * math.sqrt(80 / 2) * 4.4 > 3e-2          # 80 layers, maximum over 32000 logits
    assert r7 * math.sqrt(32 / 2) * 4.5 < 3e-2           # the benchmark's 32-layer stack stays inside
