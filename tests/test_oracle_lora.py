"""Pins of the adapter-merging oracle (CPU)."""
import torch

from oracle import lora as OL


def test_fold_is_the_sum_of_the_two_paths():
    """(W + s B A) x = W x + s B (A x): the merged matrix applied to a vector equals the dense path plus the
    adapter path evaluated separately with scalar loops, so a transposed factor, a dropped scale or a wrong
    contraction index fails."""
    g = torch.Generator().manual_seed(3)
    out_f, in_f, r, s = 5, 7, 3, 0.37
    W = torch.randn(out_f, in_f, generator=g, dtype=torch.float64)
    A = torch.randn(r, in_f, generator=g, dtype=torch.float64)
    B = torch.randn(out_f, r, generator=g, dtype=torch.float64)
    x = torch.randn(in_f, generator=g, dtype=torch.float64)
    want = []
    for o in range(out_f):
        dense = sum(float(W[o, i]) * float(x[i]) for i in range(in_f))
        low = 0.0
        for j in range(r):
            ax = sum(float(A[j, i]) * float(x[i]) for i in range(in_f))
            low += float(B[o, j]) * ax
        want.append(dense + s * low)
    got = OL.fold(W, A, B, s) @ x
    assert torch.allclose(got, torch.tensor(want, dtype=torch.float64), rtol=0, atol=1e-12)


def test_fold_special_cases():
    g = torch.Generator().manual_seed(4)
    W = torch.randn(4, 6, generator=g).bfloat16()
    A = torch.randn(2, 6, generator=g).bfloat16()
    B = torch.randn(4, 2, generator=g).bfloat16()
    assert torch.equal(OL.fold(W, A, B, 0.0), W.double())                       # scale 0: unchanged
    assert torch.equal(OL.fold(W, A, torch.zeros_like(B), 2.0), W.double())     # B = 0 (LoRA's initial state)
    # rank-1 outer product written out
    a, b = A[:1], B[:, :1]
    want = W.double() + 1.5 * b.double() * a.double()
    assert torch.equal(OL.fold(W, a, b, 1.5), want)


def test_fold_weights_touches_only_named_matrices():
    g = torch.Generator().manual_seed(5)
    w = {"tok_emb": torch.randn(3, 4, generator=g), "lm_head": torch.randn(3, 4, generator=g), "final_norm": torch.ones(4),
         "layers": [{"wqkv": torch.randn(6, 4, generator=g), "wo": torch.randn(4, 2, generator=g)} for _ in range(2)]}
    lora = {"scale": 2.0, "layers": [{"wqkv": (torch.randn(1, 4, generator=g), torch.randn(6, 1, generator=g))}, {}]}
    f = OL.fold_weights(w, lora)
    assert f["layers"][0]["wo"] is w["layers"][0]["wo"] and f["layers"][1]["wqkv"] is w["layers"][1]["wqkv"]
    assert f["lm_head"] is w["lm_head"]
    assert not torch.equal(f["layers"][0]["wqkv"], w["layers"][0]["wqkv"].double())
