"""TEST INFRASTRUCTURE ONLY (CPU oracle; imported by tests, the smoke check and the benchmark's CPU baseline).

Folding of low-rank adapters into the dense weights of the Actor (the trainable models carry LoRA adapters of
dimension 4, Sec. V-A "Hyperparameters"; the inference replica receives the merged parameters at each
synchronisation, Sec. IV-A, Disaggregated strategy).  The merged matrix is the definition itself:

    W_eff = W + scale * B A          W [out, in], A [rank, in], B [out, rank]

computed in float64 from the stored values.
"""
from __future__ import annotations

import torch


def fold(W: torch.Tensor, A: torch.Tensor, B: torch.Tensor, scale: float) -> torch.Tensor:
    W64, A64, B64 = (t.detach().to("cpu").to(torch.float64) for t in (W, A, B))
    assert A64.shape[1] == W64.shape[1] and B64.shape[0] == W64.shape[0] and A64.shape[0] == B64.shape[1]
    return W64 + float(scale) * (B64 @ A64)


def fold_weights(w: dict, lora: dict) -> dict:
    """Weights dictionary with every adapter of `lora` merged ({"scale", "layers": [{name: (A, B)}], "lm_head"})."""
    s = float(lora.get("scale", 1.0))
    out = {k: v for k, v in w.items() if k != "layers"}
    if lora.get("lm_head") is not None:
        out["lm_head"] = fold(w["lm_head"], *lora["lm_head"], s)
    out["layers"] = []
    layers = lora.get("layers") or [{} for _ in w["layers"]]
    for lw, la in zip(w["layers"], layers):
        nl = dict(lw)
        for name, pair in la.items():
            if pair is not None:
                nl[name] = fold(lw[name], pair[0], pair[1], s)
        out["layers"].append(nl)
    return out
