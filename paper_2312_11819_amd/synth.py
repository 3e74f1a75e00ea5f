"""Seeded synthetic inputs for the Actor-rollout path: model shapes, weights, queries.

This module is the only code that both the CPU oracle's tests and the HIP path's
callers share.  It holds none of the method's arithmetic: it draws random
numbers and lays them out, nothing else.

The paper trains on a public chat dataset with a fixed 256-token query and a
fixed 256-token response on Llama backbones of several sizes (Sec. V-A,
"LLM Backbones", "Hyperparameters", "Dataset").  Neither the dataset nor trained
weights are available here, so the inputs are stand-ins with the same shape:
uniform random token ids and N(0, 0.02^2) weight matrices with unit norm gains.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional

import torch


@dataclasses.dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def qkv_rows(self) -> int:
        return (self.n_heads + 2 * self.n_kv_heads) * self.head_dim


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    dtype: str              # "fp32" or "bf16": storage type of weights / KV cache
    batch: int
    len_lo: int             # query lengths are uniform integers in [len_lo, len_hi]
    len_hi: int
    resp_len: int
    greedy: bool
    temperature: float
    top_p: float
    weight_seed: int
    token_seed: int
    sample_seed: int


TINY = ModelShape(2, 128, 4, 4, 32, 344, 512)
TINY_GQA = ModelShape(2, 128, 4, 2, 32, 344, 512)
LLAMA_7B = ModelShape(32, 4096, 32, 32, 128, 11008, 32000)
LLAMA_13B = ModelShape(40, 5120, 40, 40, 128, 13824, 32000)
LLAMA_70B_GQA = ModelShape(80, 8192, 64, 8, 128, 28672, 32000)

WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", TINY, "fp32", 4, 16, 16, 16, True, 1.0, 1.0, 1234, 1, 1),
    "7b_b64": Workload("7b_b64", LLAMA_7B, "bf16", 64, 512, 512, 512, False, 1.0, 1.0, 2, 2, 2),
    "13b_ragged": Workload("13b_ragged", LLAMA_13B, "bf16", 32, 64, 1024, 256, False, 0.8, 0.9, 3, 3, 3),
    "7b_b256": Workload("7b_b256", LLAMA_7B, "bf16", 256, 256, 256, 256, True, 1.0, 1.0, 2, 4, 4),
    "70b_gqa": Workload("70b_gqa", LLAMA_70B_GQA, "bf16", 32, 512, 512, 256, False, 1.0, 0.9, 5, 5, 5),
}


def with_layers(shape: ModelShape, n_layers: int) -> ModelShape:
    """The same per-layer shape with a different depth (cheaper oracle runs)."""
    return dataclasses.replace(shape, n_layers=n_layers)


def _normal(gen: torch.Generator, rows: int, cols: int, std: float, dtype: torch.dtype,
            device: torch.device) -> torch.Tensor:
    # Drawn in fp32 in row chunks so that a 90M-element matrix never needs more
    # than ~256 MB of temporary fp32 storage, then rounded once (to nearest even).
    out = torch.empty(rows, cols, dtype=dtype, device=device)
    step = max(1, (64 << 20) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        blk = torch.randn(r1 - r0, cols, generator=gen, device=device, dtype=torch.float32)
        out[r0:r1] = (blk * std).to(dtype)
    return out


def make_weights(shape: ModelShape, seed: int, dtype: str = "fp32",
                 device: str | torch.device = "cpu", std: float = 0.02) -> dict:
    """Random-init Actor weights.  Matrices ~ N(0, std^2); norm gains are 1.

    Layout (row-major, [out_features, in_features]):
      tok_emb [V, d], lm_head [V, d] (untied), final_norm [d],
      per layer: attn_norm [d], wqkv [(Hq + 2 Hkv) h, d] (q rows, then k, then v),
      wo [d, Hq h], ffn_norm [d], w_gate_up [2F, d] (gate rows, then up), w_down [d, F].
    The generator is the device's own seeded generator, so a given (seed, device
    type) pair always yields the same values.
    """
    device = torch.device(device)
    tdt = {"fp32": torch.float32, "bf16": torch.bfloat16}[dtype]
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    s = shape
    w = {
        "tok_emb": _normal(gen, s.vocab, s.d_model, std, tdt, device),
        "lm_head": _normal(gen, s.vocab, s.d_model, std, tdt, device),
        "final_norm": torch.ones(s.d_model, dtype=tdt, device=device),
        "layers": [],
    }
    for _ in range(s.n_layers):
        w["layers"].append({
            "attn_norm": torch.ones(s.d_model, dtype=tdt, device=device),
            "wqkv": _normal(gen, s.qkv_rows, s.d_model, std, tdt, device),
            "wo": _normal(gen, s.d_model, s.n_heads * s.head_dim, std, tdt, device),
            "ffn_norm": torch.ones(s.d_model, dtype=tdt, device=device),
            "w_gate_up": _normal(gen, 2 * s.d_ffn, s.d_model, std, tdt, device),
            "w_down": _normal(gen, s.d_model, s.d_ffn, std, tdt, device),
        })
    return w


def randomize_norm_gains(w: dict, seed: int, spread: float = 0.25) -> None:
    """Replace the unit norm gains by 1 + U(-spread, spread), in place (tests only:
    with unit gains a kernel that ignored the gain vector would go unnoticed)."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)

    def draw(t: torch.Tensor) -> None:
        u = torch.rand(t.numel(), generator=gen, dtype=torch.float32) * 2 - 1
        t.copy_((1.0 + spread * u).to(t.dtype).to(t.device))

    draw(w["final_norm"])
    for lw in w["layers"]:
        draw(lw["attn_norm"])
        draw(lw["ffn_norm"])


def weights_to(w: dict, device: str | torch.device) -> dict:
    """Copy of the weight dictionary on another device (same values, same dtype)."""
    out = {k: v.to(device) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: v.to(device) for k, v in lw.items()} for lw in w["layers"]]
    return out


def make_queries(vocab: int, batch: int, len_lo: int, len_hi: int, seed: int,
                 pad_token: int = 0, lmax: Optional[int] = None):
    """Uniform token ids in [0, vocab), lengths uniform integers in [len_lo, len_hi].

    Returns (tokens [batch, Lmax] int32 right-padded with pad_token, lengths [batch] int32),
    both CPU tensors drawn from a CPU generator (identical on every machine).
    """
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    if len_lo == len_hi:
        lengths = torch.full((batch,), len_lo, dtype=torch.int32)
    else:
        lengths = torch.randint(len_lo, len_hi + 1, (batch,), generator=gen, dtype=torch.int32)
    width = int(lengths.max()) if lmax is None else lmax
    toks = torch.randint(0, vocab, (batch, width), generator=gen, dtype=torch.int32)
    cols = torch.arange(width, dtype=torch.int32)[None, :]
    toks = torch.where(cols < lengths[:, None], toks, torch.full_like(toks, pad_token))
    return toks, lengths


def workload_queries(wl: Workload):
    return make_queries(wl.shape.vocab, wl.batch, wl.len_lo, wl.len_hi, wl.token_seed)


def param_count(shape: ModelShape) -> int:
    s = shape
    per_layer = (s.qkv_rows * s.d_model + s.d_model * s.n_heads * s.head_dim
                 + 2 * s.d_ffn * s.d_model + s.d_model * s.d_ffn + 2 * s.d_model)
    return s.n_layers * per_layer + 2 * s.vocab * s.d_model + s.d_model
