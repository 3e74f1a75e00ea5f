"""Helpers shared by the GPU parity tests (no method arithmetic: conversions and plumbing)."""
import math

import torch

from oracle import transformer as OT


def need_gpu():
    import pytest
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def bf16_round(t: torch.Tensor) -> torch.Tensor:
    """Values rounded to bf16 (to nearest even) and returned as float64 on the CPU."""
    return t.detach().to("cpu").to(torch.bfloat16).to(torch.float64)


def rope_tables(max_pos: int, head_dim: int, theta: float = 10000.0):
    half = head_dim // 2
    i = torch.arange(half, dtype=torch.float64)
    ang = torch.arange(max_pos, dtype=torch.float64)[:, None] * theta ** (-2.0 * i / head_dim)[None, :]
    return torch.cos(ang).float(), torch.sin(ang).float()


def oracle_attention_rows(q, k, v, scale):
    """q [h], k/v [L, h] float64 -> softmax(q k^T * scale) v using the oracle's softmax."""
    p = OT.softmax_rows((k @ q * scale)[None, :])[0]
    return p @ v
