"""Seeded sampler and log-probabilities for the rollout.  TEST INFRASTRUCTURE ONLY.

The paper gives no sampling parameters (Sec. V-A lists lengths only), so the
sampler is the usual temperature / nucleus one, stated step by step:
  z = logits / T; p = softmax(z); nucleus = shortest prefix of the tokens sorted
  by (p descending, index ascending) whose mass reaches top_p (the crossing token
  is kept); p' = p renormalised on the nucleus; with u in [0,1) the token is the
  first nucleus member, in ascending token-index order, whose running p' sum
  exceeds u (the last member if rounding leaves the sum <= u).
Greedy = argmax, lowest index on exact ties.
Log-prob mode 0 is the raw model log-softmax at the chosen token (what a later
`Actor.forward` over query+response would return, Alg. 1); mode 1 is log p'.

The uniform u is a pure function of (seed, row b, response index t): a 64-bit
integer mix followed by taking the top 24 bits, so any implementation using
integer arithmetic reproduces it exactly.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import torch

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_MUL1 = 0xBF58476D1CE4E5B9
_MUL2 = 0x94D049BB133111EB


def mix64(x: int) -> int:
    """The splitmix64 output function applied to x + golden-ratio increment."""
    z = (x + _GOLDEN) & _M64
    z = ((z ^ (z >> 30)) * _MUL1) & _M64
    z = ((z ^ (z >> 27)) * _MUL2) & _M64
    return z ^ (z >> 31)


def uniform(seed: int, b: int, t: int) -> float:
    """u in [0, 1) with 24 random bits for batch row b, response index t."""
    key = (seed ^ ((b * _GOLDEN) & _M64) ^ ((t * _MUL1) & _M64)) & _M64
    return (mix64(key) >> 40) * (2.0 ** -24)


@dataclasses.dataclass
class Sampling:
    temperature: float = 1.0
    top_p: float = 1.0
    seed: int = 0
    greedy: bool = False
    logprob_mode: int = 0


def log_softmax(logits: torch.Tensor) -> torch.Tensor:
    m = logits.max()
    return logits - m - torch.log(torch.exp(logits - m).sum())


def nucleus(p: torch.Tensor, top_p: float) -> torch.Tensor:
    """Boolean membership mask of the top-p nucleus of a probability vector."""
    V = p.numel()
    if top_p >= 1.0:
        return torch.ones(V, dtype=torch.bool)
    order = sorted(range(V), key=lambda i: (-float(p[i]), i))
    keep = torch.zeros(V, dtype=torch.bool)
    mass = 0.0
    for i in order:
        keep[i] = True
        mass += float(p[i])
        if mass >= top_p:
            break
    return keep


def sample(logits: torch.Tensor, s: Sampling, b: int, t: int, u: Optional[float] = None):
    """One row.  Returns (token, logprob, info) with info = dict(p_prime=..., keep=..., u=...)."""
    z64 = logits.to(torch.float64)
    raw_lp = log_softmax(z64)
    if s.greedy:
        best = float(z64.max())
        tok = next(i for i in range(z64.numel()) if float(z64[i]) == best)
        return tok, float(raw_lp[tok]), {"u": None, "keep": None, "p_prime": None}
    p = torch.exp(log_softmax(z64 / s.temperature))
    keep = nucleus(p, s.top_p)
    pp = torch.where(keep, p, torch.zeros_like(p))
    pp = pp / pp.sum()
    if u is None:
        u = uniform(s.seed, b, t)
    run, tok, last = 0.0, None, None
    for i in range(pp.numel()):
        if not bool(keep[i]):
            continue
        last = i
        run += float(pp[i])
        if run > u:
            tok = i
            break
    if tok is None:
        tok = last
    lp = float(raw_lp[tok]) if s.logprob_mode == 0 else math.log(float(pp[tok]))
    return tok, lp, {"u": u, "keep": keep, "p_prime": pp}


def cdf_margin(info: dict, tok: int) -> float:
    """Distance from u to the nearest edge of the chosen token's CDF interval."""
    pp, keep, u = info["p_prime"], info["keep"], info["u"]
    lo = float(pp[:tok][keep[:tok]].sum())
    hi = lo + float(pp[tok])
    return min(u - lo, hi - u)
