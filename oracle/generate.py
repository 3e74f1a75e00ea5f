"""Batched rollout: Response <- Actor.generate(Query).  TEST INFRASTRUCTURE ONLY.

Follows Alg. 1 / Alg. 2's generate step with the fixed response length of
Sec. V-A ("Hyperparameters": minimum = maximum generation length): every query
gets exactly R response tokens, no end-of-sequence stop.  The first response
token is drawn from the logits at the last query position; the last drawn token
is not fed back.  Sequences are independent, so the batch is a plain loop.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from .sampling import Sampling, sample
from .transformer import CachedDecoder, forward_full


def generate(w: dict, shape, queries: Sequence[Sequence[int]], resp_len: int, s: Sampling,
             forced: Optional[Sequence[Sequence[int]]] = None, method: str = "cached",
             dtype=torch.float64, rows: Optional[Sequence[int]] = None, keep_logits: bool = True):
    """Roll out `resp_len` tokens for each query.

    queries[b] is the unpadded query of batch row b.  `forced[b][t]`, if given,
    replaces the token drawn at step t as the NEXT step's input (teacher
    forcing); the drawn token and its log-prob are still reported.  `rows`
    restricts the work to some batch rows (their outputs do not depend on the
    others); the random stream still uses the true row index.
    method "cached" uses the KV-cached decoder, "full" recomputes the whole
    sequence at every step.
    Returns dict(tokens [n, R] int64, logprobs [n, R] float64, logits [n, R, V] or None, rows).
    """
    rows = list(range(len(queries))) if rows is None else list(rows)
    toks = torch.zeros(len(rows), resp_len, dtype=torch.long)
    lps = torch.zeros(len(rows), resp_len, dtype=torch.float64)
    all_logits = torch.zeros(len(rows), resp_len, shape.vocab, dtype=torch.float64) if keep_logits else None
    for ri, b in enumerate(rows):
        context: List[int] = [int(x) for x in queries[b]]
        dec = CachedDecoder(w, shape, dtype) if method == "cached" else None
        feed = context
        for t in range(resp_len):
            if method == "cached":
                logits = dec.extend(feed)
            else:
                logits = forward_full(w, shape, context, dtype, logits_at=[len(context) - 1])[0]
            tok, lp, _ = sample(logits, s, b, t)
            toks[ri, t], lps[ri, t] = tok, lp
            if keep_logits:
                all_logits[ri, t] = logits.to(torch.float64)
            nxt = int(forced[b][t]) if forced is not None else tok
            context = context + [nxt]
            feed = [nxt]
    return {"tokens": toks, "logprobs": lps, "logits": all_logits, "rows": rows}


def score(w: dict, shape, query: Sequence[int], response: Sequence[int], dtype=torch.float64) -> torch.Tensor:
    """Raw-model log-probs of `response` given `query` by one teacher-forced full
    forward over query ++ response (the paper's Actor.forward, Alg. 1)."""
    seq = [int(x) for x in query] + [int(x) for x in response]
    n, r = len(query), len(response)
    logits = forward_full(w, shape, seq, dtype, logits_at=list(range(n - 1, n + r - 1)))
    lsm = logits - logits.max(dim=-1, keepdim=True).values
    lsm = lsm - torch.log(torch.exp(lsm).sum(dim=-1, keepdim=True))
    return lsm[torch.arange(r), torch.as_tensor([int(x) for x in response])]
