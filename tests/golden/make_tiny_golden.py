"""Writes tests/golden/tiny_greedy.json: the oracle's rollout of the tiny fp32 workload (4 queries of 16 tokens,
16 greedy response tokens, weights seed 1234, tokens seed 1).  Calls only oracle/ and the seeded input generators.
Run from the repository root: python tests/golden/make_tiny_golden.py"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle.generate import generate  # noqa: E402
from oracle.sampling import Sampling  # noqa: E402
from paper_2312_11819_amd import synth  # noqa: E402

wl = synth.WORKLOADS["tiny"]
w = synth.make_weights(wl.shape, wl.weight_seed)
toks, lens = synth.workload_queries(wl)
qs = [toks[b, : lens[b]].tolist() for b in range(wl.batch)]
out = generate(w, wl.shape, qs, wl.resp_len, Sampling(greedy=True), keep_logits=False)
doc = {"source": "oracle/generate.py, float64, written by tests/golden/make_tiny_golden.py",
       "workload": "tiny", "tokens": out["tokens"].tolist(),
       "logprobs": [[round(v, 12) for v in row] for row in out["logprobs"].tolist()]}
with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_greedy.json"), "w") as f:
    json.dump(doc, f, indent=1)
print("wrote tiny_greedy.json")
