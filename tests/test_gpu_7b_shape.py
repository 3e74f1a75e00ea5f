"""Parity at the benchmark's real per-token shapes (7B width, B = 64, 512-token queries, bf16), in the launch
configuration bench.py times.  The oracle (float64) runs on a few batch rows only - rows are independent - and
every comparison is teacher-forced with the oracle's tokens on those rows.  Full-depth runs (32, 40 and 80 layers) are
in test_gpu_depth.py.

Token parity at V = 32000 with T = 1, top-p = 1 is "unpinned by design": the distribution over random-init logits is
nearly flat, so a draw almost always lies within the logit tolerance of a CDF edge and `_run` can only require that
every differing token is such a case (it reports the fraction).  What pins the tokens at this shape is
test_7b_width_sampler_agrees_with_oracle_on_every_row, which runs the oracle's sampler on the GPU's own logits."""
import time

import pytest
import torch

from oracle import sampling as OS
from oracle.generate import generate as oracle_generate
from oracle.sampling import Sampling as OSampling
from paper_2312_11819_amd import synth
from tests.gpu_util import need_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    need_gpu()
    from paper_2312_11819_amd import binding
    binding.lib()
    return binding


def _run(B, shape, batch, len_lo, len_hi, rows, steps, cfgs, weight_seed, token_seed, flags=0, dtype=torch.float64):
    t0 = time.time()
    w = synth.make_weights(shape, weight_seed, "bf16", "cuda")
    toks, lens = synth.make_queries(shape.vocab, batch, len_lo, len_hi, token_seed)
    w_cpu = synth.weights_to(w, "cpu")
    # widened once here (the values do not change), so that the oracle's per-call conversion of the weights is a no-op
    w_cpu = {**{k: v.to(dtype) for k, v in w_cpu.items() if k != "layers"},
             "layers": [{k: v.to(dtype) for k, v in lw.items()} for lw in w_cpu["layers"]]}
    qs = [toks[b, : lens[b]].tolist() for b in range(batch)]
    osp = OSampling(**cfgs)
    ref = oracle_generate(w_cpu, shape, qs, steps, osp, rows=rows, dtype=dtype)
    t1 = time.time()
    ctx = B.Context(w, shape, "bf16", batch, int(lens.max()) + steps + 1, flags=flags)
    sp = B.make_sampling(**cfgs)
    got_t, got_lp, got_lg = [], [], []
    tok, lp = ctx.rlhf_gen_prefill(toks.cuda(), lens.tolist(), sp)
    for s in range(steps):
        lg = ctx.rlhf_gen_get_logits()
        got_t.append(tok[rows].cpu().long()); got_lp.append(lp[rows].cpu().double()); got_lg.append(lg[rows].cpu().double())
        if s + 1 < steps:
            forced = tok.clone()
            forced[rows] = ref["tokens"][:, s].to(torch.int32).cuda()
            tok, lp = ctx.rlhf_gen_decode_step(forced)
    ctx.synchronize()
    got_t, got_lp, got_lg = torch.stack(got_t, 1), torch.stack(got_lp, 1), torch.stack(got_lg, 1)
    dl = (got_lg - ref["logits"]).abs().max().item()
    rms = (got_lg - ref["logits"]).pow(2).mean().sqrt().item()
    skipped = 0
    dlp = 0.0
    for ri, b in enumerate(rows):
        for t in range(steps):
            want = int(ref["tokens"][ri, t])
            if int(got_t[ri, t]) != want:
                if osp.greedy:
                    top2 = ref["logits"][ri, t].topk(2).values
                    assert float(top2[0] - top2[1]) < 6e-2, (b, t)
                else:
                    _, _, info = OS.sample(ref["logits"][ri, t], osp, b, t)
                    assert OS.cdf_margin(info, want) < 3e-2, (b, t)   # a 3e-2 logit error moves CDF edges by up to ~3e-2
                skipped += 1
                continue
            dlp = max(dlp, abs(float(got_lp[ri, t]) - float(ref["logprobs"][ri, t])))
    print(f"\n[{shape.n_layers} layers, B={batch}] max|dlogit|={dl:.4f} rms={rms:.5f} max|dlogprob|={dlp:.4f} "
          f"skipped={skipped}/{len(rows) * steps} oracle {t1 - t0:.1f}s total {time.time() - t0:.1f}s", flush=True)
    ctx.rlhf_gen_destroy()
    return dl, dlp, skipped / (len(rows) * steps)


def test_7b_width_4_layers_full_batch(B):
    shape = synth.with_layers(synth.LLAMA_7B, 4)
    dl, dlp, frac = _run(B, shape, 64, 512, 512, [0, 31, 63], 6, dict(temperature=1.0, top_p=1.0, seed=2), 2, 2)
    assert dl <= 3e-2 and dlp <= 2e-2 and frac <= 0.34


def test_7b_width_2_layers_ragged_long_context(B):
    # lengths 64..1024 (ragged, pages partly filled), nucleus sampling, shuffled page placement
    shape = synth.with_layers(synth.LLAMA_7B, 2)
    toks, lens = synth.make_queries(shape.vocab, 32, 64, 1024, 3)
    rows = [int(lens.argmax()), int(lens.argmin()), 7]
    dl, dlp, frac = _run(B, shape, 32, 64, 1024, rows, 5, dict(temperature=0.8, top_p=0.9, seed=3), 3, 3, flags=1)
    assert dl <= 3e-2 and dlp <= 2e-2 and frac <= 0.34


def test_7b_width_b256_2_layers(B):
    """The large-batch configuration (256 queries of 256 tokens, greedy, 16-token pages) at the real 7B width: decode
    batches of 129..256 rows take the split-K form of the large-tile GEMM, the separate SwiGLU kernel and the tiled LM
    head, which no other configuration exercises.  Rows 0, 128 and 255; 21 decode steps, so every context crosses a
    page boundary (256 -> 277 tokens)."""
    shape = synth.with_layers(synth.LLAMA_7B, 2)
    dl, dlp, frac = _run(B, shape, 256, 256, 256, [0, 128, 255], 22, dict(greedy=True), 2, 4)
    assert dl <= 3e-2 and dlp <= 2e-2 and frac <= 0.34


def test_70b_width_gqa_2_layers(B):
    shape = synth.with_layers(synth.LLAMA_70B_GQA, 2)
    dl, dlp, frac = _run(B, shape, 32, 200, 520, [0, 17], 4, dict(temperature=1.0, top_p=0.9, seed=5), 5, 5)
    assert dl <= 3e-2 and dlp <= 2e-2 and frac <= 0.5


def test_13b_width_ragged_2_layers(B):
    # d_model 5120: ten 512-column splits in the QKV projection, 108 k-steps in the down projection
    shape = synth.with_layers(synth.LLAMA_13B, 2)
    toks, lens = synth.make_queries(shape.vocab, 32, 64, 700, 6)
    rows = [int(lens.argmax()), int(lens.argmin()), 11]
    dl, dlp, frac = _run(B, shape, 32, 64, 700, rows, 4, dict(temperature=1.0, top_p=0.9, seed=6), 6, 6)
    assert dl <= 3e-2 and dlp <= 2e-2 and frac <= 0.5


def test_7b_width_score_pass(B):
    """rlhf_gen_score at the 7B width (2 layers, 16 sequences of 300 + 40 tokens) against the oracle's score()."""
    from oracle.generate import score as oracle_score
    shape = synth.with_layers(synth.LLAMA_7B, 2)
    w = synth.make_weights(shape, 7, "bf16", "cuda")
    toks, lens = synth.make_queries(shape.vocab, 16, 100, 300, 8)
    g = torch.Generator().manual_seed(9)
    resp = torch.randint(0, shape.vocab, (16, 40), generator=g, dtype=torch.int32)
    ctx = B.Context(w, shape, "bf16", 16, 340)
    got = ctx.rlhf_gen_score(toks.cuda(), lens.tolist(), resp.cuda()).cpu().double()
    w_cpu = synth.weights_to(w, "cpu")
    worst = 0.0
    for b in (0, 15):
        want = oracle_score(w_cpu, shape, toks[b, : lens[b]].tolist(), resp[b].tolist())
        worst = max(worst, float((got[b] - want).abs().max()))
    print(f"\n[score, 2 layers] max|dlogprob|={worst:.4f}", flush=True)
    assert worst <= 2e-2
    ctx.rlhf_gen_destroy()


def test_7b_width_sampler_agrees_with_oracle_on_every_row(B):
    """At the benchmark's batch and vocabulary (2 layers of the 7B width): on the logits the GPU itself produced, the
    oracle's sampler must pick the token the GPU picked for every one of the 64 rows and steps (same stateless random
    numbers, same nucleus), and the returned log-prob must be the log-softmax of those logits at that token.  This
    isolates the sampling path from the model's 16-bit rounding."""
    shape = synth.with_layers(synth.LLAMA_7B, 2)
    w = synth.make_weights(shape, 9, "bf16", "cuda")
    toks, lens = synth.make_queries(shape.vocab, 64, 512, 512, 9)
    for cfgs in (dict(temperature=1.0, top_p=1.0, seed=77), dict(temperature=0.7, top_p=0.8, seed=78)):
        osp = OSampling(**cfgs)
        ctx = B.Context(w, shape, "bf16", 64, 512 + 8)
        tok, lp = ctx.rlhf_gen_prefill(toks.cuda(), lens.tolist(), B.make_sampling(**cfgs))
        mismatches = 0
        for t in range(4):
            lg = ctx.rlhf_gen_get_logits().cpu().double()
            ctx.synchronize()
            ref_lp = torch.log_softmax(lg, dim=-1)
            for b in range(64):
                want, _, info = OS.sample(lg[b], osp, b, t)
                got = int(tok[b])
                if got != want:
                    # only a draw within rounding distance of a CDF edge (fp32 weights on the GPU) may differ
                    assert OS.cdf_margin(info, want) < 1e-5, (b, t, got, want)
                    mismatches += 1
                assert abs(float(lp[b]) - float(ref_lp[b, got])) < 2e-5, (b, t)
            if t < 3:
                tok, lp = ctx.rlhf_gen_decode_step()
        assert mismatches <= 1
        ctx.rlhf_gen_destroy()
