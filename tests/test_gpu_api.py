"""Behaviour of the boundary beyond the numbers: graph reuse across rollouts, deferred and immediate error reports for
bad token ids, the sampler on rows without a maximum, fp16 saturation, stream-ordered use of the binding's outputs."""
import pytest
import torch

from oracle.generate import generate as oracle_generate
from oracle.sampling import Sampling as OSampling
from paper_2312_11819_amd import synth
from tests.gpu_util import need_gpu
from tests.test_gpu_rollout import BF16_SMALL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    need_gpu()
    from paper_2312_11819_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("dtype,shape", [("bf16", BF16_SMALL), ("fp32", synth.TINY)])
def test_one_graph_serves_rollouts_with_new_seeds_and_buffers(B, dtype, shape):
    """A PPO loop calls generate with a new seed (and, through the binding, freshly allocated outputs) every round: the
    decode graph is recorded once per batch width and replayed; results equal those of a fresh context."""
    w = synth.weights_to(synth.make_weights(shape, 31, dtype), "cuda")
    toks, lens = synth.make_queries(shape.vocab, 5, 3, 30, 32, pad_token=1)
    R = 9
    ctx = B.Context(w, shape, dtype, 8, 48)
    outs = []
    for seed, temp, top_p in ((1, 1.0, 1.0), (2, 0.8, 0.9), (3, 1.3, 0.5)):
        t, lp = ctx.rlhf_gen_generate(toks.cuda(), lens.tolist(), R, B.make_sampling(temp, top_p, seed))   # fresh outputs
        outs.append((t.clone(), lp.clone()))
        assert ctx.rlhf_gen_graph_captures() == 1
    assert not torch.equal(outs[0][0], outs[1][0])                    # the seed did change the rollout
    # greedy too, and a narrower batch (a second graph), then the first width again (no third)
    ctx.rlhf_gen_generate(toks.cuda(), lens.tolist(), R, B.make_sampling(greedy=True))
    assert ctx.rlhf_gen_graph_captures() == 1
    ctx.rlhf_gen_generate(toks[:3].cuda(), lens[:3].tolist(), R, B.make_sampling(greedy=True))
    assert ctx.rlhf_gen_graph_captures() == 2
    t, lp = ctx.rlhf_gen_generate(toks.cuda(), lens.tolist(), R, B.make_sampling(0.8, 0.9, 2))
    assert ctx.rlhf_gen_graph_captures() == 2
    assert torch.equal(t, outs[1][0]) and torch.equal(lp, outs[1][1])
    fresh = B.Context(w, shape, dtype, 8, 48)
    ft, flp = fresh.rlhf_gen_generate(toks.cuda(), lens.tolist(), R, B.make_sampling(1.3, 0.5, 3))
    assert torch.equal(ft, outs[2][0]) and torch.equal(flp, outs[2][1])
    # a weight refresh at the same addresses keeps the graphs
    ctx.rlhf_gen_update_weights(ctx._weights)
    ctx.rlhf_gen_generate(toks.cuda(), lens.tolist(), R, B.make_sampling(1.0, 1.0, 1))
    assert ctx.rlhf_gen_graph_captures() == 2
    ctx.rlhf_gen_destroy(); fresh.rlhf_gen_destroy()


def test_decode_step_reports_a_forced_token_outside_the_vocabulary(B):
    shape = synth.TINY
    w = synth.weights_to(synth.make_weights(shape, 41), "cuda")
    toks, lens = synth.make_queries(shape.vocab, 3, 4, 9, 42)
    sp = B.make_sampling(greedy=True)
    ctx = B.Context(w, shape, "fp32", 4, 32)
    tok, _ = ctx.rlhf_gen_prefill(toks.cuda(), lens.tolist(), sp)
    good = tok.clone()
    ctx.rlhf_gen_decode_step(good)                                     # valid ids: nothing to report
    ctx.synchronize()
    ctx.rlhf_gen_decode_step(good)
    bad = good.clone(); bad[1] = shape.vocab + 7
    ctx.rlhf_gen_decode_step(bad)                                      # cannot be refused without waiting for the device
    ctx.synchronize()
    with pytest.raises(B.RlhfGenError) as e:                           # ... so the next step reports it
        ctx.rlhf_gen_decode_step(good)
    assert e.value.status == B.E_INVALID and "forced token" in e.value.message
    ctx.rlhf_gen_decode_step(good)                                     # reported once, then cleared
    bad[1] = -1
    ctx.rlhf_gen_decode_step(bad)
    with pytest.raises(B.RlhfGenError) as e:                           # get_logits waits for the step and reports as well
        ctx.rlhf_gen_get_logits()
    assert e.value.status == B.E_INVALID
    lg = ctx.rlhf_gen_get_logits()
    assert bool(torch.isfinite(lg).all())
    ctx.rlhf_gen_destroy()


def test_score_rejects_every_bad_token_id_including_the_last_response_token(B):
    shape = synth.TINY
    w = synth.weights_to(synth.make_weights(shape, 43), "cuda")
    toks, lens = synth.make_queries(shape.vocab, 3, 4, 9, 44)
    resp = torch.randint(0, shape.vocab, (3, 5), generator=torch.Generator().manual_seed(45), dtype=torch.int32)
    ctx = B.Context(w, shape, "fp32", 4, 32)
    ok = ctx.rlhf_gen_score(toks.cuda(), lens.tolist(), resp.cuda())
    assert bool(torch.isfinite(ok).all())
    for col in (0, 4):                                                 # a fed token, and the last one (scored, never fed)
        for val in (-3, shape.vocab):
            bad = resp.clone(); bad[2, col] = val
            with pytest.raises(B.RlhfGenError) as e:
                ctx.rlhf_gen_score(toks.cuda(), lens.tolist(), bad.cuda())
            assert e.value.status == B.E_INVALID
    one = resp[:, :1].contiguous()                                     # R = 1: the only response token is the last one
    bad = one.clone(); bad[0, 0] = shape.vocab
    with pytest.raises(B.RlhfGenError):
        ctx.rlhf_gen_score(toks.cuda(), lens.tolist(), bad.cuda())
    assert bool(torch.isfinite(ctx.rlhf_gen_score(toks.cuda(), lens.tolist(), one.cuda())).all())
    ctx.rlhf_gen_destroy()


@pytest.mark.parametrize("V", [512, 32000, 40000])
def test_sampler_returns_a_valid_token_for_rows_without_a_maximum(B, V):
    """Rows of NaNs (and a row with some NaNs) have no arg-max and no nucleus member; the sampler must still hand back
    an id inside the vocabulary in every mode, because that id is fed to the next step's embedding gather."""
    g = torch.Generator().manual_seed(5)
    logits = torch.randn(4, V, generator=g)
    logits[1] = float("nan")
    logits[2, ::3] = float("nan")
    logits = logits.cuda()
    step = torch.zeros(1, dtype=torch.int32, device="cuda")
    for sp in (B.make_sampling(greedy=True), B.make_sampling(1.0, 1.0, 7), B.make_sampling(0.7, 0.5, 8),
               B.make_sampling(0.7, 0.5, 8, logprob_mode=1)):
        tok = torch.full((4,), -99, dtype=torch.int32, device="cuda")
        lp = torch.zeros(4, device="cuda")
        cur = torch.full((4,), -99, dtype=torch.int32, device="cuda")
        assert B.rlhf_gen_op_sample(logits, sp, step, tok, lp, cur) == B.OK
        torch.cuda.synchronize()
        assert int(tok.min()) >= 0 and int(tok.max()) < V and torch.equal(tok, cur)
        assert bool(torch.isfinite(lp[0])) and bool(torch.isfinite(lp[3]))   # ordinary rows are unaffected by their neighbours


def test_fp16_saturation_instead_of_infinity(B):
    """The 16-bit path stores activations as fp16; a value beyond the fp16 range is stored as +-65504, never as
    infinity.  Kernel level: the SwiGLU epilogues and the fp16 store of both GEMM forms.  End to end: a norm gain of
    1e5 drives the FFN input, the gate/up products and the SwiGLU output far past 65504 - logits stay finite."""
    M, K, F = 48, 256, 256
    a = torch.full((M, K), 60.0, device="cuda", dtype=torch.float16)
    w0 = torch.full((2 * F, K), 1.0, device="cuda", dtype=torch.float16)      # gate = up = 60 * 256 = 15360 -> 2.4e8
    w0[F:] *= -1                                                                 # up negative: the product saturates at -65504
    w = torch.empty_like(w0)
    assert B.rlhf_gen_op_tile_weights(w0, w) == B.OK
    for kind in (B.GEMM_TILED, B.GEMM_STREAMING):
        out = torch.zeros(M, F, device="cuda", dtype=torch.float16)
        assert B.rlhf_gen_op_gemm(kind, a, w, out, M, F, K, B.EPI_SWIGLU, 1, 0) == B.OK
        torch.cuda.synchronize()
        assert bool((out == -65504.0).all()), (kind, out.flatten()[:4])
    wp = torch.empty(F, K, device="cuda", dtype=torch.float16)
    assert B.rlhf_gen_op_tile_weights(torch.full((F, K), 8.0, device="cuda", dtype=torch.float16), wp) == B.OK
    out = torch.zeros(M, F, device="cuda", dtype=torch.float16)
    assert B.rlhf_gen_op_gemm(B.GEMM_TILED, a, wp, out, M, F, K, B.EPI_STORE_H16, 1, 0) == B.OK   # 60 * 8 * 256 = 122880
    torch.cuda.synchronize()
    assert bool((out == 65504.0).all())

    shape = BF16_SMALL
    wts = synth.make_weights(shape, 51, "bf16")
    for lw in wts["layers"]:
        lw["ffn_norm"].fill_(1e5)
        lw["attn_norm"].fill_(3e4)
    toks, lens = synth.make_queries(shape.vocab, 4, 5, 40, 52, pad_token=1)
    ctx = B.Context(synth.weights_to(wts, "cuda"), shape, "bf16", 4, 64)
    sp = B.make_sampling(1.0, 0.9, 3)
    tok, lp = ctx.rlhf_gen_prefill(toks.cuda(), lens.tolist(), sp)
    for _ in range(3):
        lg = ctx.rlhf_gen_get_logits()
        assert bool(torch.isfinite(lg).all()) and bool(torch.isfinite(lp).all())
        assert int(tok.min()) >= 0 and int(tok.max()) < shape.vocab
        tok, lp = ctx.rlhf_gen_decode_step()
    gt, glp = ctx.rlhf_gen_generate(toks.cuda(), lens.tolist(), 8, sp)
    assert bool(torch.isfinite(glp).all()) and bool((glp <= 0).all())
    ctx.rlhf_gen_destroy()


def test_outputs_can_be_used_in_stream_order_without_synchronising(B):
    """The step calls enqueue on the context's stream and return; the binding makes the caller's stream wait for that
    work and tells the allocator where the buffers are in use, so reading a result - or dropping it and allocating
    again - needs no explicit synchronisation.  Compared with a run that synchronises after every call."""
    shape = synth.TINY
    wc = synth.make_weights(shape, 61)
    w = synth.weights_to(wc, "cuda")
    toks, lens = synth.make_queries(shape.vocab, 4, 4, 12, 62)
    sp = B.make_sampling(greedy=True)

    def run(sync):
        ctx = B.Context(w, shape, "fp32", 4, 40)
        seen = []
        tok, lp = ctx.rlhf_gen_prefill(toks.cuda(), lens.tolist(), sp)
        for _ in range(12):
            if sync:
                ctx.synchronize()
            seen.append(tok.clone())                                   # reads on the caller's stream
            forced = tok + 0                                           # a temporary that dies right after the call
            tok, lp = ctx.rlhf_gen_decode_step(forced)
            del forced
            junk = torch.full((4,), -1, dtype=torch.int32, device="cuda")   # may reuse whatever the allocator thinks is free
            del junk
        ctx.synchronize()
        seen.append(tok.clone())
        ctx.rlhf_gen_destroy()
        return torch.stack(seen, 1)

    a, b = run(True), run(False)
    assert torch.equal(a, b)
    ref = oracle_generate(wc, shape, [toks[i, : lens[i]].tolist() for i in range(4)], 13, OSampling(greedy=True))
    top2 = ref["logits"].topk(2, dim=-1).values
    if float((top2[..., 0] - top2[..., 1]).min()) > 2e-4:
        assert torch.equal(a.cpu().long(), ref["tokens"])
