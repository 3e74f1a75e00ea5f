"""Micro-batched rollout: same result as the oracle's Actor.generate and as the whole-batch rollout, completion events
in order, and a consumer on a second stream that picks finished micro-batches up while the next ones are generated."""
import pytest
import torch

from oracle.generate import generate as oracle_generate
from oracle.sampling import Sampling as OSampling
from paper_2312_11819_amd import synth
from tests.gpu_util import need_gpu
from tests.test_gpu_rollout import BF16_SMALL_GQA

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    need_gpu()
    from paper_2312_11819_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("dtype,shape,batch,mb", [("bf16", BF16_SMALL_GQA, 11, 4), ("bf16", BF16_SMALL_GQA, 40, 17),
                                                  ("fp32", synth.TINY_GQA, 7, 3), ("bf16", BF16_SMALL_GQA, 6, 8)])
def test_stream_equals_whole_batch(B, dtype, shape, batch, mb):
    w = synth.weights_to(synth.make_weights(shape, 71, dtype), "cuda")
    toks, lens = synth.make_queries(shape.vocab, batch, 2, 45, 72, pad_token=1)
    R = 14
    sp = B.make_sampling(temperature=0.9, top_p=0.92, seed=1234)
    whole = B.Context(w, shape, dtype, batch, 64)
    want_t, want_lp = whole.rlhf_gen_generate(toks.cuda(), lens.tolist(), R, sp)
    ctx = B.Context(w, shape, dtype, min(mb, batch), 64)          # sized for one micro-batch only
    side = torch.cuda.Stream()
    host_t = torch.zeros(batch, R, dtype=torch.int32).pin_memory()
    host_lp = torch.zeros(batch, R, dtype=torch.float32).pin_memory()
    seen = []
    out_t = torch.empty(batch, R, dtype=torch.int32, device="cuda")
    out_lp = torch.empty(batch, R, dtype=torch.float32, device="cuda")

    def on_ready(index, row0, rows, event):
        seen.append((index, row0, rows))
        side.wait_event(event)
        with torch.cuda.stream(side):                              # copy-out overlaps the next micro-batch
            host_t[row0:row0 + rows].copy_(out_t[row0:row0 + rows], non_blocking=True)
            host_lp[row0:row0 + rows].copy_(out_lp[row0:row0 + rows], non_blocking=True)

    got_t, got_lp, events = ctx.rlhf_gen_generate_stream(toks.cuda(), lens.tolist(), R, sp, mb, on_ready, out_t, out_lp)
    side.synchronize()
    n_mb = -(-batch // mb)
    assert seen == [(i, i * mb, min(mb, batch - i * mb)) for i in range(n_mb)]
    assert torch.equal(got_t, want_t) and torch.equal(got_lp, want_lp)
    assert torch.equal(host_t, want_t.cpu()) and torch.equal(host_lp, want_lp.cpu())
    assert all(e.query() for e in events)
    for a, b in zip(events, events[1:]):
        assert a.elapsed_time(b) > 0                                # recorded in micro-batch order


def test_stream_fp32_matches_oracle(B):
    """Alg. 1 `Response <- Actor.generate(Query)` by micro-batches of 3 out of 7 rows (a ragged last one), fp32, greedy:
    every token equals the oracle's free-running rollout and every log-prob is within 1e-4."""
    shape = synth.TINY_GQA
    w = synth.make_weights(shape, 177)                                # (seeds 171..178 tried on the oracle: 177 has the widest top-2 gaps)
    synth.randomize_norm_gains(w, 172)
    toks, lens = synth.make_queries(shape.vocab, 7, 2, 30, 173, pad_token=2)
    R = 12
    ref = oracle_generate(w, shape, [toks[b, : lens[b]].tolist() for b in range(7)], R, OSampling(greedy=True))
    top2 = ref["logits"].topk(2, dim=-1).values
    assert float((top2[..., 0] - top2[..., 1]).min()) > 2e-4          # no near-tie for this seed: tokens are decided
    ctx = B.Context(synth.weights_to(w, "cuda"), shape, "fp32", 3, 48)
    got_t, got_lp, _ = ctx.rlhf_gen_generate_stream(toks.cuda(), lens.tolist(), R, B.make_sampling(greedy=True), 3)
    ctx.synchronize()
    assert torch.equal(got_t.cpu().long(), ref["tokens"])
    assert float((got_lp.cpu().double() - ref["logprobs"]).abs().max()) < 1e-4
    # seeded sampling: row b of micro-batch i must draw what row b of the whole batch draws (the oracle's stream for
    # (seed, b, t)); compared up to each row's first draw that sits next to a CDF edge
    from oracle import sampling as OS
    cfgs = dict(temperature=0.9, top_p=0.9, seed=4321)
    osp = OSampling(**cfgs)
    got_t, got_lp, _ = ctx.rlhf_gen_generate_stream(toks.cuda(), lens.tolist(), R, B.make_sampling(**cfgs), 3)
    ctx.synchronize()
    ref = oracle_generate(w, shape, [toks[b, : lens[b]].tolist() for b in range(7)], R, osp)
    compared = 0
    for b in range(7):
        for t in range(R):
            _, _, info = OS.sample(ref["logits"][b, t], osp, b, t)
            if OS.cdf_margin(info, int(ref["tokens"][b, t])) < 1e-4:
                break
            assert int(got_t[b, t]) == int(ref["tokens"][b, t]), (b, t)
            assert abs(float(got_lp[b, t]) - float(ref["logprobs"][b, t])) < 1e-4, (b, t)
            compared += 1
    assert compared >= 7 * R // 2
    ctx.rlhf_gen_destroy()


def test_stream_16bit_matches_oracle(B):
    """The 16-bit path through rlhf_gen_generate_stream against the oracle: free-running greedy, every row compared up
    to its first near-tie (top-2 gap below twice the logit tolerance), log-probs within 2e-2."""
    shape = BF16_SMALL_GQA
    w = synth.make_weights(shape, 181, "bf16")
    synth.randomize_norm_gains(w, 182)
    toks, lens = synth.make_queries(shape.vocab, 10, 3, 40, 183, pad_token=1)
    R = 10
    ref = oracle_generate(w, shape, [toks[b, : lens[b]].tolist() for b in range(10)], R, OSampling(greedy=True))
    ctx = B.Context(synth.weights_to(w, "cuda"), shape, "bf16", 4, 64)
    got_t, got_lp, _ = ctx.rlhf_gen_generate_stream(toks.cuda(), lens.tolist(), R, B.make_sampling(greedy=True), 4)
    ctx.synchronize()
    compared = 0
    for b in range(10):
        for t in range(R):
            top2 = ref["logits"][b, t].topk(2).values
            if float(top2[0] - top2[1]) < 6e-2:
                break
            assert int(got_t[b, t]) == int(ref["tokens"][b, t]), (b, t)
            assert abs(float(got_lp[b, t]) - float(ref["logprobs"][b, t])) <= 2e-2, (b, t)
            compared += 1
    assert compared >= 30, compared
    ctx.rlhf_gen_destroy()


def test_stream_errors(B):
    shape = synth.TINY
    w = synth.weights_to(synth.make_weights(shape, 73), "cuda")
    toks, lens = synth.make_queries(shape.vocab, 6, 2, 9, 74)
    sp = B.make_sampling(greedy=True)
    ctx = B.Context(w, shape, "fp32", 2, 32)
    for mb in (0, 3):                                               # not positive / larger than max_batch
        with pytest.raises(B.RlhfGenError) as e:
            ctx.rlhf_gen_generate_stream(toks.cuda(), lens.tolist(), 4, sp, mb)
        assert e.value.status == B.E_INVALID
    # a failure inside a later micro-batch is reported and the earlier ones were delivered
    bad = toks.clone(); bad[5, 0] = shape.vocab
    seen = []
    with pytest.raises(B.RlhfGenError) as e:
        ctx.rlhf_gen_generate_stream(bad.cuda(), lens.tolist(), 4, sp, 2, lambda i, r0, n, ev: seen.append(i))
    assert e.value.status == B.E_INVALID and seen == [0, 1]
    # a callback that raises does not corrupt the context
    def boom(i, r0, n, ev):
        raise ValueError("consumer failed")
    with pytest.raises(ValueError):
        ctx.rlhf_gen_generate_stream(toks.cuda(), lens.tolist(), 4, sp, 2, boom)
    t, lp, _ = ctx.rlhf_gen_generate_stream(toks.cuda(), lens.tolist(), 4, sp, 2)
    assert int(t.min()) >= 0
