"""rlhf_gen_generate_continuous: micro-batches that share one decode loop.  Rows join a micro-batch at a time, decode
steps carry rows at different response indices, finished rows hand their pages back.  Checked against the oracle's
Actor.generate, against the whole-batch rollout (bit for bit), under a KV pool too small for the whole batch, and for the
order and content of the completion callbacks."""
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


def _pages(lens, R):
    return [-(-(int(l) + R - 1) // 16) for l in lens]


def test_continuous_fp32_matches_oracle(B):
    """Free-running greedy rollout of 7 rows admitted 3 at a time every 2 decode steps (so steps carry rows at response
    indices t, t - 2, t - 4): every token equals the oracle's, log-probs within 1e-4; and seeded sampling follows the
    oracle's stream for (seed, row, response index) up to each row's first draw next to a CDF edge."""
    from oracle import sampling as OS
    shape = synth.TINY_GQA
    w = synth.make_weights(shape, 177)
    synth.randomize_norm_gains(w, 172)
    toks, lens = synth.make_queries(shape.vocab, 7, 2, 30, 173, pad_token=2)
    qs = [toks[b, : lens[b]].tolist() for b in range(7)]
    R = 12
    ref = oracle_generate(w, shape, qs, R, OSampling(greedy=True))
    top2 = ref["logits"].topk(2, dim=-1).values
    assert float((top2[..., 0] - top2[..., 1]).min()) > 2e-4
    ctx = B.Context(synth.weights_to(w, "cuda"), shape, "fp32", 7, 48)
    for stagger in (2, 0, 30):
        got_t, got_lp, _ = ctx.rlhf_gen_generate_continuous(toks.cuda(), lens.tolist(), R, B.make_sampling(greedy=True), 3, stagger)
        assert torch.equal(got_t.cpu().long(), ref["tokens"]), stagger
        assert float((got_lp.cpu().double() - ref["logprobs"]).abs().max()) < 1e-4
    cfgs = dict(temperature=0.9, top_p=0.9, seed=4321)
    osp = OSampling(**cfgs)
    ref = oracle_generate(w, shape, qs, R, osp)
    got_t, got_lp, _ = ctx.rlhf_gen_generate_continuous(toks.cuda(), lens.tolist(), R, B.make_sampling(**cfgs), 3, 2)
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


@pytest.mark.parametrize("dtype,shape,batch,mb,stagger,flags", [
    ("bf16", BF16_SMALL_GQA, 11, 4, 3, 0), ("bf16", BF16_SMALL_GQA, 40, 17, 5, 0), ("bf16", BF16_SMALL_GQA, 40, 8, 1, 2),
    ("fp32", synth.TINY_GQA, 7, 3, 0, 0), ("fp32", synth.TINY_GQA, 9, 2, 4, 0), ("bf16", BF16_SMALL_GQA, 6, 8, 2, 0),
    ("bf16", BF16_SMALL_GQA, 20, 5, 100, 0)])
def test_continuous_equals_whole_batch(B, dtype, shape, batch, mb, stagger, flags):
    """Same tokens and log-probs, bit for bit, as rlhf_gen_generate over the whole batch; completion callbacks in
    micro-batch order with the right rows; the decode-step count is the plan's."""
    w = synth.weights_to(synth.make_weights(shape, 71, dtype), "cuda")
    toks, lens = synth.make_queries(shape.vocab, batch, 2, 45, 72, pad_token=1)
    R = 14
    sp = B.make_sampling(temperature=0.9, top_p=0.92, seed=1234)
    whole = B.Context(w, shape, dtype, batch, 64)
    want_t, want_lp = whole.rlhf_gen_generate(toks.cuda(), lens.tolist(), R, sp)
    ctx = B.Context(w, shape, dtype, batch, 64, flags=flags)
    seen = []
    got_t, got_lp, events = ctx.rlhf_gen_generate_continuous(toks.cuda(), lens.tolist(), R, sp, mb, stagger,
                                                             lambda i, r0, n, ev: seen.append((i, r0, n)))
    ctx.synchronize()
    m = min(mb, batch)
    n_mb = -(-batch // m)
    assert seen == [(i, i * m, min(m, batch - i * m)) for i in range(n_mb)]
    assert torch.equal(got_t, want_t) and torch.equal(got_lp, want_lp)
    assert all(e.query() for e in events)
    admit, done, peak = B.rlhf_gen_plan_admission(lens.tolist(), R, mb, stagger, batch * 4)
    assert ctx.rlhf_gen_last_timing()[2] == done[-1] and ctx.rlhf_gen_last_peak_rows() == peak
    # a second rollout on the same context (graphs for the same row windows are reused) gives the same bits
    caps = ctx.rlhf_gen_graph_captures()
    again_t, again_lp, _ = ctx.rlhf_gen_generate_continuous(toks.cuda(), lens.tolist(), R, sp, mb, stagger)
    assert torch.equal(again_t, want_t) and torch.equal(again_lp, want_lp)
    assert ctx.rlhf_gen_graph_captures() == caps
    # and the context still serves the other entry points
    t2, lp2 = ctx.rlhf_gen_generate(toks.cuda(), lens.tolist(), R, sp)
    assert torch.equal(t2, want_t) and torch.equal(lp2, want_lp)
    whole.rlhf_gen_destroy(); ctx.rlhf_gen_destroy()


def test_continuous_under_a_small_kv_pool(B):
    """A pool that holds two micro-batches of four: the third is admitted when the first has finished and returned its
    pages (Sec. IV-C: the batch in flight is what memory allows).  Shuffled page hand-out on top; result unchanged."""
    shape, dtype = BF16_SMALL_GQA, "bf16"
    w = synth.weights_to(synth.make_weights(shape, 75, dtype), "cuda")
    toks, lens = synth.make_queries(shape.vocab, 16, 20, 40, 76, pad_token=1)
    R = 20
    sp = B.make_sampling(temperature=1.0, top_p=0.9, seed=5)
    whole = B.Context(w, shape, dtype, 16, 64)
    want_t, want_lp = whole.rlhf_gen_generate(toks.cuda(), lens.tolist(), R, sp)
    pg = _pages(lens, R)
    per_mb = [sum(pg[i:i + 4]) for i in range(0, 16, 4)]
    pool = max(per_mb[0] + per_mb[1], per_mb[1] + per_mb[2], per_mb[2] + per_mb[3])
    admit, done, peak = B.rlhf_gen_plan_admission(lens.tolist(), R, 4, 3, pool)
    assert peak == 8 and admit[2] == done[0] and admit[3] == done[1]
    for flags in (0, B.FLAG_SHUFFLE_BLOCKS):
        ctx = B.Context(w, shape, dtype, 16, 64, kv_pool_blocks=pool, flags=flags)
        order = []
        got_t, got_lp, events = ctx.rlhf_gen_generate_continuous(toks.cuda(), lens.tolist(), R, sp, 4, 3,
                                                                 lambda i, r0, n, ev: order.append(i))
        ctx.synchronize()
        assert order == [0, 1, 2, 3] and ctx.rlhf_gen_last_peak_rows() == 8
        assert ctx.rlhf_gen_last_timing()[2] == done[-1]
        assert torch.equal(got_t, want_t) and torch.equal(got_lp, want_lp)
        for a, b in zip(events, events[1:]):
            assert a.elapsed_time(b) > 0
        # the whole batch at once does not fit this pool
        with pytest.raises(B.RlhfGenError) as e:
            ctx.rlhf_gen_generate(toks.cuda(), lens.tolist(), R, sp)
        assert e.value.status == B.E_NOMEM
        ctx.rlhf_gen_destroy()
    whole.rlhf_gen_destroy()


def test_continuous_errors(B):
    shape = synth.TINY
    w = synth.weights_to(synth.make_weights(shape, 73), "cuda")
    toks, lens = synth.make_queries(shape.vocab, 6, 2, 9, 74)
    sp = B.make_sampling(greedy=True)
    ctx = B.Context(w, shape, "fp32", 4, 32)
    with pytest.raises(B.RlhfGenError) as e:                         # more rows than state rows
        ctx.rlhf_gen_generate_continuous(toks.cuda(), lens.tolist(), 4, sp, 2, 0)
    assert e.value.status == B.E_INVALID
    ctx = B.Context(w, shape, "fp32", 6, 32, kv_pool_blocks=3)
    with pytest.raises(B.RlhfGenError) as e:                         # a micro-batch of 4 rows needs 4 pages
        ctx.rlhf_gen_generate_continuous(toks.cuda(), lens.tolist(), 4, sp, 4, 0)
    assert e.value.status == B.E_NOMEM
    for mb, st in ((0, 0), (2, -1)):
        with pytest.raises(B.RlhfGenError) as e:
            ctx.rlhf_gen_generate_continuous(toks.cuda(), lens.tolist(), 4, sp, mb, st)
        assert e.value.status == B.E_INVALID
    bad = toks.clone(); bad[5, 0] = shape.vocab                     # a bad id in a later micro-batch: the earlier ones were delivered
    seen = []
    with pytest.raises(B.RlhfGenError) as e:
        ctx.rlhf_gen_generate_continuous(bad.cuda(), lens.tolist(), 4, sp, 2, 50, lambda i, r0, n, ev: seen.append(i))
    assert e.value.status == B.E_INVALID and seen == [0, 1]
    t, lp, _ = ctx.rlhf_gen_generate_continuous(toks.cuda(), lens.tolist(), 4, sp, 2, 1)   # the context is still usable
    assert int(t.min()) >= 0 and int(t.max()) < shape.vocab
    t1, _, _ = ctx.rlhf_gen_generate_continuous(toks.cuda(), lens.tolist(), 1, sp, 2, 1)   # R = 1: prefill only
    assert torch.equal(t1[:, 0], t[:, 0])
