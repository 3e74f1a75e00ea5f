"""Micro-batched rollout: same result as the whole-batch rollout, completion events in order, and a consumer on a
second stream that picks finished micro-batches up while the next ones are generated."""
import pytest
import torch

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
