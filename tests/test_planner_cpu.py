"""Host logic of rlhf_gen_plan_capacity (no GPU: the capacity is passed in)."""
import pytest

from paper_2312_11819_amd import binding as B
from paper_2312_11819_amd import synth

GiB = 1 << 30


def _plan(shape, dtype, max_seq, cap, frac=1.0, reserved=0, flags=0):
    return B.rlhf_gen_plan_capacity(shape, dtype, max_seq, cap, frac, reserved, flags)


def test_answer_is_the_largest_batch_that_fits():
    shape, max_seq = synth.LLAMA_7B, 1024
    b, n = _plan(shape, "bf16", max_seq, 200 * GiB)
    assert b > 1 and 0 < n <= 200 * GiB
    # exactly its own footprint is enough, one byte less is not
    assert _plan(shape, "bf16", max_seq, n)[0] == b
    assert _plan(shape, "bf16", max_seq, n - 1)[0] < b
    # half a sequence's KV cache more does not admit another sequence, a whole one (plus slack) does
    kv = 32 * 32 * 64 * 8192
    assert _plan(shape, "bf16", max_seq, n + kv // 2)[0] == b
    assert _plan(shape, "bf16", max_seq, n + kv + kv // 50)[0] == b + 1


def test_growth_per_sequence_is_the_kv_cache():
    """Per extra sequence the pool grows by n_layers * n_kv_heads * ceil(max_seq / 16) pages of 8 KiB (K and V of 16
    tokens x 128 dims in 16 bit), plus a little bookkeeping and logits."""
    shape, max_seq = synth.LLAMA_7B, 1024
    n1 = _plan(shape, "bf16", max_seq, 150 * GiB)
    n2 = _plan(shape, "bf16", max_seq, 250 * GiB)
    per_seq = (n2[1] - n1[1]) / (n2[0] - n1[0])
    kv = shape.n_layers * shape.n_kv_heads * ((max_seq + 15) // 16) * 8192
    assert kv == 32 * 32 * 64 * 8192 == 2 * 2 * shape.n_layers * shape.n_kv_heads * shape.head_dim * max_seq
    assert kv <= per_seq <= kv * 1.01
    # grouped-query attention shrinks it by the group size
    g1 = _plan(synth.LLAMA_70B_GQA, "bf16", 640, 200 * GiB, flags=B.FLAG_CONVERT_IN_PLACE)
    g2 = _plan(synth.LLAMA_70B_GQA, "bf16", 640, 280 * GiB, flags=B.FLAG_CONVERT_IN_PLACE)
    s = synth.LLAMA_70B_GQA
    kv70 = s.n_layers * s.n_kv_heads * 40 * 8192
    assert kv70 <= (g2[1] - g1[1]) / (g2[0] - g1[0]) <= kv70 * 1.02


def test_paper_rule_on_one_mi355x():
    """Stop before 95 % of 288 GB with the bf16 model resident: a 7B Actor at 512 + 512 tokens holds a few hundred
    sequences (0.5 GiB of KV each), far beyond the benchmark's batch of 64."""
    cap = 288 * 10 ** 9
    b, n = _plan(synth.LLAMA_7B, "bf16", 1024, cap, 0.95, -1)
    weights = synth.param_count(synth.LLAMA_7B) * 2
    assert n + weights <= 0.95 * cap
    assert 400 <= b <= 520
    assert _plan(synth.LLAMA_7B, "bf16", 1024, cap, 0.5, -1)[0] < b          # monotone in the fraction
    assert _plan(synth.LLAMA_7B, "bf16", 2048, cap, 0.95, -1)[0] < b         # and in the sequence length
    # in-place conversion saves the fp16 working copies: room for more sequences
    assert _plan(synth.LLAMA_7B, "bf16", 1024, cap, 0.95, -1, B.FLAG_CONVERT_IN_PLACE)[0] > b


def test_nothing_fits_and_errors():
    assert _plan(synth.LLAMA_7B, "bf16", 1024, 1 * GiB) == (0, 0)
    for kwargs in (dict(frac=0.0), dict(frac=1.5)):
        with pytest.raises(B.RlhfGenError) as e:
            _plan(synth.TINY, "fp32", 32, GiB, **kwargs)
        assert e.value.status == B.E_INVALID
    bad = synth.ModelShape(2, 256, 2, 2, 64, 384, 512)                        # 16-bit path needs head_dim 128
    with pytest.raises(B.RlhfGenError) as e:
        _plan(bad, "bf16", 64, GiB)
    assert e.value.status == B.E_UNSUPPORTED
    assert _plan(synth.TINY, "fp32", 32, GiB)[0] > 1000


# ---- admission schedule of the continuous-batching rollout (host only) ---------------------------------------------
def _brute_force_schedule(lengths, R, mb, stagger, pool):
    """One decode step at a time: retire what is complete, then admit while the stagger and the free pages allow it."""
    B = len(lengths)
    n = -(-B // mb)
    pages = [sum(-(-(lengths[b] + R - 1) // 16) for b in range(i * mb, min(B, (i + 1) * mb))) for i in range(n)]
    admit, done = [None] * n, [None] * n
    free, step, last, front, nxt, peak = pool, 0, 0, 0, 0, 0
    while front < n:
        moved = True
        while moved:
            moved = False
            while front < nxt and done[front] <= step:
                free += pages[front]; front += 1; moved = True
            while nxt < n and (nxt == 0 or step - last >= stagger) and pages[nxt] <= free:
                admit[nxt], done[nxt] = step, step + R - 1
                free -= pages[nxt]; last = step; nxt += 1; moved = True
        assert 0 <= free <= pool
        if front < n:
            peak = max(peak, min(B, nxt * mb) - front * mb)
        step += 1
        assert step < 10 ** 6
    return admit, done, peak


def test_admission_plan_closed_forms():
    from paper_2312_11819_amd import binding as B
    lens = [100] * 64                                   # 100 + 50 - 1 = 149 tokens -> 10 pages per row, 160 per micro-batch of 16
    R = 50
    ample = 64 * 10
    assert B.rlhf_gen_plan_admission(lens, R, 16, 0, ample) == ([0, 0, 0, 0], [49] * 4, 64)          # everything at once
    assert B.rlhf_gen_plan_admission(lens, R, 16, 7, ample) == ([0, 7, 14, 21], [49, 56, 63, 70], 64)
    assert B.rlhf_gen_plan_admission(lens, R, 16, 49, ample) == ([0, 49, 98, 147], [49, 98, 147, 196], 16)   # one after the other
    assert B.rlhf_gen_plan_admission(lens, R, 16, 200, ample) == ([0, 200, 400, 600], [49, 249, 449, 649], 16)
    # a pool for two micro-batches: the third waits for the first to finish, the fourth for the second
    assert B.rlhf_gen_plan_admission(lens, R, 16, 7, 320) == ([0, 7, 49, 56], [49, 56, 98, 105], 32)
    assert B.rlhf_gen_plan_admission(lens, R, 16, 0, 320) == ([0, 0, 49, 49], [49, 49, 98, 98], 32)
    assert B.rlhf_gen_plan_admission(lens, R, 16, 0, 479) == ([0, 0, 49, 49], [49, 49, 98, 98], 32)  # one page short of three
    assert B.rlhf_gen_plan_admission(lens, 1, 16, 5, 160)[:2] == ([0, 5, 10, 15], [0, 5, 10, 15])    # R = 1: no decode steps
    assert B.rlhf_gen_plan_admission(lens[:40], R, 16, 3, ample) == ([0, 3, 6], [49, 52, 55], 40)     # ragged last micro-batch
    assert B.rlhf_gen_plan_admission(lens, R, 100, 3, ample) == ([0], [49], 64)                       # micro_batch > B
    with pytest.raises(B.RlhfGenError) as e:
        B.rlhf_gen_plan_admission(lens, R, 16, 0, 159)                                                # not even one micro-batch fits
    assert e.value.status == B.E_NOMEM
    for bad in (dict(max_resp_len=0), dict(micro_batch=0), dict(stagger_steps=-1), dict(kv_pool_blocks=0)):
        args = dict(lengths=lens, max_resp_len=R, micro_batch=16, stagger_steps=0, kv_pool_blocks=ample); args.update(bad)
        with pytest.raises(B.RlhfGenError) as e:
            B.rlhf_gen_plan_admission(**args)
        assert e.value.status == B.E_INVALID


def test_admission_plan_equals_step_by_step_simulation():
    """Seeded ragged batches, pools from 'barely one micro-batch' to 'everything': the plan is the earliest-admission
    schedule of a step-by-step simulation, pages in use never exceed the pool, micro-batches enter and leave in order."""
    import random
    from paper_2312_11819_amd import binding as B
    rng = random.Random(7)
    for _ in range(200):
        n_rows = rng.randint(1, 70)
        lens = [rng.randint(1, 300) for _ in range(n_rows)]
        R = rng.randint(1, 80)
        mb = rng.randint(1, 24)
        stagger = rng.choice([0, 1, 2, 5, 17, 100])
        per_mb = [sum(-(-(lens[b] + R - 1) // 16) for b in range(i, min(n_rows, i + mb))) for i in range(0, n_rows, mb)]
        pool = rng.randint(max(per_mb), sum(per_mb) + 5)
        want = _brute_force_schedule(lens, R, mb, stagger, pool)
        got = B.rlhf_gen_plan_admission(lens, R, mb, stagger, pool)
        assert got == want, (lens, R, mb, stagger, pool)
        admit, done, peak = got
        assert admit == sorted(admit) and all(d == a + R - 1 for a, d in zip(admit, done))
        assert all(b - a >= stagger for a, b in zip(admit, admit[1:]))
        assert (1 if R > 1 else 0) <= peak <= n_rows            # (R = 1: no row ever decodes)
