"""Kernel-by-kernel parity of the HIP library against CPU definitions (oracle pieces, float64)."""
import math

import pytest
import torch

from oracle import sampling as OS
from oracle import transformer as OT
from tests.gpu_util import bf16_round, need_gpu, oracle_attention_rows, rope_tables

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    need_gpu()
    from paper_2312_11819_amd import binding
    binding.lib()
    return binding


def _tiled(B, w: torch.Tensor) -> torch.Tensor:
    """Device copy of the fp16 matrix w [N, K] in the working layout of the 16-bit GEMMs."""
    src = w.cuda().contiguous()
    dst = torch.empty_like(src)
    assert B.rlhf_gen_op_tile_weights(src, dst) == 0
    return dst


@pytest.mark.parametrize("N,K", [(48, 384), (256, 256), (592, 128), (1040, 384)])
def test_tile_weights_layout(B, N, K):
    """Tiles of 16 rows x 128 columns, inside a tile [k/32 % 4][row % 16][k % 32]; slabs of 16 row-blocks (the last one
    may be shorter), inside a slab [k/128][row-block]."""
    w = torch.arange(N * K, dtype=torch.int32).remainder(30000).to(torch.int16).view(N, K)
    got = _tiled(B, w.view(torch.float16)).cpu().view(torch.int16).flatten()
    slabs = []
    for r0 in range(0, N, 256):
        sl = w[r0:r0 + 256]                                                   # [rows, K], rows a multiple of 16
        nb = sl.shape[0] // 16
        # [rb, 16, ks, 4, 32] -> [ks, rb, 4 (k/32), 16 (row), 32]
        slabs.append(sl.reshape(nb, 16, K // 128, 4, 32).permute(2, 0, 3, 1, 4).contiguous().flatten())
    assert torch.equal(got, torch.cat(slabs))
    t = torch.zeros(16, 128, dtype=torch.float16, device="cuda")
    assert B.rlhf_gen_op_tile_weights(t, t) == B.E_INVALID                   # in place is not possible
    assert B.rlhf_gen_op_tile_weights(torch.zeros(8, 128, dtype=torch.float16, device="cuda"),
                                      torch.zeros(8, 128, dtype=torch.float16, device="cuda")) == B.E_INVALID


def _rand(shape, seed, scale=1.0, dtype=torch.float16):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(*shape, generator=g) * scale).to(dtype)


@pytest.mark.parametrize("M,N,K", [(300, 512, 256), (1024, 256, 384), (7, 256, 128), (513, 768, 1024)])
def test_gemm_tiled_store_and_accumulate(B, M, N, K):
    a, w = _rand((M, K), 1), _rand((N, K), 2, 0.05)
    ref = a.double() @ w.double().T
    A, W = a.cuda(), _tiled(B, w)
    out = torch.full((M, N), 7.0, dtype=torch.float32, device="cuda")
    assert B.rlhf_gen_op_gemm(B.GEMM_TILED, A, W, out, M, N, K, B.EPI_STORE_F32) == 0
    torch.cuda.synchronize()
    tol = 1e-5 * math.sqrt(K) + 1e-6
    assert (out.cpu().double() - ref).abs().max() < tol
    assert B.rlhf_gen_op_gemm(B.GEMM_TILED, A, W, out, M, N, K, B.EPI_RESID_F32) == 0
    torch.cuda.synchronize()
    assert (out.cpu().double() - 2 * ref).abs().max() < 2 * tol
    outb = torch.zeros((M, N), dtype=torch.float16, device="cuda")
    assert B.rlhf_gen_op_gemm(B.GEMM_TILED, A, W, outb, M, N, K, B.EPI_STORE_H16) == 0
    torch.cuda.synchronize()
    assert (outb.cpu().double() - ref).abs().max() <= ref.abs().max() * 2 ** -11 + tol


@pytest.mark.parametrize("M,F,K", [(300, 384, 256), (64, 128, 128), (1000, 1152, 512)])
def test_gemm_tiled_swiglu(B, M, F, K):
    a, w = _rand((M, K), 3), _rand((2 * F, K), 4, 0.1)
    gu = a.double() @ w.double().T
    ref = OT.silu(gu[:, :F]) * gu[:, F:]
    out = torch.zeros((M, F), dtype=torch.float16, device="cuda")
    assert B.rlhf_gen_op_gemm(B.GEMM_TILED, a.cuda(), _tiled(B, w), out, M, F, K, B.EPI_SWIGLU) == 0
    torch.cuda.synchronize()
    err = (out.cpu().double() - ref).abs()
    assert (err <= ref.abs() * 2 ** -11 + 1e-4).all()


@pytest.mark.parametrize("M,N,K,ns", [(4, 128, 256, 1), (16, 512, 1024, 3), (64, 640, 1024, 2), (50, 256, 1408, 4),
                                      (200, 256, 512, 2), (256, 192, 1024, 8), (33, 64, 128, 1)])
def test_gemm_streaming(B, M, N, K, ns):
    a, w = _rand((M, K), 5), _rand((N, K), 6, 0.05)
    ref = a.double() @ w.double().T
    part = torch.full((ns, M, N), float("nan"), dtype=torch.float32, device="cuda")
    assert B.rlhf_gen_op_gemm(B.GEMM_STREAMING, a.cuda(), _tiled(B, w), part, M, N, K, 0, ns) == 0
    torch.cuda.synchronize()
    got = part.cpu().double().sum(0)
    assert (got - ref).abs().max() < 1e-5 * math.sqrt(K) + 1e-6


def test_gemm_seeded_shape_sweep(B):
    """Thirty seeded shapes across the three forms of the decode GEMM and the split-K tile form: every batch-width
    instantiation, ragged row counts, split counts with a short last split, gate/up widths with a ragged last
    workgroup."""
    rng = torch.Generator().manual_seed(2024)
    ri = lambda lo, hi: int(torch.randint(lo, hi + 1, (1,), generator=rng))
    for case in range(30):
        form = ("plain", "pairs", "swiglu", "tile_split")[case % 4]
        K = 128 * ri(1, 12)
        steps = K // 128
        if form == "swiglu":
            M, F = ri(1, 128), 32 * ri(1, 40)
            a, w = _rand((M, K), 100 + case), _rand((2 * F, K), 200 + case, 0.1)
            gu = a.double() @ w.double().T
            ref = OT.silu(gu[:, :F]) * gu[:, F:]
            out = torch.zeros((M, F), dtype=torch.float16, device="cuda")
            assert B.rlhf_gen_op_gemm(B.GEMM_STREAMING, a.cuda(), _tiled(B, w), out, M, F, K, B.EPI_SWIGLU, 1) == 0, (case, M, F, K)
            torch.cuda.synchronize()
            assert ((out.cpu().double() - ref).abs() <= ref.abs() * 2 ** -11 + 1e-4).all(), (case, M, F, K)
            continue
        pairs = form == "pairs"
        if form == "tile_split":
            M, N = ri(129, 300), 256 * ri(1, 4)
            nkw = K // 32
            per = -(-nkw // ri(2, 8))
            ns = -(-nkw // per)
            pairs = bool(case % 8 >= 4)
        else:
            M, N = ri(1, 128), 64 * ri(1, 12)
            per = -(-steps // ri(1, min(8, steps)))
            ns = -(-steps // per)
        x = torch.randn(M, K, generator=rng, dtype=torch.float64)
        hi = x.to(torch.float16)
        w = _rand((N, K), 300 + case, 0.05)
        if pairs:
            lo = (x - hi.double()).to(torch.float16)
            a = torch.cat([hi, lo], dim=1).contiguous().cuda()
            ref = (hi.double() + lo.double()) @ w.double().T
        else:
            a, ref = hi.cuda(), hi.double() @ w.double().T
        part = torch.full((ns, M, N), float("nan"), dtype=torch.float32, device="cuda")
        kind = B.GEMM_TILED if form == "tile_split" else B.GEMM_STREAMING
        rc = B.rlhf_gen_op_gemm(kind, a, _tiled(B, w), part, M, N, K, 0, ns, int(pairs))
        if form == "tile_split" and ns == 1:
            part = part[0]
        assert rc == 0, (case, form, M, N, K, ns)
        torch.cuda.synchronize()
        got = part.cpu().double().sum(0) if part.dim() == 3 else part.cpu().double()
        assert (got - ref).abs().max() < 1e-5 * math.sqrt(K) + 1e-6, (case, form, M, N, K, ns)


@pytest.mark.parametrize("M,F,K", [(64, 352, 256), (5, 32, 128), (200, 96, 512),
                                   # widths that 8, 7 or 6 wavefronts of 8 features do not divide (ragged last workgroup),
                                   # at every batch-width instantiation; the last is the 7B width (230 workgroups of 6)
                                   (16, 1376, 256), (32, 13824, 128), (128, 480, 256), (64, 11008, 512)])
def test_gemm_streaming_swiglu(B, M, F, K):
    a, w = _rand((M, K), 13), _rand((2 * F, K), 14, 0.1)
    gu = a.double() @ w.double().T
    ref = OT.silu(gu[:, :F]) * gu[:, F:]
    out = torch.zeros((M, F), dtype=torch.float16, device="cuda")
    assert B.rlhf_gen_op_gemm(B.GEMM_STREAMING, a.cuda(), _tiled(B, w), out, M, F, K, B.EPI_SWIGLU, 1) == 0
    torch.cuda.synchronize()
    err = (out.cpu().double() - ref).abs()
    assert (err <= ref.abs() * 2 ** -11 + 1e-4).all()


@pytest.mark.parametrize("kind,M,N,K,ns", [("tiled", 300, 512, 256, 1), ("tiled", 1024, 256, 384, 1),
                                            ("stream", 64, 256, 512, 2), ("stream", 17, 128, 128, 1), ("stream", 128, 192, 1024, 3),
                                            ("stream", 64, 256, 1024, 2), ("stream", 20, 384, 2048, 4), ("stream", 9, 128, 512, 1),
                                            # K / 512 splits, <= 64 rows and at least two 128-row tiles per workgroup:
                                            # the resident-slice kernel
                                            ("stream", 64, 8192, 4096, 8), ("stream", 20, 12288, 4096, 8), ("stream", 7, 8320, 2048, 4)])
def test_gemm_with_activation_pairs(B, kind, M, N, K, ns):
    g = torch.Generator().manual_seed(31)
    x = torch.randn(M, K, generator=g, dtype=torch.float64)
    hi = x.to(torch.float16)
    lo = (x - hi.double()).to(torch.float16)
    w = _rand((N, K), 32, 0.05)
    ref = x @ w.double().T
    a = torch.cat([hi, lo], dim=1).contiguous().cuda()                      # [M, 2K]
    if kind == "tiled":
        out = torch.zeros((M, N), dtype=torch.float32, device="cuda")
        assert B.rlhf_gen_op_gemm(B.GEMM_TILED, a, _tiled(B, w), out, M, N, K, B.EPI_STORE_F32, 1, 1) == 0
        got = out.cpu().double()
    else:
        part = torch.zeros((ns, M, N), dtype=torch.float32, device="cuda")
        assert B.rlhf_gen_op_gemm(B.GEMM_STREAMING, a, _tiled(B, w), part, M, N, K, 0, ns, 1) == 0
        got = part.cpu().double().sum(0)
    torch.cuda.synchronize()
    # the pair carries ~22 bits, so the result is far more accurate than a single fp16 operand would allow
    assert (got - ref).abs().max() < 2e-5 * math.sqrt(K)
    assert (got - hi.double() @ w.double().T).abs().max() > (got - ref).abs().max()


def test_gemm_pairs_same_bits_for_any_row_count(B):
    """The pair-input streaming GEMM accumulates every output element in the same order whichever kernel serves the
    row count (resident-slice kernel up to 64 rows, ring kernel above): a row's partial sums do not depend on how
    many other rows are in the call."""
    N, K, ns = 8320, 4096, 8          # 65 tiles over 32 workgroups per split: 2 or 3 tiles each
    g = torch.Generator().manual_seed(41)
    x = torch.randn(100, K, generator=g, dtype=torch.float64)
    hi = x.to(torch.float16)
    lo = (x - hi.double()).to(torch.float16)
    a = torch.cat([hi, lo], dim=1).contiguous().cuda()
    w = _tiled(B, _rand((N, K), 42, 0.05))
    outs = {}
    for M in (100, 64, 40, 16, 7):
        part = torch.zeros((ns, M, N), dtype=torch.float32, device="cuda")
        assert B.rlhf_gen_op_gemm(B.GEMM_STREAMING, a[:M].contiguous(), w, part, M, N, K, 0, ns, 1) == 0
        torch.cuda.synchronize()
        outs[M] = part.cpu()
    for M in (64, 40, 16, 7):
        assert torch.equal(outs[M], outs[100][:, :M])


def test_gemm_fp32(B):
    M, N, K = 37, 344, 128
    a, w = _rand((M, K), 7, 1.0, torch.float32), _rand((N, K), 8, 0.05, torch.float32)
    ref = a.double() @ w.double().T
    out = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    assert B.rlhf_gen_op_gemm(B.GEMM_FP32, a.cuda(), w.cuda(), out, M, N, K, B.EPI_STORE_F32) == 0
    assert B.rlhf_gen_op_gemm(B.GEMM_FP32, a.cuda(), w.cuda(), out, M, N, K, B.EPI_RESID_F32) == 0
    torch.cuda.synchronize()
    assert (out.cpu().double() - 2 * ref).abs().max() < 1e-5


@pytest.mark.parametrize("M,N,K,ns,pairs", [(256, 512, 1024, 4, 0), (200, 768, 384, 3, 1), (129, 256, 128, 2, 0),
                                             (256, 256, 1408, 16, 0), (300, 512, 512, 5, 1), (256, 12288, 4096, 5, 1)])
def test_gemm_tiled_split_k(B, M, N, K, ns, pairs):
    """Split-K form of the tiled GEMM (decode batches of 129..256 rows): the planes add up to the product; a split
    count that would leave a split empty is refused."""
    nkw = K // 32
    per = -(-nkw // ns)
    ns = -(-nkw // per)                                                      # the nearest count with no empty split
    g = torch.Generator().manual_seed(41)
    x = torch.randn(M, K, generator=g, dtype=torch.float64)
    hi = x.to(torch.float16)
    w = _rand((N, K), 42, 0.05)
    if pairs:
        lo = (x - hi.double()).to(torch.float16)
        a = torch.cat([hi, lo], dim=1).contiguous().cuda()
        ref = (hi.double() + lo.double()) @ w.double().T
    else:
        a = hi.cuda()
        ref = hi.double() @ w.double().T
    part = torch.full((ns, M, N), 3.0, dtype=torch.float32, device="cuda")
    assert B.rlhf_gen_op_gemm(B.GEMM_TILED, a, _tiled(B, w), part, M, N, K, B.EPI_STORE_F32, ns, pairs) == 0
    torch.cuda.synchronize()
    assert (part.cpu().double().sum(0) - ref).abs().max() < 1e-5 * math.sqrt(K) + 1e-6
    if ns > 1:
        # every plane holds a share of the sum (none is left at its fill value, none is the whole product)
        assert float((part[0].cpu().double() - ref).abs().max()) > 1e-3
    if nkw % 7 and nkw > 7 and -(-nkw // (-(-nkw // 7))) != 7:
        assert B.rlhf_gen_op_gemm(B.GEMM_TILED, a, _tiled(B, w), part, M, N, K, B.EPI_STORE_F32, 7, pairs) == B.E_UNSUPPORTED


def test_gemm_rejects_bad_shapes(B):
    t = torch.zeros(256, 256, dtype=torch.float16, device="cuda")
    o = torch.zeros(256, 256, dtype=torch.float32, device="cuda")
    assert B.rlhf_gen_op_gemm(B.GEMM_TILED, t, t, o, 256, 200, 256, 0) == B.E_UNSUPPORTED
    assert B.rlhf_gen_op_gemm(B.GEMM_TILED, t, t, o, 256, 256, 100, 0) == B.E_UNSUPPORTED
    assert B.rlhf_gen_op_gemm(B.GEMM_STREAMING, t, t, o, 300, 256, 256, 0, 1) == B.E_UNSUPPORTED
    assert B.rlhf_gen_op_gemm(9, t, t, o, 256, 256, 256, 0, 1) == B.E_INVALID


@pytest.mark.parametrize("Hq,Hkv,lens", [(2, 2, [1, 17, 64, 5]), (8, 1, [33, 100]), (4, 2, [16, 48, 31])])
def test_attention_prefill_then_decode(B, Hq, Hkv, lens):
    h, nseq = 128, len(lens)
    width = (Hq + 2 * Hkv) * h
    T = sum(lens)
    maxpos = max(lens) + 1
    max_blocks = (maxpos + 15) // 16
    n_blocks = nseq * max_blocks + 3
    g = torch.Generator().manual_seed(11)
    table = torch.randperm(n_blocks, generator=g)[: nseq * max_blocks].reshape(nseq, max_blocks).to(torch.int32)
    qkv = torch.randn(T + nseq, width, generator=g)                      # prefill rows, then one decode row per sequence
    cos_t, sin_t = rope_tables(maxpos, h)
    row_seq = torch.tensor([b for b, L in enumerate(lens) for _ in range(L)], dtype=torch.int32)
    row_pos = torch.tensor([p for L in lens for p in range(L)], dtype=torch.int32)
    cu = torch.tensor([0] + list(torch.tensor(lens).cumsum(0)), dtype=torch.int32)
    pool = torch.zeros(Hkv, n_blocks, 8192, dtype=torch.uint8, device="cuda")
    dev = lambda t: t.cuda().contiguous()
    qkv_d, cos_d, sin_d, table_d = dev(qkv), dev(cos_t), dev(sin_t), dev(table)
    q_out = torch.zeros(T, Hq, 2, h, dtype=torch.float16, device="cuda")
    assert B.rlhf_gen_op_rope_append(qkv_d[:T].contiguous(), dev(row_pos), dev(row_seq), cos_d, sin_d, q_out, pool,
                                     table_d, max_blocks, n_blocks, T, Hq, Hkv, h, True) == 0
    out = torch.zeros(T, 2, Hq * h, dtype=torch.float16, device="cuda")
    seq_ids = torch.arange(nseq, dtype=torch.int32, device="cuda")
    assert B.rlhf_gen_op_attn_prefill(q_out, pool, table_d, max_blocks, n_blocks, dev(cu), seq_ids, out, nseq, max(lens), Hq, Hkv) == 0
    # decode row for each sequence at position len
    qd = torch.zeros(nseq, Hq, 2, h, dtype=torch.float16, device="cuda")
    seq_len = torch.tensor(lens, dtype=torch.int32, device="cuda")
    assert B.rlhf_gen_op_rope_append(qkv_d[T:].contiguous(), seq_len, None, cos_d, sin_d, qd, pool, table_d, max_blocks,
                                     n_blocks, nseq, Hq, Hkv, h, True) == 0
    outd = torch.zeros(nseq, 2, Hq * h, dtype=torch.float16, device="cuda")
    assert B.rlhf_gen_op_attn_decode(qd, pool, table_d, max_blocks, n_blocks, seq_len, outd, nseq, Hq, Hkv) == 0
    torch.cuda.synchronize()
    # CPU definition on the unrounded fp32 inputs
    scale = 1.0 / math.sqrt(h)
    worst = 0.0
    for b, L in enumerate(lens):
        rows = torch.cat([qkv[cu[b]: cu[b] + L], qkv[T + b: T + b + 1]]).double()
        pos = torch.arange(L + 1)
        q = OT.rope(rows[:, : Hq * h].reshape(L + 1, Hq, h), pos, 10000.0)
        k = OT.rope(rows[:, Hq * h: (Hq + Hkv) * h].reshape(L + 1, Hkv, h), pos, 10000.0)
        v = rows[:, (Hq + Hkv) * h:].reshape(L + 1, Hkv, h)
        for i in range(L + 1):
            for j in range(Hq):
                kv = j // (Hq // Hkv)
                want = oracle_attention_rows(q[i, j], k[: i + 1, kv], v[: i + 1, kv], scale)
                src = out[cu[b] + i] if i < L else outd[b]
                got = src[:, j * h:(j + 1) * h].cpu().double().sum(0)                 # hi + lo
                worst = max(worst, float((got - want).abs().max()))
    assert worst < 3e-3, worst   # fp16 rounding of k and v on values of order 1


def test_attention_long_context(B):
    """Contexts beyond 4096 tokens: a wavefront's pages no longer fit one batch of 64 block-table entries (decode),
    and the prefill tiles walk hundreds of pages.  Sampled rows against the CPU definition."""
    Hq, Hkv, h = 4, 2, 128
    lens = [4400, 130]
    nseq, T = len(lens), sum(lens)
    width = (Hq + 2 * Hkv) * h
    maxpos = max(lens) + 1
    max_blocks = (maxpos + 15) // 16
    n_blocks = nseq * max_blocks + 5
    g = torch.Generator().manual_seed(12)
    table = torch.randperm(n_blocks, generator=g)[: nseq * max_blocks].reshape(nseq, max_blocks).to(torch.int32)
    qkv = torch.randn(T + nseq, width, generator=g)
    cos_t, sin_t = rope_tables(maxpos, h)
    row_seq = torch.tensor([b for b, L in enumerate(lens) for _ in range(L)], dtype=torch.int32)
    row_pos = torch.tensor([p for L in lens for p in range(L)], dtype=torch.int32)
    cu = torch.tensor([0] + list(torch.tensor(lens).cumsum(0)), dtype=torch.int32)
    pool = torch.zeros(Hkv, n_blocks, 8192, dtype=torch.uint8, device="cuda")
    dev = lambda t: t.cuda().contiguous()
    qkv_d, cos_d, sin_d, table_d = dev(qkv), dev(cos_t), dev(sin_t), dev(table)
    q_out = torch.zeros(T, Hq, 2, h, dtype=torch.float16, device="cuda")
    assert B.rlhf_gen_op_rope_append(qkv_d[:T].contiguous(), dev(row_pos), dev(row_seq), cos_d, sin_d, q_out, pool,
                                     table_d, max_blocks, n_blocks, T, Hq, Hkv, h, True) == 0
    out = torch.zeros(T, 2, Hq * h, dtype=torch.float16, device="cuda")
    seq_ids = torch.arange(nseq, dtype=torch.int32, device="cuda")
    assert B.rlhf_gen_op_attn_prefill(q_out, pool, table_d, max_blocks, n_blocks, dev(cu), seq_ids, out, nseq, max(lens), Hq, Hkv) == 0
    qd = torch.zeros(nseq, Hq, 2, h, dtype=torch.float16, device="cuda")
    seq_len = torch.tensor(lens, dtype=torch.int32, device="cuda")
    assert B.rlhf_gen_op_rope_append(qkv_d[T:].contiguous(), seq_len, None, cos_d, sin_d, qd, pool, table_d, max_blocks,
                                     n_blocks, nseq, Hq, Hkv, h, True) == 0
    outd = torch.zeros(nseq, 2, Hq * h, dtype=torch.float16, device="cuda")
    assert B.rlhf_gen_op_attn_decode(qd, pool, table_d, max_blocks, n_blocks, seq_len, outd, nseq, Hq, Hkv) == 0
    torch.cuda.synchronize()
    scale = 1.0 / math.sqrt(h)
    worst = 0.0
    for b, L in enumerate(lens):
        rows = torch.cat([qkv[cu[b]: cu[b] + L], qkv[T + b: T + b + 1]]).double()
        pos = torch.arange(L + 1)
        q = OT.rope(rows[:, : Hq * h].reshape(L + 1, Hq, h), pos, 10000.0)
        k = OT.rope(rows[:, Hq * h: (Hq + Hkv) * h].reshape(L + 1, Hkv, h), pos, 10000.0)
        v = rows[:, (Hq + Hkv) * h:].reshape(L + 1, Hkv, h)
        for i in sorted({0, 15, 16, L // 2, L - 1, L}):          # L = the decode row
            for j in range(Hq):
                kv = j // (Hq // Hkv)
                want = oracle_attention_rows(q[i, j], k[: i + 1, kv], v[: i + 1, kv], scale)
                src = out[cu[b] + i] if i < L else outd[b]
                got = src[:, j * h:(j + 1) * h].cpu().double().sum(0)
                worst = max(worst, float((got - want).abs().max()))
    assert worst < 3e-3, worst


@pytest.mark.parametrize("mode", ["greedy", "plain", "nucleus", "nucleus_lp1", "tight"])
def test_sampler(B, mode):
    V, rows = 32000, 6
    g = torch.Generator().manual_seed(21)
    logits = torch.randn(rows, V, generator=g) * 2.0
    logits[2, 777] = logits[2].max() + 3.0                                  # one peaked row
    cfgs = {"greedy": dict(greedy=True), "plain": dict(temperature=1.0, top_p=1.0, seed=5),
            "nucleus": dict(temperature=0.8, top_p=0.9, seed=6), "nucleus_lp1": dict(temperature=1.3, top_p=0.5, seed=7, logprob_mode=1),
            "tight": dict(temperature=1.0, top_p=1e-6, seed=8)}[mode]
    sp = B.make_sampling(**cfgs)
    osp = OS.Sampling(**cfgs)
    ld = logits.cuda()
    for t in (0, 3, 500):
        step = torch.tensor([t], dtype=torch.int32, device="cuda")
        tok = torch.zeros(rows, dtype=torch.int32, device="cuda")
        lp = torch.zeros(rows, dtype=torch.float32, device="cuda")
        scr = torch.zeros(rows, dtype=torch.int32, device="cuda")
        assert B.rlhf_gen_op_sample(ld, sp, step, tok, lp, scr) == 0
        torch.cuda.synchronize()
        assert torch.equal(tok, scr)
        for b in range(rows):
            want_tok, want_lp, info = OS.sample(logits[b], osp, b, t)
            got = int(tok[b])
            if got != want_tok:
                # allowed only when u sits within 1e-3 of an edge of the oracle's CDF interval
                assert not osp.greedy and OS.cdf_margin(info, want_tok) < 1e-3, (b, t, got, want_tok)
                continue
            assert abs(float(lp[b]) - want_lp) < 1e-4, (b, t, float(lp[b]), want_lp)


def test_hardware_probes_run(B):
    scratch = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    buf = torch.zeros(1 << 20, dtype=torch.int32, device="cuda")
    assert B.rlhf_gen_op_probe_stream_read(buf, False, scratch) == 0
    assert B.rlhf_gen_op_probe_stream_read(buf, True, scratch) == 0
    assert B.rlhf_gen_op_probe_stream_read(buf[:16], True, scratch) == B.E_INVALID        # less than one 8 KB chunk
    ops = torch.ones(8192, dtype=torch.float16, device="cuda")
    assert B.rlhf_gen_op_probe_mfma_loop(ops, 4, 10, scratch) == 0
    assert B.rlhf_gen_op_probe_mfma_loop(ops, 0, 10, scratch) == B.E_INVALID
    torch.cuda.synchronize()
    assert int(scratch.sum()) == 0                                                           # the probes write nothing
