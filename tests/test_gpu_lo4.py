"""The 4-bit side format of the prefill GEMMs' low halves, kernel by kernel.

The inputs of the QKV and the output projection travel as pairs hi + lo (fp16 high half, low half 2^-11 of it).  In the
large-tile GEMM the low half is contracted by the block-scaled 4-bit MFMA against a 4-bit copy of the weights.  The format
is defined here once more on the CPU, from its description in include/rlhf_gen_ops.h: e2m1 elements (sign; magnitudes 0,
0.5, 1, 1.5, 2, 3, 4, 6), nearest value with ties towards zero, two per byte with the even k in the low nibble, and a
power-of-two scale 2^(byte - 127) per group, the smallest that brings the group's largest magnitude to 6 or below.
Checked: the weight copy byte for byte, the activation rows against a float64 RMSNorm, the GEMM against (a) the float64
product of exactly the values its operands encode - which pins layout, scales and accumulation - and (b) the float64
product of the unrounded activations, where it has to beat a single fp16 operand by a wide margin; and the whole prefill
against the fp16-pair form of the same context."""
import math

import pytest
import torch

from paper_2312_11819_amd import synth
from tests.gpu_util import need_gpu

pytestmark = pytest.mark.gpu

GRID = torch.tensor([0, 0.5, 1, 1.5, 2, 3, 4, 6], dtype=torch.float64)
EDGES = torch.tensor([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0], dtype=torch.float64)


@pytest.fixture(scope="module")
def B():
    need_gpu()
    from paper_2312_11819_amd import binding
    binding.lib()
    return binding


def scale_bytes(amax: torch.Tensor) -> torch.Tensor:
    """Smallest power of two s = 2^(byte - 127) with amax <= 6 s."""
    e = torch.ceil(torch.log2(amax.double().clamp_min(1e-300) / 6.0))
    return (e + 127).clamp(1, 254).to(torch.int64)


def encode(v: torch.Tensor) -> torch.Tensor:
    """e2m1 code (4 bits) of v, already divided by its scale."""
    mag = (v.abs().double()[..., None] > EDGES).sum(-1)
    return mag + 8 * (v < 0).to(torch.int64)


def decode(codes: torch.Tensor) -> torch.Tensor:
    return GRID[codes & 7] * (1 - 2 * (codes >> 3)).double()


def tiled16(words: torch.Tensor) -> torch.Tensor:
    """[N, C] 16-bit words (C % 128 == 0) in the working layout of the GEMMs: slabs of 256 rows, [k/128][row-block] inside a
    slab, [k/32 % 4][row % 16][k % 32] inside a tile."""
    N, C = words.shape
    out = []
    for r0 in range(0, N, 256):
        sl = words[r0:r0 + 256]
        nb = sl.shape[0] // 16
        out.append(sl.reshape(nb, 16, C // 128, 4, 32).permute(2, 0, 3, 1, 4).contiguous().flatten())
    return torch.cat(out)


def untiled16(flat: torch.Tensor, N: int, C: int) -> torch.Tensor:
    out = torch.empty(N, C, dtype=flat.dtype)
    pos = 0
    for r0 in range(0, N, 256):
        rows = min(256, N - r0)
        nb = rows // 16
        blk = flat[pos:pos + rows * C].reshape(C // 128, nb, 4, 16, 32).permute(1, 3, 0, 2, 4).reshape(rows, C)
        out[r0:r0 + rows] = blk
        pos += rows * C
    return out


def nibbles_to_codes(words: torch.Tensor) -> torch.Tensor:
    """[N, C] 16-bit words -> [N, 4C] codes, k = 4 c + i in bits [4 i, 4 i + 4)."""
    w = words.to(torch.int64) & 0xFFFF
    return torch.stack([(w >> (4 * i)) & 15 for i in range(4)], dim=-1).reshape(words.shape[0], -1)


def _tiled(B, w: torch.Tensor) -> torch.Tensor:
    src = w.cuda().contiguous()
    dst = torch.empty_like(src)
    assert B.rlhf_gen_op_tile_weights(src, dst) == 0
    return dst


def _w4(B, wt: torch.Tensor, N: int, K: int):
    w4 = torch.zeros(N * K // 2, dtype=torch.uint8, device="cuda")
    ws = torch.zeros(N, dtype=torch.uint8, device="cuda")
    assert B.rlhf_gen_op_tile_weights4(wt, w4, ws, N, K) == 0
    torch.cuda.synchronize()
    return w4, ws


@pytest.mark.parametrize("N,K", [(256, 512), (592, 1024), (48, 2048)])
def test_weight_copy_byte_for_byte(B, N, K):
    g = torch.Generator().manual_seed(5)
    w = (torch.randn(N, K, generator=g) * 0.02 * (1 + 3 * torch.rand(N, 1, generator=g))).to(torch.float16)   # rows of different scale
    w[3] = 0                                                                                                   # an all-zero row
    w4, ws = _w4(B, _tiled(B, w), N, K)
    sb = scale_bytes(w.double().abs().amax(1))
    assert torch.equal(ws.cpu().to(torch.int64), sb)
    codes = encode(w.double() / torch.exp2((sb - 127).double())[:, None])                       # [N, K]
    words = sum(codes.reshape(N, K // 4, 4)[:, :, i] << (4 * i) for i in range(4))             # [N, K / 4]
    want = tiled16(words.to(torch.int32)).to(torch.int16)
    assert torch.equal(w4.cpu().view(torch.int16), want)
    assert B.rlhf_gen_op_tile_weights4(_tiled(B, w), w4, ws, N, K + 128) == B.E_INVALID        # K % 512


def _rmsnorm_lo4(B, x: torch.Tensor, gain: torch.Tensor, groups: int):
    M, d = x.shape
    y = torch.zeros(M, 4 * d, dtype=torch.uint8, device="cuda")
    sc = torch.zeros(d // 128 * groups * 128, dtype=torch.uint8, device="cuda")
    assert B.rlhf_gen_op_rmsnorm_lo4(x.cuda(), gain.cuda(), y, sc, groups, M, d, 1e-5) == 0
    torch.cuda.synchronize()
    return y, sc


def _decode_rows(y: torch.Tensor, sc: torch.Tensor, M: int, d: int, groups: int):
    """hi [M, d] float64, lo [M, d] float64 (decoded), scale bytes [M, d / 128]."""
    yc = y.cpu()
    hi = yc[:, : 2 * d].contiguous().view(torch.float16).double()
    lo_bytes = yc[:, 2 * d: 2 * d + d // 2].to(torch.int64)
    codes = torch.stack([lo_bytes & 15, lo_bytes >> 4], dim=-1).reshape(M, d)
    m = torch.arange(M)[:, None]
    t = torch.arange(d // 128)[None, :]
    idx = ((t * groups + m // 128) * 32 + m % 32) * 4 + (m // 32) % 4
    sb = sc.cpu().to(torch.int64)[idx]                                                           # [M, d / 128]
    lo = decode(codes) * torch.exp2((sb - 127).double()).repeat_interleave(128, dim=1)
    return hi, lo, sb


@pytest.mark.parametrize("M,d", [(300, 512), (77, 4096), (1500, 1024)])
def test_rmsnorm_rows_in_the_4bit_pair_form(B, M, d):
    g = torch.Generator().manual_seed(9)
    x = torch.randn(M, d, generator=g) * (0.1 + torch.rand(M, 1, generator=g))
    gain = (0.5 + torch.rand(d, generator=g)).to(torch.bfloat16)
    groups = 2 * ((M + 255) // 256)
    y, sc = _rmsnorm_lo4(B, x, gain, groups)
    hi, lo, sb = _decode_rows(y, sc, M, d, groups)
    xd = x.double()
    ref = xd / torch.sqrt((xd * xd).mean(-1, keepdim=True) + 1e-5) * gain.double()
    # high half: the fp16 nearest to the (fp32) result; low half: what is left, to within the quantisation step
    assert (hi - ref).abs().max() <= ref.abs().max() * 2 ** -11
    resid = ref - hi
    s = torch.exp2((sb - 127).double())
    amax = resid.reshape(M, d // 128, 128).abs().amax(-1)
    assert (6 * s >= amax * (1 - 1e-2)).all() and (3 * s <= amax * (1 + 1e-2) + 1e-12).all()   # the smallest power of two that covers the group
    err = (hi + lo - ref)
    assert (err.abs().reshape(M, d // 128, 128).amax(-1) <= s * 1.02 + 2e-6).all()              # coarsest step (4 .. 6) is 2 s: error <= s
    assert err.pow(2).mean().sqrt() < 0.3 * resid.pow(2).mean().sqrt()                         # ~ 5x closer than the fp16 value alone


@pytest.mark.parametrize("M,N,K,resid", [(300, 512, 1024, False), (1024, 256, 512, True), (513, 768, 4096, False), (16384, 256, 512, False),
                                         (777, 1280, 5120, True), (130, 10240, 8192, False), (1, 256, 512, False)])
def test_gemm_with_4bit_low_halves(B, M, N, K, resid):
    g = torch.Generator().manual_seed(11)
    x = torch.randn(M, K, generator=g)
    gain = torch.ones(K, dtype=torch.bfloat16)
    w = (torch.randn(N, K, generator=g) * 0.05).to(torch.float16)
    groups = 2 * ((M + 255) // 256)
    y, sc = _rmsnorm_lo4(B, x, gain, groups)
    wt = _tiled(B, w)
    w4, ws = _w4(B, wt, N, K)
    out = torch.full((M, N), 7.0 if resid else 0.0, dtype=torch.float32, device="cuda")
    assert B.rlhf_gen_op_gemm_lo4(y, wt, w4, ws, sc, groups, out, M, N, K, B.EPI_RESID_F32 if resid else B.EPI_STORE_F32) == 0
    torch.cuda.synchronize()
    got = out.cpu().double() - (7.0 if resid else 0.0)
    # (a) against the values the operands encode: pins the layouts, the scale plumbing and the accumulation
    hi, lo, _ = _decode_rows(y, sc, M, K, groups)
    wcodes = nibbles_to_codes(untiled16(w4.cpu().view(torch.int16), N, K // 4))
    w4v = decode(wcodes) * torch.exp2((ws.cpu().to(torch.int64) - 127).double())[:, None]
    enc = hi @ w.double().T + lo @ w4v.T
    assert (got - enc).abs().max() < 2e-6 * math.sqrt(K) + (1e-6 if not resid else 2e-6)
    # (b) against the unrounded activations: far closer than the fp16 high halves alone
    xd = x.double()
    ref = (xd / torch.sqrt((xd * xd).mean(-1, keepdim=True) + 1e-5)) @ w.double().T
    e_lo4 = (got - ref).pow(2).mean().sqrt()
    e_hi = (hi @ w.double().T - ref).pow(2).mean().sqrt()
    assert e_lo4 < 0.3 * e_hi
    assert (got - ref).abs().max() < 4e-5 * math.sqrt(K)


def test_gemm_lo4_rejects_bad_shapes(B):
    z = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    o = torch.zeros(256 * 256, dtype=torch.float32, device="cuda")
    assert B.rlhf_gen_op_gemm_lo4(z, z, z, z, z, 2, o, 256, 256, 384, 0) == B.E_UNSUPPORTED   # K % 512
    assert B.rlhf_gen_op_gemm_lo4(z, z, z, z, z, 2, o, 256, 128, 512, 0) == B.E_UNSUPPORTED   # N % 256
    assert B.rlhf_gen_op_gemm_lo4(z, z, z, z, z, 1, o, 256, 256, 512, 0) == B.E_UNSUPPORTED   # too few scale groups
    assert B.rlhf_gen_op_gemm_lo4(z, z, z, z, z, 2, o, 256, 256, 512, B.EPI_SWIGLU) == B.E_INVALID


def test_prefill_with_4bit_low_halves_is_as_close_to_the_oracle_as_fp16_pairs(B):
    """Two contexts on the same weights, one with RLHF_GEN_FLAG_PREFILL_FP16_PAIRS: first-token logits of a ragged batch
    at the 7B layer width (2 layers) against the oracle.  The two forms differ from each other about as much as each
    differs from the oracle - a perturbation of 1e-5 re-draws the fp16 roundings downstream of it - so what is compared
    is each form's own distance to the oracle: the 4-bit low halves may cost a few per cent of the rms error, no more."""
    from oracle.generate import generate as oracle_generate
    from oracle.sampling import Sampling as OSampling
    shape = synth.with_layers(synth.LLAMA_7B, 2)
    w = synth.make_weights(shape, 61, "bf16", "cuda")
    toks, lens = synth.make_queries(shape.vocab, 6, 40, 300, 62)
    lg = []
    for flags in (0, B.FLAG_PREFILL_FP16_PAIRS):
        ctx = B.Context(w, shape, "bf16", 6, 320, flags=flags)
        ctx.rlhf_gen_prefill(toks.cuda(), lens.tolist(), B.make_sampling(1.0, 1.0, 3))
        lg.append(ctx.rlhf_gen_get_logits().cpu().double())
        ctx.rlhf_gen_destroy()
    assert not torch.equal(lg[0], lg[1])                                        # the flag does select another kernel
    w_host = {k: v.cpu().float() for k, v in w.items() if k != "layers"}
    w_host["layers"] = [{k: v.cpu().float() for k, v in lw.items()} for lw in w["layers"]]
    qs = [toks[b, : lens[b]].tolist() for b in range(6)]
    ref = oracle_generate(w_host, shape, qs, 1, OSampling(temperature=1.0, top_p=1.0, seed=3), dtype=torch.float32)["logits"][:, 0].double()
    rms = [float((x - ref).pow(2).mean().sqrt()) for x in lg]
    mx = [float((x - ref).abs().max()) for x in lg]
    print(f"\n4-bit low halves: max {mx[0]:.5f} rms {rms[0]:.6f}; fp16 pairs: max {mx[1]:.5f} rms {rms[1]:.6f}")
    assert max(mx) < 3e-2
    assert rms[0] < 1.15 * rms[1]


@pytest.mark.parametrize("Hq,Hkv,lens", [(2, 2, [1, 17, 64, 5]), (8, 1, [33, 100]), (4, 2, [16, 48, 31, 130])])
def test_attention_outputs_in_the_4bit_pair_form(B, Hq, Hkv, lens):
    """Prefill and decode attention write their output rows either as fp16 pairs or with 4-bit low halves.  On the same
    cache and queries the high halves are the same bits, every scale byte is the smallest power of two that covers its
    (row, head) group of fp16 low halves, and the decoded 4-bit low halves follow the fp16 ones to within the format's
    step.  (The pair form itself is checked against the CPU definition in tests/test_gpu_ops.py.)"""
    from tests.gpu_util import rope_tables
    h, nseq = 128, len(lens)
    width = (Hq + 2 * Hkv) * h
    T = sum(lens)
    maxpos = max(lens) + 1
    max_blocks = (maxpos + 15) // 16
    n_blocks = nseq * max_blocks + 3
    g = torch.Generator().manual_seed(11)
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
    seq_ids = torch.arange(nseq, dtype=torch.int32, device="cuda")
    groups = 2 * ((nseq * max(lens) + 255) // 256)

    def both_forms(rows, pair_call, lo4_call):
        pair = torch.zeros(rows, 2, Hq * h, dtype=torch.float16, device="cuda")
        assert pair_call(pair) == 0
        four = torch.zeros(rows, 4 * Hq * h, dtype=torch.uint8, device="cuda")
        sc = torch.zeros(Hq * groups * 128, dtype=torch.uint8, device="cuda")
        assert lo4_call(four, sc) == 0
        torch.cuda.synchronize()
        hi, lo, sb = _decode_rows(four, sc, rows, Hq * h, groups)
        p = pair.cpu().double()
        assert torch.equal(hi, p[:, 0])
        s = torch.exp2((sb - 127).double())
        amax = p[:, 1].reshape(rows, Hq, h).abs().amax(-1)
        assert (6 * s >= amax * (1 - 1e-2)).all() and (3 * s <= amax * (1 + 1e-2) + 1e-12).all()
        err = (lo - p[:, 1]).reshape(rows, Hq, h)
        # the fp16 low half is itself rounded (2^-11 of it), the 4-bit one to the nearest of 0, .5, 1, 1.5, 2, 3, 4, 6 scales
        assert (err.abs().amax(-1) <= s * 1.02 + 1e-9).all()
        assert err.pow(2).mean().sqrt() < 0.3 * p[:, 1].pow(2).mean().sqrt()

    both_forms(T,
               lambda o: B.rlhf_gen_op_attn_prefill(q_out, pool, table_d, max_blocks, n_blocks, dev(cu), seq_ids, o, nseq, max(lens), Hq, Hkv),
               lambda o, sc: B.rlhf_gen_op_attn_prefill_lo4(q_out, pool, table_d, max_blocks, n_blocks, dev(cu), seq_ids, o, sc, groups, nseq,
                                                           max(lens), Hq, Hkv))
    qd = torch.zeros(nseq, Hq, 2, h, dtype=torch.float16, device="cuda")
    seq_len = torch.tensor(lens, dtype=torch.int32, device="cuda")
    assert B.rlhf_gen_op_rope_append(qkv_d[T:].contiguous(), seq_len, None, cos_d, sin_d, qd, pool, table_d, max_blocks,
                                     n_blocks, nseq, Hq, Hkv, h, True) == 0
    both_forms(nseq,
               lambda o: B.rlhf_gen_op_attn_decode(qd, pool, table_d, max_blocks, n_blocks, seq_len, o, nseq, Hq, Hkv),
               lambda o, sc: B.rlhf_gen_op_attn_decode_lo4(qd, pool, table_d, max_blocks, n_blocks, seq_len, o, sc, groups, nseq, Hq, Hkv))
