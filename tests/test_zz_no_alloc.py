"""The allocation-free entry point rlhf_gen_op_gemm_static against the existing rlhf_gen_op_gemm (STREAMING), whose
split-K partial sums the caller holds: same kernels, same split count, planes added in the same order, so the two must
agree bit for bit.  Two calls in a row share the library's static workspace, the second with a smaller input (what the
first call left behind must not leak into it)."""
import pytest
import torch

from tests.gpu_util import need_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    need_gpu()
    from paper_2312_11819_amd import binding
    binding.lib()
    return binding


def _case(B, M, N, K, pairs, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    a = torch.randn(M, K * (2 if pairs else 1), generator=g, device="cuda").half()
    w0 = (torch.randn(N, K, generator=g, device="cuda") * 0.05).half()
    w = torch.empty_like(w0)
    assert B.rlhf_gen_op_tile_weights(w0, w) == B.OK
    out = torch.full((M, N), float("nan"), device="cuda")
    rc, ns = B.rlhf_gen_op_gemm_static(a, w, out, M, N, K, int(pairs))
    assert rc == B.OK and ns >= 1
    planes = torch.full((ns, M, N), float("nan"), device="cuda")
    assert B.rlhf_gen_op_gemm(B.GEMM_STREAMING, a, w, planes, M, N, K, B.EPI_STORE_F32, ns, int(pairs)) == B.OK
    torch.cuda.synchronize()
    want = planes[0].clone()
    for s in range(1, ns):
        want += planes[s]
    assert torch.equal(out, want), (M, N, K, pairs, ns, float((out - want).abs().max()))
    # and against the definition, in float64 (fp32 accumulation over K products of fp16 values)
    a64 = a.double()
    if pairs:
        a64 = a64[:, :K] + a64[:, K:]
    ref = a64 @ w0.double().T
    assert float((out.double() - ref).abs().max()) <= 2e-5 * (K ** 0.5) * float(ref.abs().max() + 1)


def test_static_workspace_matches_the_caller_workspace_entry_point(B):
    _case(B, 64, 4096, 4096, True, 1)      # 7B output projection at the benchmark's batch: 8 planes of 1 MB
    _case(B, 7, 256, 512, True, 2)         # much smaller, right after: nothing of the previous call may show
    _case(B, 64, 4096, 11008, False, 3)    # 7B down projection
    _case(B, 100, 1024, 1408, False, 4)    # ragged rows, a split count that does not divide the k-steps evenly
    _case(B, 3, 64, 128, False, 5)


def test_static_workspace_limits(B):
    a = torch.zeros(128, 2 * 4096, device="cuda", dtype=torch.float16)
    w = torch.zeros(12288, 4096, device="cuda", dtype=torch.float16)
    out = torch.zeros(128, 12288, device="cuda")
    # the 7B QKV projection with pair inputs runs 8 splits: at 128 rows the planes take 8 x 128 x 12288 floats = 48 MiB
    rc, _ = B.rlhf_gen_op_gemm_static(a, w, out, 128, 12288, 4096, 1)
    assert rc == B.E_INVALID
    assert b"static workspace" in B.lib().rlhf_gen_last_error(None)
    rc, ns = B.rlhf_gen_op_gemm_static(a, w, out, 80, 12288, 4096, 1)      # 30 MiB: fits
    assert rc == B.OK and ns == 8
    rc, _ = B.rlhf_gen_op_gemm_static(a, w, out, 300, 4096, 4096, 0)       # more rows than the streaming GEMM takes
    assert rc == B.E_UNSUPPORTED
    rc, _ = B.rlhf_gen_op_gemm_static(a, w, out, 16, 4000, 4096, 0)        # N not a multiple of 64
    assert rc == B.E_UNSUPPORTED
    torch.cuda.synchronize()
