"""CPU-only checks of the C-ABI library: it loads, exports every symbol the headers declare, and rejects bad
arguments before touching a GPU.  Also the stored fixtures under tests/golden/."""
import ctypes as C
import json
import math
import os
import re

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2312_11819_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build(verbose=False)
    binding.lib()
    return binding


def test_every_declared_symbol_is_exported(B):
    declared = set()
    for name in ("rlhf_gen.h", "rlhf_gen_ops.h"):
        text = open(os.path.join(ROOT, "include", name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        declared |= set(re.findall(r"\b(rlhf_gen_\w+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for sym in sorted(declared):
        assert hasattr(L, sym), sym


def _cfg(B, **over):
    base = dict(n_layers=2, d_model=128, n_heads=4, n_kv_heads=4, head_dim=32, d_ffn=344, vocab=512, rms_eps=1e-5,
                rope_theta=10000.0, dtype=0, max_batch=4, max_seq=32, kv_block=16, kv_pool_blocks=0, device=0,
                stream=None, flags=0)
    base.update(over)
    return B.Cfg(*[base[f[0]] for f in B.Cfg._fields_])


def _weights(B, n_layers=2, null_layer=False):
    fake = 0x1000  # never dereferenced: validation fails first
    arr = (C.c_void_p * n_layers)(*([fake] * n_layers))
    if null_layer:
        arr[1] = None
    p = C.cast(arr, C.POINTER(C.c_void_p))
    return B.Weights(fake, fake, fake, p, p, p, p, p, p), arr


def test_init_rejects_bad_arguments_without_a_gpu(B):
    L = B.lib()
    h = C.c_void_p()
    w, keep = _weights(B)
    assert L.rlhf_gen_init(None, C.byref(_cfg(B)), C.byref(h)) == B.E_INVALID
    assert L.rlhf_gen_init(C.byref(w), None, C.byref(h)) == B.E_INVALID
    assert L.rlhf_gen_init(C.byref(w), C.byref(_cfg(B)), None) == B.E_INVALID
    cases = [(dict(n_layers=0), B.E_INVALID), (dict(n_heads=4, n_kv_heads=3), B.E_INVALID), (dict(kv_block=32), B.E_UNSUPPORTED),
             (dict(dtype=7), B.E_INVALID), (dict(max_seq=1), B.E_INVALID), (dict(head_dim=48), B.E_UNSUPPORTED),
             (dict(dtype=1), B.E_UNSUPPORTED), (dict(kv_pool_blocks=-1), B.E_INVALID), (dict(rms_eps=0.0), B.E_INVALID),
             (dict(d_model=9000), B.E_UNSUPPORTED)]
    for over, want in cases:
        assert L.rlhf_gen_init(C.byref(w), C.byref(_cfg(B, **over)), C.byref(h)) == want, over
        assert not h.value
        assert L.rlhf_gen_last_error(None)
    w2, keep2 = _weights(B, null_layer=True)
    assert L.rlhf_gen_init(C.byref(w2), C.byref(_cfg(B)), C.byref(h)) == B.E_INVALID
    if not torch.cuda.is_available():
        assert L.rlhf_gen_init(C.byref(w), C.byref(_cfg(B)), C.byref(h)) == B.E_DEVICE
        assert b"device" in L.rlhf_gen_last_error(None).lower()


def test_calls_on_a_null_context_fail_cleanly(B):
    L = B.lib()
    assert L.rlhf_gen_decode_step(None, None, None, None) == B.E_INVALID
    assert L.rlhf_gen_get_logits(None, None) == B.E_INVALID
    assert L.rlhf_gen_set_profile(None, 1) == B.E_INVALID
    L.rlhf_gen_destroy(None)
    assert L.rlhf_gen_op_gemm(None, 0, None, None, None, 1, 1, 1, 0, 1, 0) == B.E_INVALID
    assert L.rlhf_gen_op_sample(None, None, 1, 1, None, None, None, None, None) == B.E_INVALID


def test_golden_closed_forms():
    rows = [l.split("\t") for l in open(os.path.join(ROOT, "tests", "golden", "closed_forms.txt")) if l[0].isdigit()]
    assert len(rows) == 2
    for v, want in rows:
        assert abs(-math.log(int(v)) - float(want)) < 1e-12


def test_oracle_reproduces_its_stored_tiny_rollout():
    from oracle.generate import generate
    from oracle.sampling import Sampling
    from paper_2312_11819_amd import synth
    doc = json.load(open(os.path.join(ROOT, "tests", "golden", "tiny_greedy.json")))
    wl = synth.WORKLOADS["tiny"]
    w = synth.make_weights(wl.shape, wl.weight_seed)
    toks, lens = synth.workload_queries(wl)
    qs = [toks[b, : lens[b]].tolist() for b in range(wl.batch)]
    out = generate(w, wl.shape, qs, wl.resp_len, Sampling(greedy=True), method="full", keep_logits=False)
    assert out["tokens"].tolist() == doc["tokens"]
    assert (out["logprobs"] - torch.tensor(doc["logprobs"], dtype=torch.float64)).abs().max() < 1e-9
