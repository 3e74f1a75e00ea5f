"""ctypes binding of librlhf_gen.so: argument marshalling only.

Every function here has the name of the C entry point it forwards to
(`rlhf_gen_init`, `rlhf_gen_prefill`, ...).  PyTorch supplies device memory and
the HIP stream; no arithmetic of the method happens in Python.  If the shared
library is missing the import of the functions fails loudly - there is no CPU
fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librlhf_gen.so")

OK, E_INVALID, E_NOMEM, E_STATE, E_DEVICE, E_UNSUPPORTED = 0, -1, -2, -3, -4, -5
DTYPE_FP32, DTYPE_BF16 = 0, 1
FLAG_SHUFFLE_BLOCKS, FLAG_NO_GRAPH, FLAG_GENERIC_GEMM, FLAG_CONVERT_IN_PLACE, FLAG_FUSED_ROPE, FLAG_PREFILL_FP16_PAIRS = 1, 2, 4, 8, 16, 32
GEMM_TILED, GEMM_STREAMING, GEMM_FP32 = 0, 1, 2
EPI_STORE_F32, EPI_RESID_F32, EPI_SWIGLU, EPI_STORE_H16 = 0, 1, 2, 3

PROF_CLASSES = ["embed", "norm", "gemm_qkv", "rope_append", "attn_decode", "gemm_wo", "gemm_gate_up", "swiglu",
                "gemm_down", "lm_head", "sampler"]

EXPORTS = [
    "rlhf_gen_init", "rlhf_gen_prefill", "rlhf_gen_decode_step", "rlhf_gen_generate", "rlhf_gen_generate_stream", "rlhf_gen_generate_continuous", "rlhf_gen_last_peak_rows", "rlhf_gen_plan_admission", "rlhf_gen_score", "rlhf_gen_update_weights",
    "rlhf_gen_plan_capacity", "rlhf_gen_context_bytes", "rlhf_gen_graph_captures",
    "rlhf_gen_get_logits",
    "rlhf_gen_last_timing", "rlhf_gen_last_step_ms", "rlhf_gen_set_profile", "rlhf_gen_get_profile", "rlhf_gen_last_error", "rlhf_gen_destroy",
    "rlhf_gen_op_probe_stream_read", "rlhf_gen_op_probe_mfma_loop", "rlhf_gen_op_tile_weights", "rlhf_gen_op_gemm", "rlhf_gen_op_rope_append", "rlhf_gen_op_attn_decode", "rlhf_gen_op_attn_prefill",
    "rlhf_gen_op_sample", "rlhf_gen_op_gemm_static", "rlhf_gen_op_tile_weights4", "rlhf_gen_op_rmsnorm_lo4", "rlhf_gen_op_gemm_lo4",
    "rlhf_gen_op_attn_decode_lo4", "rlhf_gen_op_attn_prefill_lo4",
]


class Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + [
        ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32), ("max_batch", C.c_int32),
        ("max_seq", C.c_int32), ("kv_block", C.c_int32), ("kv_pool_blocks", C.c_int32), ("device", C.c_int32),
        ("stream", C.c_void_p), ("flags", C.c_uint32)]


class Weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wqkv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)),
                ("ffn_norm", C.POINTER(C.c_void_p)), ("w_gate_up", C.POINTER(C.c_void_p)),
                ("w_down", C.POINTER(C.c_void_p))]


class LoraPair(C.Structure):
    _fields_ = [("a", C.c_void_p), ("b", C.c_void_p), ("rank", C.c_int32)]


class Lora(C.Structure):
    _fields_ = [("scale", C.c_float), ("wqkv", C.POINTER(LoraPair)), ("wo", C.POINTER(LoraPair)),
                ("w_gate_up", C.POINTER(LoraPair)), ("w_down", C.POINTER(LoraPair)), ("lm_head", LoraPair)]


class Sampling(C.Structure):
    _fields_ = [("temperature", C.c_float), ("top_p", C.c_float), ("seed", C.c_uint64), ("greedy", C.c_int32),
                ("logprob_mode", C.c_int32)]


class RlhfGenError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"rlhf_gen status {status}: {message}")
        self.status = status
        self.message = message


MICROBATCH_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p)

_lib = None


def lib() -> C.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        L.rlhf_gen_init.argtypes = [C.POINTER(Weights), C.POINTER(Cfg), C.POINTER(C.c_void_p)]
        L.rlhf_gen_prefill.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.c_int32, C.c_int32,
                                       C.POINTER(Sampling), C.c_void_p, C.c_void_p]
        L.rlhf_gen_decode_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.rlhf_gen_generate.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.c_int32,
                                        C.POINTER(Sampling), C.c_void_p, C.c_void_p]
        L.rlhf_gen_generate_stream.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.c_int32,
                                               C.POINTER(Sampling), C.c_void_p, C.c_void_p, C.c_int32,
                                               C.POINTER(C.c_void_p), MICROBATCH_FN, C.c_void_p]
        L.rlhf_gen_generate_continuous.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.c_int32,
                                                   C.POINTER(Sampling), C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                                   C.POINTER(C.c_void_p), MICROBATCH_FN, C.c_void_p]
        L.rlhf_gen_last_peak_rows.argtypes = [C.c_void_p]
        L.rlhf_gen_plan_admission.argtypes = [C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                              C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.rlhf_gen_score.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.c_void_p,
                                     C.c_int32, C.c_void_p]
        L.rlhf_gen_update_weights.argtypes = [C.c_void_p, C.POINTER(Weights), C.POINTER(Lora)]
        L.rlhf_gen_plan_capacity.argtypes = [C.POINTER(Cfg), C.c_int64, C.c_double, C.c_int64, C.POINTER(C.c_int32),
                                             C.POINTER(C.c_int64)]
        L.rlhf_gen_context_bytes.argtypes = [C.c_void_p]
        L.rlhf_gen_context_bytes.restype = C.c_int64
        L.rlhf_gen_graph_captures.argtypes = [C.c_void_p]
        L.rlhf_gen_graph_captures.restype = C.c_int64
        L.rlhf_gen_get_logits.argtypes = [C.c_void_p, C.c_void_p]
        L.rlhf_gen_last_timing.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_int32)]
        L.rlhf_gen_last_step_ms.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.c_int32, C.POINTER(C.c_int32)]
        L.rlhf_gen_set_profile.argtypes = [C.c_void_p, C.c_int32]
        L.rlhf_gen_get_profile.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                           C.POINTER(C.c_int32)]
        L.rlhf_gen_last_error.argtypes = [C.c_void_p]
        L.rlhf_gen_last_error.restype = C.c_char_p
        L.rlhf_gen_destroy.argtypes = [C.c_void_p]
        L.rlhf_gen_destroy.restype = None
        L.rlhf_gen_op_probe_stream_read.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p]
        L.rlhf_gen_op_probe_mfma_loop.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        L.rlhf_gen_op_tile_weights.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32]
        L.rlhf_gen_op_gemm.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                       C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.rlhf_gen_op_rope_append.argtypes = [C.c_void_p] * 9 + [C.c_int32] * 7
        L.rlhf_gen_op_attn_decode.argtypes = [C.c_void_p] * 4 + [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p] + [C.c_int32] * 3
        L.rlhf_gen_op_attn_prefill.argtypes = [C.c_void_p] * 4 + [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p] + [C.c_int32] * 4
        L.rlhf_gen_op_sample.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.POINTER(Sampling), C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p]
        L.rlhf_gen_op_gemm_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                              C.c_int32, C.POINTER(C.c_int32)]
        L.rlhf_gen_op_attn_decode_lo4.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                                  C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.rlhf_gen_op_attn_prefill_lo4.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.rlhf_gen_op_tile_weights4.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32]
        L.rlhf_gen_op_rmsnorm_lo4.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                              C.c_int32, C.c_float]
        L.rlhf_gen_op_gemm_lo4.argtypes = [C.c_void_p] + [C.c_void_p] * 5 + [C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                                                            C.c_int32]
        for name in EXPORTS:
            if name not in ("rlhf_gen_last_error", "rlhf_gen_destroy", "rlhf_gen_context_bytes", "rlhf_gen_graph_captures"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA/HIP tensors"
    return t.data_ptr()


def rlhf_gen_plan_capacity(shape, dtype: str, max_seq: int, capacity_bytes: int, fraction: float = 0.95,
                           reserved_bytes: int = -1, flags: int = 0, device: int = 0):
    """Largest batch a context of this shape can hold, and the device bytes it would allocate."""
    cfg = Cfg(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
              shape.vocab, shape.rms_eps, shape.rope_theta, DTYPE_BF16 if dtype == "bf16" else DTYPE_FP32,
              1, max_seq, 16, 0, device, None, flags)
    b, n = C.c_int32(), C.c_int64()
    _check(None, lib().rlhf_gen_plan_capacity(C.byref(cfg), int(capacity_bytes), float(fraction), int(reserved_bytes),
                                              C.byref(b), C.byref(n)))
    return b.value, n.value


def rlhf_gen_plan_admission(lengths: Sequence[int], max_resp_len: int, micro_batch: int, stagger_steps: int,
                            kv_pool_blocks: int):
    """(admit_step per micro-batch, done_step per micro-batch, peak rows in flight) - host only, no GPU."""
    B = len(lengths)
    n_mb = -(-B // max(min(micro_batch, B), 1))
    lens = (C.c_int32 * B)(*[int(x) for x in lengths])
    admit, done, peak = (C.c_int32 * n_mb)(), (C.c_int32 * n_mb)(), C.c_int32()
    _check(None, lib().rlhf_gen_plan_admission(lens, B, max_resp_len, micro_batch, stagger_steps, kv_pool_blocks, admit, done,
                                               C.byref(peak)))
    return list(admit), list(done), peak.value


def make_sampling(temperature=1.0, top_p=1.0, seed=0, greedy=False, logprob_mode=0) -> Sampling:
    return Sampling(float(temperature), float(top_p), int(seed), int(bool(greedy)), int(logprob_mode))


def _check(ctx: Optional[int], status: int) -> None:
    if status != OK:
        msg = lib().rlhf_gen_last_error(ctx)
        raise RlhfGenError(status, msg.decode() if msg else "")


class Context:
    """Owns one rlhf_gen_ctx.  Methods carry the names of the C entry points."""

    def __init__(self, weights: dict, shape, dtype: str, max_batch: int, max_seq: int, device: int = 0,
                 kv_pool_blocks: int = 0, flags: int = 0, stream: Optional[torch.cuda.Stream] = None):
        L = lib()
        self.shape, self.dtype, self.device = shape, dtype, torch.device("cuda", device)
        self.stream = stream if stream is not None else torch.cuda.Stream(device=self.device)
        w = self._marshal_weights(weights)
        cfg = Cfg(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                  shape.vocab, shape.rms_eps, shape.rope_theta, DTYPE_BF16 if dtype == "bf16" else DTYPE_FP32,
                  max_batch, max_seq, 16, kv_pool_blocks, device, self.stream.cuda_stream, flags)
        self.cfg = cfg
        h = C.c_void_p()
        torch.cuda.synchronize(self.device)
        _check(None, L.rlhf_gen_init(C.byref(w), C.byref(cfg), C.byref(h)))
        self._h = h
        self.B = 0

    def _enqueued(self, *tensors) -> None:
        """After a call that enqueued work on the context's stream: the tensors it reads or writes were allocated on
        the caller's stream, so tell the allocator they are in use on ours (their memory is not handed out again
        before that work has run), and make the caller's stream wait for ours, so that the caller may read the
        outputs, or drop them, in stream order without an explicit synchronisation."""
        for t in tensors:
            if t is not None:
                t.record_stream(self.stream)
        torch.cuda.current_stream(self.device).wait_stream(self.stream)

    def _marshal_weights(self, weights: dict) -> Weights:
        self._weights = weights  # borrowed by the library: keep alive
        n = self.shape.n_layers
        arr = lambda key: (C.c_void_p * n)(*[_ptr(lw[key]) for lw in weights["layers"]])
        self._arrs = {k: arr(k) for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")}
        return Weights(_ptr(weights["tok_emb"]), _ptr(weights["lm_head"]), _ptr(weights["final_norm"]),
                       *[C.cast(self._arrs[k], C.POINTER(C.c_void_p)) for k in
                         ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")])

    # -- the C entry points ------------------------------------------------------------------
    def rlhf_gen_update_weights(self, weights: dict, lora: Optional[dict] = None) -> None:
        """weights as for the constructor.  lora: {"scale": s, "layers": [{"wqkv": (A, B), ...}, ...], "lm_head": (A, B)}
        with any entry optional; A is [rank, in], B is [out, rank]."""
        w = self._marshal_weights(weights)
        lp = None
        if lora is not None:
            n = self.shape.n_layers
            self._lora = lora  # keep the adapter tensors alive until the conversion has run
            def pairs(key):
                arr = (LoraPair * n)()
                for l, lw in enumerate(lora.get("layers", [{}] * n)):
                    if lw.get(key) is not None:
                        a, b = lw[key]
                        arr[l] = LoraPair(_ptr(a), _ptr(b), a.shape[0])
                return arr
            self._lora_arrs = {k: pairs(k) for k in ("wqkv", "wo", "w_gate_up", "w_down")}
            head = LoraPair()
            if lora.get("lm_head") is not None:
                a, b = lora["lm_head"]
                head = LoraPair(_ptr(a), _ptr(b), a.shape[0])
            lp = Lora(float(lora.get("scale", 1.0)), *[C.cast(self._lora_arrs[k], C.POINTER(LoraPair)) for k in
                                                        ("wqkv", "wo", "w_gate_up", "w_down")], head)
        self.stream.wait_stream(torch.cuda.current_stream(self.device))
        _check(self._h, lib().rlhf_gen_update_weights(self._h, C.byref(w), C.byref(lp) if lp is not None else None))
        # the conversion reads the sources and the adapters on our stream: later writes to them must come after it
        torch.cuda.current_stream(self.device).wait_stream(self.stream)
        self.B = 0

    def rlhf_gen_prefill(self, query_tokens: torch.Tensor, lengths: Sequence[int], sampling: Sampling):
        B, Lmax = query_tokens.shape
        lens = (C.c_int32 * B)(*[int(x) for x in lengths])
        tok = torch.empty(B, dtype=torch.int32, device=self.device)
        lp = torch.empty(B, dtype=torch.float32, device=self.device)
        self.stream.wait_stream(torch.cuda.current_stream(self.device))
        try:
            _check(self._h, lib().rlhf_gen_prefill(self._h, _ptr(query_tokens), lens, B, Lmax, C.byref(sampling), _ptr(tok), _ptr(lp)))
        finally:
            self._enqueued(query_tokens, tok, lp)
        self.B = B
        return tok, lp

    def rlhf_gen_decode_step(self, forced_tokens: Optional[torch.Tensor] = None):
        tok = torch.empty(max(self.B, 1), dtype=torch.int32, device=self.device)
        lp = torch.empty(max(self.B, 1), dtype=torch.float32, device=self.device)
        self.stream.wait_stream(torch.cuda.current_stream(self.device))
        try:
            _check(self._h, lib().rlhf_gen_decode_step(self._h, _ptr(forced_tokens), _ptr(tok), _ptr(lp)))
        finally:
            self._enqueued(forced_tokens, tok, lp)
        return tok, lp

    def rlhf_gen_generate(self, query_tokens: torch.Tensor, lengths: Sequence[int], max_resp_len: int,
                          sampling: Sampling, out_tokens: Optional[torch.Tensor] = None,
                          out_logprobs: Optional[torch.Tensor] = None):
        B, Lmax = query_tokens.shape
        lens = (C.c_int32 * B)(*[int(x) for x in lengths])
        toks = out_tokens if out_tokens is not None else torch.empty(B, max_resp_len, dtype=torch.int32, device=self.device)
        lps = out_logprobs if out_logprobs is not None else torch.empty(B, max_resp_len, dtype=torch.float32, device=self.device)
        self.stream.wait_stream(torch.cuda.current_stream(self.device))
        try:
            _check(self._h, lib().rlhf_gen_generate(self._h, _ptr(query_tokens), lens, B, Lmax, max_resp_len,
                                                    C.byref(sampling), _ptr(toks), _ptr(lps)))
        finally:
            self._enqueued(query_tokens, toks, lps)
        self.B = B
        return toks, lps

    def rlhf_gen_generate_stream(self, query_tokens: torch.Tensor, lengths: Sequence[int], max_resp_len: int,
                                 sampling: Sampling, micro_batch: int, on_ready=None,
                                 out_tokens: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None):
        """on_ready(index, row0, rows, event) runs on this thread right after micro-batch `index` has been generated and
        `event` (a torch.cuda.Event recorded on the context's stream) marks its rows complete.
        Returns (tokens, logprobs, events)."""
        B, Lmax = query_tokens.shape
        lens = (C.c_int32 * B)(*[int(x) for x in lengths])
        toks = out_tokens if out_tokens is not None else torch.empty(B, max_resp_len, dtype=torch.int32, device=self.device)
        lps = out_logprobs if out_logprobs is not None else torch.empty(B, max_resp_len, dtype=torch.float32, device=self.device)
        n_mb = -(-B // max(micro_batch, 1))
        events = [torch.cuda.Event(enable_timing=True) for _ in range(n_mb)]
        with torch.cuda.stream(self.stream):
            for e in events:
                e.record()          # torch creates the HIP event at its first record
        handles = (C.c_void_p * n_mb)(*[e.cuda_event for e in events])
        failure = []

        def trampoline(_user, index, row0, rows, _ev):
            try:
                if on_ready is not None:
                    on_ready(index, row0, rows, events[index])
            except BaseException as exc:   # never unwind through the C frames
                failure.append(exc)

        cb = MICROBATCH_FN(trampoline)
        self.stream.wait_stream(torch.cuda.current_stream(self.device))
        try:
            _check(self._h, lib().rlhf_gen_generate_stream(self._h, _ptr(query_tokens), lens, B, Lmax, max_resp_len,
                                                           C.byref(sampling), _ptr(toks), _ptr(lps), micro_batch, handles, cb,
                                                           None))
        finally:
            self._enqueued(query_tokens, toks, lps)
        if failure:
            raise failure[0]
        self.B = min(micro_batch, B)
        return toks, lps, events

    def rlhf_gen_generate_continuous(self, query_tokens: torch.Tensor, lengths: Sequence[int], max_resp_len: int,
                                     sampling: Sampling, micro_batch: int, stagger_steps: int = 0, on_ready=None,
                                     out_tokens: Optional[torch.Tensor] = None, out_logprobs: Optional[torch.Tensor] = None):
        """Arguments and return value as rlhf_gen_generate_stream, plus the admission spacing in decode steps."""
        B, Lmax = query_tokens.shape
        lens = (C.c_int32 * B)(*[int(x) for x in lengths])
        toks = out_tokens if out_tokens is not None else torch.empty(B, max_resp_len, dtype=torch.int32, device=self.device)
        lps = out_logprobs if out_logprobs is not None else torch.empty(B, max_resp_len, dtype=torch.float32, device=self.device)
        n_mb = -(-B // max(min(micro_batch, B), 1))
        events = [torch.cuda.Event(enable_timing=True) for _ in range(n_mb)]
        with torch.cuda.stream(self.stream):
            for e in events:
                e.record()          # torch creates the HIP event at its first record
        handles = (C.c_void_p * n_mb)(*[e.cuda_event for e in events])
        failure = []

        def trampoline(_user, index, row0, rows, _ev):
            try:
                if on_ready is not None:
                    on_ready(index, row0, rows, events[index])
            except BaseException as exc:   # never unwind through the C frames
                failure.append(exc)

        cb = MICROBATCH_FN(trampoline)
        self.stream.wait_stream(torch.cuda.current_stream(self.device))
        try:
            _check(self._h, lib().rlhf_gen_generate_continuous(self._h, _ptr(query_tokens), lens, B, Lmax, max_resp_len,
                                                               C.byref(sampling), _ptr(toks), _ptr(lps), micro_batch,
                                                               stagger_steps, handles, cb, None))
        finally:
            self._enqueued(query_tokens, toks, lps)
        if failure:
            raise failure[0]
        self.B = 0
        return toks, lps, events

    def rlhf_gen_last_peak_rows(self) -> int:
        return int(lib().rlhf_gen_last_peak_rows(self._h))

    def rlhf_gen_score(self, query_tokens: torch.Tensor, lengths: Sequence[int], resp_tokens: torch.Tensor) -> torch.Tensor:
        B, Lmax = query_tokens.shape
        R = resp_tokens.shape[1]
        lens = (C.c_int32 * B)(*[int(x) for x in lengths])
        out = torch.empty(B, R, dtype=torch.float32, device=self.device)
        self.stream.wait_stream(torch.cuda.current_stream(self.device))
        try:
            _check(self._h, lib().rlhf_gen_score(self._h, _ptr(query_tokens), lens, B, Lmax, _ptr(resp_tokens), R, _ptr(out)))
        finally:
            self._enqueued(query_tokens, resp_tokens, out)
        self.synchronize()
        self.B = 0
        return out

    def rlhf_gen_context_bytes(self) -> int:
        return int(lib().rlhf_gen_context_bytes(self._h))

    def rlhf_gen_graph_captures(self) -> int:
        return int(lib().rlhf_gen_graph_captures(self._h))

    def rlhf_gen_get_logits(self) -> torch.Tensor:
        out = torch.empty(self.B, self.shape.vocab, dtype=torch.float32, device=self.device)
        self.stream.wait_stream(torch.cuda.current_stream(self.device))
        try:
            _check(self._h, lib().rlhf_gen_get_logits(self._h, _ptr(out)))
        finally:
            self._enqueued(out)
        self.synchronize()
        return out

    def rlhf_gen_last_timing(self):
        a, b, n = C.c_float(), C.c_float(), C.c_int32()
        _check(self._h, lib().rlhf_gen_last_timing(self._h, C.byref(a), C.byref(b), C.byref(n)))
        return a.value, b.value, n.value

    def rlhf_gen_last_step_ms(self):
        n = C.c_int32()
        _check(self._h, lib().rlhf_gen_last_step_ms(self._h, None, 0, C.byref(n)))
        buf = (C.c_float * max(n.value, 1))()
        _check(self._h, lib().rlhf_gen_last_step_ms(self._h, buf, n.value, C.byref(n)))
        return [buf[i] for i in range(n.value)]

    def rlhf_gen_set_profile(self, every: int) -> None:
        _check(self._h, lib().rlhf_gen_set_profile(self._h, every))

    def rlhf_gen_get_profile(self):
        ms = (C.c_double * len(PROF_CLASSES))()
        n = (C.c_int64 * len(PROF_CLASSES))()
        tok, steps = C.c_int64(), C.c_int32()
        _check(self._h, lib().rlhf_gen_get_profile(self._h, ms, n, C.byref(tok), C.byref(steps)))
        return {"ms": dict(zip(PROF_CLASSES, list(ms))), "launches": dict(zip(PROF_CLASSES, list(n))),
                "attn_tokens": tok.value, "steps": steps.value}

    def synchronize(self) -> None:
        self.stream.synchronize()

    def rlhf_gen_destroy(self) -> None:
        if getattr(self, "_h", None):
            lib().rlhf_gen_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.rlhf_gen_destroy()
        except Exception:
            pass


# -- single-operation entry points -------------------------------------------------------------------
def rlhf_gen_op_probe_stream_read(buf: torch.Tensor, nontemporal: bool, scratch: torch.Tensor) -> int:
    return lib().rlhf_gen_op_probe_stream_read(None, _ptr(buf), buf.numel() * buf.element_size(), int(nontemporal), _ptr(scratch))


def rlhf_gen_op_probe_mfma_loop(operands: torch.Tensor, workgroups: int, iters: int, scratch: torch.Tensor) -> int:
    return lib().rlhf_gen_op_probe_mfma_loop(None, _ptr(operands), workgroups, iters, _ptr(scratch))


def rlhf_gen_op_tile_weights(w_rowmajor: torch.Tensor, w_tiled: torch.Tensor) -> int:
    N, K = w_rowmajor.shape
    return lib().rlhf_gen_op_tile_weights(None, _ptr(w_rowmajor), _ptr(w_tiled), N, K)


def rlhf_gen_op_gemm(kind, A, W, out, M, N, K, epilogue=0, nsplit=1, a_pairs=0) -> int:
    return lib().rlhf_gen_op_gemm(None, kind, _ptr(A), _ptr(W), _ptr(out), M, N, K, epilogue, nsplit, a_pairs)


def rlhf_gen_op_tile_weights4(w_tiled, w4, w_scale, N, K) -> int:
    return lib().rlhf_gen_op_tile_weights4(None, _ptr(w_tiled), _ptr(w4), _ptr(w_scale), N, K)


def rlhf_gen_op_rmsnorm_lo4(x, gain_bf16, y, row_scale, scale_groups, M, d, eps) -> int:
    return lib().rlhf_gen_op_rmsnorm_lo4(None, _ptr(x), _ptr(gain_bf16), _ptr(y), _ptr(row_scale), scale_groups, M, d, eps)


def rlhf_gen_op_gemm_lo4(A, W, W4, w_scale, a_scale, scale_groups, out, M, N, K, epilogue=0) -> int:
    return lib().rlhf_gen_op_gemm_lo4(None, _ptr(A), _ptr(W), _ptr(W4), _ptr(w_scale), _ptr(a_scale), scale_groups, _ptr(out),
                                      M, N, K, epilogue)


def rlhf_gen_op_gemm_static(A, W, out, M, N, K, a_pairs=0):
    """Returns (status, split count used)."""
    ns = C.c_int32(0)
    rc = lib().rlhf_gen_op_gemm_static(None, _ptr(A), _ptr(W), _ptr(out), M, N, K, a_pairs, C.byref(ns))
    return rc, ns.value


def rlhf_gen_op_rope_append(qkv, row_pos, row_seq, cos_t, sin_t, q_out, kv_pool, block_table, max_blocks, n_blocks, M,
                            Hq, Hkv, head_dim, half16) -> int:
    return lib().rlhf_gen_op_rope_append(None, _ptr(qkv), _ptr(row_pos), _ptr(row_seq), _ptr(cos_t), _ptr(sin_t),
                                         _ptr(q_out), _ptr(kv_pool), _ptr(block_table), max_blocks, n_blocks, M, Hq,
                                         Hkv, head_dim, int(half16))


def rlhf_gen_op_attn_decode(q, kv_pool, block_table, max_blocks, n_blocks, seq_len, out, B, Hq, Hkv) -> int:
    return lib().rlhf_gen_op_attn_decode(None, _ptr(q), _ptr(kv_pool), _ptr(block_table), max_blocks, n_blocks,
                                         _ptr(seq_len), _ptr(out), B, Hq, Hkv)


def rlhf_gen_op_attn_prefill(q, kv_pool, block_table, max_blocks, n_blocks, cu_seqlens, seq_ids, out, nseq, max_len, Hq,
                             Hkv) -> int:
    return lib().rlhf_gen_op_attn_prefill(None, _ptr(q), _ptr(kv_pool), _ptr(block_table), max_blocks, n_blocks,
                                          _ptr(cu_seqlens), _ptr(seq_ids), _ptr(out), nseq, max_len, Hq, Hkv)


def rlhf_gen_op_attn_decode_lo4(q, kv_pool, block_table, max_blocks, n_blocks, seq_len, out, row_scale, scale_groups, B, Hq, Hkv) -> int:
    return lib().rlhf_gen_op_attn_decode_lo4(None, _ptr(q), _ptr(kv_pool), _ptr(block_table), max_blocks, n_blocks, _ptr(seq_len),
                                             _ptr(out), _ptr(row_scale), scale_groups, B, Hq, Hkv)


def rlhf_gen_op_attn_prefill_lo4(q, kv_pool, block_table, max_blocks, n_blocks, cu_seqlens, seq_ids, out, row_scale, scale_groups,
                                 nseq, max_len, Hq, Hkv) -> int:
    return lib().rlhf_gen_op_attn_prefill_lo4(None, _ptr(q), _ptr(kv_pool), _ptr(block_table), max_blocks, n_blocks, _ptr(cu_seqlens),
                                              _ptr(seq_ids), _ptr(out), _ptr(row_scale), scale_groups, nseq, max_len, Hq, Hkv)


def rlhf_gen_op_sample(logits, sampling: Sampling, step, tok_out, lp_out, scratch_tok) -> int:
    B, V = logits.shape
    return lib().rlhf_gen_op_sample(None, _ptr(logits), B, V, C.byref(sampling), _ptr(step), _ptr(tok_out),
                                    _ptr(lp_out), _ptr(scratch_tok))
