"""Benchmark of the Actor rollout on one MI355X: `python bench.py --gpus 1 --steps K --warmup W`.

One "step" is one whole rollout (rlhf_gen_generate: prefill of the queries + R - 1 KV-cached decode steps)
of the 7B-shaped bf16 workload: 64 queries of 512 tokens, 512 response tokens each, temperature 1, top-p 1,
seeded sampling, random-init weights, uniform random token ids.  Inputs are resident in HBM before the
timed region.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12          # B/s, MI355X datasheet
MFMA_BF16_PEAK = 2.5e15    # flop/s dense, MI355X datasheet


def weight_bytes(shape, elt=2):
    from paper_2312_11819_amd import synth
    return (synth.param_count(shape) - shape.vocab * shape.d_model) * elt   # the embedding table is gathered, not streamed


def _time_gpu(fn, reps=5, warm=2):
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e-3


def hardware_probes(binding, dev):
    """What the card sustains with nothing in the way: a read-only stream over 4 GiB (plain and nontemporal loads, one workgroup per compute unit) and
    the fp16 MFMA pipe on register-resident operands (random values in [-1, 1], and zeros: the clock follows the data)."""
    import torch
    scratch = torch.zeros(1024, dtype=torch.uint8, device=dev)
    buf = torch.empty(1 << 30, dtype=torch.int32, device=dev).random_()   # 4 GiB: long enough that the launch ramp does not count
    out = {}
    for name, nt in (("hbm_read_plain_GBps", False), ("hbm_read_nontemporal_GBps", True)):
        t = _time_gpu(lambda: binding.rlhf_gen_op_probe_stream_read(buf, nt, scratch))
        out[name] = buf.numel() * 4 / t / 1e9
    del buf
    wgs, iters = 512, 20000
    flop = wgs * 4 * 8 * iters * 32768.0
    for name, ops in (("mfma_f16_random_operands_TFLOPs", (torch.rand(8192, device=dev) * 2 - 1).half()),
                      ("mfma_f16_zero_operands_TFLOPs", torch.zeros(8192, device=dev, dtype=torch.float16))):
        t = _time_gpu(lambda: binding.rlhf_gen_op_probe_mfma_loop(ops, wgs, iters, scratch), reps=3, warm=1)
        out[name] = flop / t / 1e12
    return out


def prefill_gemm_shapes(binding, shape, rows, dev, lo4=True):
    """The four projection GEMMs of one layer at the prefill chunk size, one by one through the kernel entry point:
    time, flop rate of the product (2 M N K; x 2 for the fused gate/up pair) and of what the kernel executes.  The QKV
    and output projections take their input as a pair hi + lo: with the low half in the 4-bit side format (the
    rollout's form where the widths allow it) the second pass costs a quarter of an fp16 pass, so the kernel executes
    1.25 x the product's flops in fp16-equivalent MFMA time; with fp16 low halves it executes 2 x."""
    import torch
    d, F, hq = shape.d_model, shape.d_ffn, shape.n_heads * shape.head_dim
    out = {}
    for name, N, K, epi, dual in (("qkv", shape.qkv_rows, d, 0, 1), ("attn_out", d, hq, 1, 1), ("gate_up_swiglu", F, d, 2, 0),
                                  ("down", d, F, 1, 0)):
        w0 = (torch.randn(N * (2 if epi == 2 else 1), K, device=dev) * 0.02).half()
        w = torch.empty_like(w0)
        binding.rlhf_gen_op_tile_weights(w0, w)
        o = torch.zeros(rows, N, device=dev, dtype=torch.float16 if epi == 2 else torch.float32)
        four_bit = bool(dual and lo4 and K % 512 == 0 and N % 256 == 0)
        if four_bit:
            groups = 2 * ((rows + 255) // 256)
            a = torch.zeros(rows, 4 * K, device=dev, dtype=torch.uint8)
            sc = torch.zeros(K // 128 * groups * 128, device=dev, dtype=torch.uint8)
            rc = binding.rlhf_gen_op_rmsnorm_lo4(torch.randn(rows, K, device=dev), torch.ones(K, device=dev, dtype=torch.bfloat16), a, sc,
                                                 groups, rows, K, 1e-5)
            w4 = torch.zeros(N * K // 2, device=dev, dtype=torch.uint8)
            ws = torch.zeros(N, device=dev, dtype=torch.uint8)
            rc = rc or binding.rlhf_gen_op_tile_weights4(w, w4, ws, N, K)
            if rc:
                raise RuntimeError(f"4-bit operands for the {name} shape: status {rc}")
            t = _time_gpu(lambda: binding.rlhf_gen_op_gemm_lo4(a, w, w4, ws, sc, groups, o, rows, N, K, epi))
            executed = 1.25
        else:
            a = torch.randn(rows, K * (2 if dual else 1), device=dev).half()
            t = _time_gpu(lambda: binding.rlhf_gen_op_gemm(binding.GEMM_TILED, a, w, o, rows, N, K, epi, 1, dual))
            executed = 2.0 if dual else 1.0
        flop = 2.0 * rows * N * K * (2 if epi == 2 else 1)
        out[name] = {"M": rows, "N": N * (2 if epi == 2 else 1), "K": K, "ms": t * 1e3, "TFLOPs": flop / t / 1e12,
                     "input": ("fp16 + 4-bit low half" if four_bit else "fp16 pair") if dual else "fp16",
                     "executed_TFLOPs": flop * executed / t / 1e12,
                     "executed_frac_of_mfma_peak": flop * executed / t / MFMA_BF16_PEAK}
        del a, w0, w, o
    return out


def traffic_ratios(workload: str):
    """Fetched / algorithmic byte ratios and written bytes per launch of the decode kernels, read from the committed
    counter summary profiles/bench_<workload>_pmc_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs).  Returns
    {kernel name prefix: (ratio, written bytes)} or raises if a kernel this bench reports on is no longer in the table
    (the summary is stale: the counters have to be collected again)."""
    path = os.path.join(ROOT, "profiles", f"bench_{workload}_pmc_traffic.md")
    if not os.path.exists(path):
        return None
    rows = {}
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) == 6 and cells[0] and cells[1].isdigit():
            try:
                rows[cells[0]] = {"launches": int(cells[1]), "fetched": float(cells[2]) * 1e6, "written": float(cells[3]) * 1e6,
                                  "algorithmic": float(cells[4]) * 1e6 if cells[4] not in ("-", "") else None}
            except ValueError:
                continue
    out = {}
    for key in ("attn_decode_kernel", "gemm_skinny"):
        sel = [r for k, r in rows.items() if k.startswith(key) and r["algorithmic"]]
        if not sel:
            raise RuntimeError(f"{path} has no row for {key}*: collect the traffic counters again for the current kernels")
        n = sum(r["launches"] for r in sel)
        out[key] = (sum(r["fetched"] * r["launches"] for r in sel) / sum(r["algorithmic"] * r["launches"] for r in sel),
                    sum(r["written"] * r["launches"] for r in sel) / n)
    return out


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline_and_parity(binding, ctx, wl, w_dev, toks, lens, rows, decode_steps=4):
    """The oracle as it stands (float32 mode, KV-cached) on a bounded sample of the workload - whole query prefill +
    `decode_steps` decode steps for the batch rows `rows` - timed on the host cores; and, with the logits it produced,
    the parity of the GPU path on the same rows in the same run: the context replays the prefill and the decode steps,
    the sampled rows teacher-forced with the oracle's tokens, and every logit and log-prob is compared."""
    import torch
    from oracle.generate import generate as oracle_generate
    from oracle.sampling import Sampling as OSampling
    from paper_2312_11819_amd import synth
    w_cpu = synth.weights_to(w_dev, "cpu")
    # the caller's bf16 values widened once, outside the timed region (the GPU path's one-time weight conversion is
    # outside its timed region too)
    w_cpu = {**{k: v.float() for k, v in w_cpu.items() if k != "layers"},
             "layers": [{k: v.float() for k, v in lw.items()} for lw in w_cpu["layers"]]}
    qs = [toks[b, : lens[b]].tolist() for b in range(toks.shape[0])]
    osp = OSampling(temperature=wl.temperature, top_p=wl.top_p, seed=wl.sample_seed, greedy=wl.greedy)
    n_tok = decode_steps + 1
    t0 = time.perf_counter()
    ref = oracle_generate(w_cpu, wl.shape, qs, n_tok, osp, rows=rows, dtype=torch.float32)
    dt = time.perf_counter() - t0
    del w_cpu
    rate = len(rows) * n_tok / dt
    B, R = toks.shape[0], wl.resp_len
    fed = sum(int(lens[b]) for b in rows) + len(rows) * decode_steps          # tokens the sample pushed through the model
    fed_full = int(lens.sum()) + B * (R - 1)
    cpu = {"value": rate, "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
           "nproc": os.cpu_count(), "cpu_model": cpu_model(),
           "sample": f"rows {rows} of the batch: {int(lens[rows[0]])}-token prefill + {decode_steps} decode steps each "
                     f"({len(rows) * n_tok} generated tokens, {fed} tokens through the model) in {dt:.1f} s; oracle in "
                     f"float32 mode on weights widened to fp32 beforehand, torch CPU threads as listed",
           "extrapolated": {"full_workload_s": dt * fed_full / fed, "tokens_per_s": B * R / (dt * fed_full / fed),
                            "how": "linear in tokens pushed through the model (prefill and decode tokens alike), so an "
                                   "underestimate of the time: attention over longer contexts is not scaled"}}
    # parity of the GPU path on the sampled rows
    sp = binding.make_sampling(wl.temperature, wl.top_p, wl.sample_seed, wl.greedy, 0)
    tok, lp = ctx.rlhf_gen_prefill(toks.to("cuda:0"), lens.tolist(), sp)
    dl = dlp = 0.0
    agree = total = 0
    for s in range(n_tok):
        lg = ctx.rlhf_gen_get_logits()[rows].cpu().double()
        dl = max(dl, float((lg - ref["logits"][:, s]).abs().max()))
        for ri, b in enumerate(rows):
            total += 1
            if int(tok[b]) == int(ref["tokens"][ri, s]):
                agree += 1
                dlp = max(dlp, abs(float(lp[b]) - float(ref["logprobs"][ri, s])))
        if s + 1 < n_tok:
            forced = tok.clone()
            forced[rows] = ref["tokens"][:, s].to(torch.int32).to(forced.device)
            tok, lp = ctx.rlhf_gen_decode_step(forced)
    ctx.synchronize()
    parity = {"rows": rows, "steps": n_tok, "max_dlogit": dl, "max_dlogprob": dlp, "tokens_equal": f"{agree}/{total}",
              "tolerance": {"dlogit": 3e-2 if wl.dtype == "bf16" else 1e-4, "dlogprob": 2e-2 if wl.dtype == "bf16" else 1e-4},
              "logits_compared": len(rows) * n_tok * wl.shape.vocab}
    parity["ok"] = bool(dl <= parity["tolerance"]["dlogit"] and dlp <= parity["tolerance"]["dlogprob"])
    return cpu, parity


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="7b_b64")
    ap.add_argument("--layers", type=int, default=0, help="override the depth (debugging only; invalidates the metric)")
    ap.add_argument("--resp-len", type=int, default=0, help="override R (debugging only; invalidates the metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-score", action="store_true")
    ap.add_argument("--micro-batch", type=int, default=16, help="rows per micro-batch of the streaming leg (0 = skip)")
    ap.add_argument("--profile-every", type=int, default=64)
    ap.add_argument("--flags", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the rollout shards by query across replicas with no "
              "communication); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2312_11819_amd import binding, synth

    binding.lib()  # fail loudly if the HIP library is missing
    wl = synth.WORKLOADS[args.workload]
    shape = wl.shape if not args.layers else synth.with_layers(wl.shape, args.layers)
    R = args.resp_len or wl.resp_len
    dev = torch.device("cuda:0")
    w = synth.make_weights(shape, wl.weight_seed, wl.dtype, dev)
    toks, lens = synth.workload_queries(wl)
    toks_d = toks.to(dev)
    B = wl.batch
    ctx = binding.Context(w, shape, wl.dtype, B, int(lens.max()) + R, flags=args.flags)
    sp = binding.make_sampling(wl.temperature, wl.top_p, wl.sample_seed, wl.greedy, 0)
    out_t = torch.empty(B, R, dtype=torch.int32, device=dev)
    out_lp = torch.empty(B, R, dtype=torch.float32, device=dev)

    for _ in range(args.warmup):
        ctx.rlhf_gen_generate(toks_d, lens.tolist(), R, sp, out_t, out_lp)
    first = (out_t.clone(), out_lp.clone()) if args.warmup > 0 else None   # same inputs and seed: must repeat exactly
    ctx.rlhf_gen_set_profile(args.profile_every)
    torch.cuda.synchronize()
    pre_ms = dec_ms = 0.0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ctx.rlhf_gen_generate(toks_d, lens.tolist(), R, sp, out_t, out_lp)
        a, b, nsteps = ctx.rlhf_gen_last_timing()
        pre_ms += a
        dec_ms += b
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prof = ctx.rlhf_gen_get_profile()
    step_ms = ctx.rlhf_gen_last_step_ms()
    ctx.rlhf_gen_set_profile(0)
    assert bool(torch.isfinite(out_lp).all()) and int(out_t.min()) >= 0 and int(out_t.max()) < shape.vocab
    repeatable = None if first is None else bool(torch.equal(first[0], out_t) and torch.equal(first[1], out_lp))

    K = args.steps
    ms_per_step = wall / K * 1e3
    tokens_per_s = B * R / (wall / K)
    pre_ms /= K
    dec_ms /= K
    # algorithmic bytes of the decode steps: weights once per step + every cached K/V byte once per step + the appended K/V
    kv_tok = 2 * shape.n_kv_heads * shape.head_dim * 2 * shape.n_layers
    lsum = int(lens.sum())
    wb = weight_bytes(shape)
    dec_bytes = 0
    for t in range(1, R):
        ctx_tokens = lsum + B * t          # cached tokens the step reads, its own included
        dec_bytes += wb + ctx_tokens * kv_tok + B * kv_tok
    dec_frac = dec_bytes / (dec_ms * 1e-3) / HBM_PEAK if dec_ms > 0 else None
    # the same per step: every step's own context lengths against its own time (steps that were run kernel by kernel
    # for the per-kernel timing carry the event overhead and are left out)
    step_fracs = []
    every = args.profile_every
    for t, ms in enumerate(step_ms, start=1):
        if ms > 0 and not (every > 0 and t % every == 0):
            step_fracs.append((wb + (lsum + B * t) * kv_tok + B * kv_tok) / (ms * 1e-3) / HBM_PEAK)
    # prefill flops: projections over all query tokens + causal attention + LM head on B rows
    layer_mm = (shape.qkv_rows * shape.d_model + shape.d_model * shape.n_heads * shape.head_dim
                + 3 * shape.d_ffn * shape.d_model)
    pre_flop = 2 * layer_mm * shape.n_layers * lsum + 2 * B * shape.vocab * shape.d_model
    pre_flop_attn = sum(2 * int(l) * int(l) * shape.n_heads * shape.head_dim * shape.n_layers for l in lens)
    pre_frac = (pre_flop + pre_flop_attn) / (pre_ms * 1e-3) / MFMA_BF16_PEAK if pre_ms > 0 else None
    # a decode step's projections as a fraction of the MFMA peak (matters at B = 256, where 2 B flop per 2-byte
    # weight is near the ridge point)
    dec_flop_step = 2 * B * (layer_mm * shape.n_layers + shape.vocab * shape.d_model)
    dec_mfma_frac = dec_flop_step * max(R - 1, 1) / (dec_ms * 1e-3) / MFMA_BF16_PEAK if dec_ms > 0 else None

    roofline = None
    kernels = {}
    if prof["steps"] > 0:
        hq = shape.n_heads * shape.head_dim
        wbytes = {"gemm_qkv": shape.qkv_rows * shape.d_model * 2, "gemm_wo": shape.d_model * hq * 2,
                  "gemm_gate_up": 2 * shape.d_ffn * shape.d_model * 2, "gemm_down": shape.d_model * shape.d_ffn * 2,
                  "lm_head": shape.vocab * shape.d_model * 2}
        for k in binding.PROF_CLASSES:
            if prof["launches"][k]:
                kernels[k] = {"ms_per_sampled_step": prof["ms"][k] / prof["steps"], "launches": prof["launches"][k],
                              "us_per_launch": prof["ms"][k] / prof["launches"][k] * 1e3}
                if k in wbytes and prof["ms"][k] > 0:   # weight bytes streamed per second by this projection
                    kernels[k]["weight_GBps"] = wbytes[k] * prof["launches"][k] / (prof["ms"][k] * 1e-3) / 1e9
        n_attn = prof["launches"]["attn_decode"]
        attn_bytes = prof["attn_tokens"] * 2 * shape.n_kv_heads * shape.head_dim * 2 * shape.n_layers  # all sampled launches
        attn_s = prof["ms"]["attn_decode"] * 1e-3
        gemm_ms = sum(prof["ms"][k] for k in ("gemm_qkv", "gemm_wo", "gemm_gate_up", "gemm_down", "lm_head"))
        gemm_bytes = prof["steps"] * (wb - (2 * shape.n_layers + 1) * shape.d_model * 2)
        if attn_s >= gemm_ms * 1e-3:
            roofline = {"kernel": "attn_decode_kernel", "bound": "hbm", "achieved": attn_bytes / attn_s / 1e9,
                        "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": attn_bytes / attn_s / HBM_PEAK, "traffic": None,
                        "avg_launch_us": attn_s / n_attn * 1e6, "launches_timed": n_attn,
                        "bytes_per_launch": attn_bytes / n_attn}
        else:
            n_g = sum(prof["launches"][k] for k in ("gemm_qkv", "gemm_wo", "gemm_gate_up", "gemm_down", "lm_head"))
            # (batches of more than 128 rows run the projections as the split-K form of the large-tile GEMM)
            roofline = {"kernel": "gemm_skinny_kernel" if B <= 128 else "gemm_h16_dma_kernel<0, true>", "bound": "hbm", "achieved": gemm_bytes / (gemm_ms * 1e-3) / 1e9,
                        "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": gemm_bytes / (gemm_ms * 1e-3) / HBM_PEAK,
                        "traffic": None, "avg_launch_us": gemm_ms / n_g * 1e3, "launches_timed": n_g,
                        "bytes_per_launch": gemm_bytes / n_g}
        # HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by what the counters read for the
        # weight-conversion copy kernel): measured on a 2-layer, 48-token run of this workload (per-launch traffic does
        # not depend on the depth); the fetched / algorithmic ratio of those launches is applied to this
        # run's launches (profiles/bench_7b_b64_pmc_traffic.md)
        ratios = traffic_ratios(wl.name)
        if ratios is not None:
            pmc = ratios["attn_decode_kernel" if roofline["kernel"].startswith("attn") else "gemm_skinny"]
            roofline["traffic"] = pmc[0] * roofline["bytes_per_launch"] + pmc[1]
            roofline["traffic_source"] = (f"fetched / algorithmic = {pmc[0]:.3f} and {pmc[1] / 1e6:.1f} MB written per launch, from the "
                                          f"rocprofv3 --pmc summary profiles/bench_{wl.name}_pmc_traffic.md (reduced-depth run of this workload)")
        roofline["attn_decode_GBps"] = attn_bytes / attn_s / 1e9 if attn_s > 0 else None
        roofline["gemm_skinny_GBps"] = gemm_bytes / (gemm_ms * 1e-3) / 1e9 if gemm_ms > 0 else None

    # scoring pass over the rollout just produced (Actor.forward of Alg. 1), outside the timed region
    score = None
    if not args.no_score:
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        sc = ctx.rlhf_gen_score(toks_d, lens.tolist(), out_t)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t1
        fed = lsum + B * (R - 1)
        sflop = 2 * layer_mm * shape.n_layers * fed + 2 * B * R * shape.vocab * shape.d_model \
            + sum(2 * (int(l) + R - 1) ** 2 * shape.n_heads * shape.head_dim * shape.n_layers for l in lens)
        score = {"ms": dt * 1e3, "scored_tokens_per_s": B * R / dt, "mfma_bf16_frac": sflop / dt / MFMA_BF16_PEAK,
                 "max_abs_diff_vs_rollout_logprobs": float((sc - out_lp).abs().max())}

    # micro-batched rollout of the same batch (the pipelining of Sec. IV-A), outside the timed region: when is the first
    # micro-batch available to the next stage, and what does the smaller decode batch cost in throughput
    micro = None
    if args.micro_batch > 0 and not args.no_score and args.micro_batch < B:
        ready = []
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        mt, mlp, _ = ctx.rlhf_gen_generate_stream(toks_d, lens.tolist(), R, sp, args.micro_batch,
                                                  lambda i, r0, n, ev: ready.append(time.perf_counter() - t1))
        ctx.synchronize()
        dt = time.perf_counter() - t1
        micro = {"micro_batch": args.micro_batch, "ms": dt * 1e3, "tokens_per_s": B * R / dt,
                 "first_micro_batch_ready_ms": ready[0] * 1e3, "ready_ms": [r * 1e3 for r in ready],
                 "equals_whole_batch_rollout": bool(torch.equal(mt, out_t) and torch.equal(mlp, out_lp))}

    # the same micro-batches inside one decode loop (continuous batching): they are admitted `stagger` decode steps apart and
    # complete that far apart, sharing every step's weight stream
    cont = None
    if args.micro_batch > 0 and not args.no_score and args.micro_batch < B:
        cont = []
        for stagger in (0, 32):
            torch.cuda.synchronize()
            ev0 = torch.cuda.Event(enable_timing=True)
            with torch.cuda.stream(ctx.stream):
                ev0.record()
            t1 = time.perf_counter()
            mt, mlp, evs = ctx.rlhf_gen_generate_continuous(toks_d, lens.tolist(), R, sp, args.micro_batch, stagger)
            ctx.synchronize()
            dt = time.perf_counter() - t1
            cont.append({"micro_batch": args.micro_batch, "stagger_steps": stagger, "ms": dt * 1e3, "tokens_per_s": B * R / dt,
                         "decode_steps": ctx.rlhf_gen_last_timing()[2], "peak_rows": ctx.rlhf_gen_last_peak_rows(),
                         "ready_ms": [ev0.elapsed_time(e) for e in evs],
                         "equals_whole_batch_rollout": bool(torch.equal(mt, out_t) and torch.equal(mlp, out_lp))})

    # weight refresh of the shadow Actor (the parameter synchronisation of Alg. 2), outside the timed region:
    # every projection matrix and the LM head is read as bf16 and rewritten as fp16
    refresh = None
    if wl.dtype == "bf16" and not args.no_score and not (args.flags & 8):   # in place, the sources no longer hold bf16
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ctx.rlhf_gen_update_weights(ctx._weights)
        ctx.synchronize()
        dt = time.perf_counter() - t1
        moved = 2 * (wb - (2 * shape.n_layers + 1) * shape.d_model * 2)
        refresh = {"ms": dt * 1e3, "GBps_read_plus_write": moved / dt / 1e9}

    probes = gemm_shapes = None
    if wl.dtype == "bf16" and not args.no_score:
        probes = hardware_probes(binding, dev)
        gemm_shapes = prefill_gemm_shapes(binding, shape, min(16384, lsum), dev, lo4=not (args.flags & 32))
        if roofline is not None:   # the same achieved rate against what a bare read-only stream sustains on this card
            roofline["measured_peak"] = probes["hbm_read_nontemporal_GBps"]
            roofline["frac_of_measured_peak"] = roofline["achieved"] / probes["hbm_read_nontemporal_GBps"]

    cpu = parity = None
    if not args.no_cpu_baseline and not (args.flags & 8):   # (converted in place, the caller's buffers no longer hold bf16)
        rows = sorted({0, B // 2})
        cpu, parity = cpu_baseline_and_parity(binding, ctx, wl if not args.layers else synth.dataclasses.replace(wl, shape=shape),
                                              w, toks, lens, rows)

    line = {
        "metric": "generated tokens/sec + % HBM roofline per decode step, 7B-shape bf16 B=64",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "layers": shape.n_layers, "d_model": shape.d_model, "batch": B,
                   "query_len": [wl.len_lo, wl.len_hi], "resp_len": R, "temperature": wl.temperature, "top_p": wl.top_p,
                   "kv_block": 16,
                   "weights": ("bf16 at the boundary; fp16 MFMA operands (exact conversion), fp32 accumulation; four activation tensors as fp16 pairs hi + lo"
                               + ("" if args.flags & 32 else ", the low halves of two of them contracted in 4-bit (e2m1, block-scaled MFMA) in prefill")) if wl.dtype == "bf16" else "fp32",
                   # the configuration is the named one, and this run's own output was checked against the oracle
                   "valid": bool(not args.layers and not args.resp_len and (parity is None or parity["ok"])),
                   "checked_against_oracle": parity is not None,
                   "rollouts_bit_identical": repeatable},
        "decode": {"ms_per_decode_step": dec_ms / max(R - 1, 1), "tokens_per_s_decode_only": B * (R - 1) / (dec_ms * 1e-3) if dec_ms else None,
                   "hbm_roofline_frac_per_decode_step": dec_frac, "mfma_bf16_frac_per_decode_step": dec_mfma_frac,
                   "gemm_TFLOP_per_step": dec_flop_step / 1e12, "algorithmic_GB_per_step_mean": dec_bytes / max(R - 1, 1) / 1e9,
                   "hbm_roofline_frac_step_min": min(step_fracs) if step_fracs else None,
                   "hbm_roofline_frac_step_max": max(step_fracs) if step_fracs else None,
                   "hbm_roofline_frac_step_mean": sum(step_fracs) / len(step_fracs) if step_fracs else None},
        "prefill": {"ms": pre_ms, "mfma_bf16_frac": pre_frac, "flop": pre_flop + pre_flop_attn},
        "roofline": roofline,
        "kernels_sampled": kernels,
        "score_pass": score,
        "micro_batched": micro,
        "micro_batched_continuous": cont,
        "prefill_gemm_shapes": gemm_shapes,
        "measured_peaks": probes,
        "weight_refresh": refresh,
        "cpu_baseline": cpu,
        "parity_vs_oracle": parity,
    }
    print(json.dumps(line))
    ctx.rlhf_gen_destroy()
    return 0


if __name__ == "__main__":
    sys.exit(main())
