/*
 * Single-operation entry points of librlhf_gen: each runs one kernel of the rollout's hot path on
 * caller-provided device buffers, so that a test can compare that kernel alone with a CPU definition.
 * They are the steps inside one Actor.generate call (Alg. 1): the projections, the rotary embedding
 * and KV-cache append, attention over the paged cache, and the sampler.  All pointers are DEVICE
 * pointers unless marked host; all calls enqueue on `stream` (hipStream_t, NULL = default) and
 * return without synchronising.  Return values are rlhf_gen_status codes.
 */
#ifndef RLHF_GEN_OPS_H
#define RLHF_GEN_OPS_H

#include <stdint.h>

#include "rlhf_gen.h"

#ifdef __cplusplus
extern "C" {
#endif

enum { RLHF_GEN_GEMM_TILED = 0, RLHF_GEN_GEMM_STREAMING = 1, RLHF_GEN_GEMM_FP32 = 2 };
/* epilogues of the tiled GEMM */
enum { RLHF_GEN_EPI_STORE_F32 = 0, RLHF_GEN_EPI_RESID_F32 = 1, RLHF_GEN_EPI_SWIGLU = 2, RLHF_GEN_EPI_STORE_H16 = 3 };

/* Hardware probes for the benchmark's roofline report (Sec. III-B names generation, a memory-bound stage, as the
 * bottleneck: the report quotes the kernels against what the card sustains as well as against datasheet peaks).
 * stream_read: one read-only pass over buf (bytes rounded down to a multiple of 8192) with 16-byte loads, plain or
 * nontemporal; nothing is written unless a checksum hits one value in 2^32 (scratch: 1 KB device buffer).
 * mfma_loop: workgroups * 4 wavefronts each issue 8 * iters v_mfma_f32_32x32x16_f16 (32768 flop each) on operand
 * registers filled from `operands` (device, 16 KB of fp16 values); no memory traffic inside the loop. */
int rlhf_gen_op_probe_stream_read(void* stream, const void* buf, int64_t bytes, int32_t nontemporal, void* scratch);
int rlhf_gen_op_probe_mfma_loop(void* stream, const void* operands, int32_t workgroups, int32_t iters, void* scratch);

/* Re-order an fp16 weight matrix W [N, K] (row-major) into the library's working layout, which the 16-bit GEMMs below
 * expect (rlhf_gen_init does the same to the Actor's matrices while converting them from bf16): tiles of 16 rows x
 * 128 columns, 4 KB each, inside a tile the halves in the order [k/32 % 4][row % 16][k % 32]; the tiles are stored
 * in slabs of 256 rows (the last slab may be shorter), slab after slab, and inside a slab in the order
 * [k/128][row/16 within the slab].  N % 16 == 0, K % 128 == 0; the two buffers must not overlap. */
int rlhf_gen_op_tile_weights(void* stream, const void* w_rowmajor, void* w_tiled, int32_t N, int32_t K);

/* out = A[M,K] * W[N,K]^T (the projections of a decoder layer, y = x W^T).
 * 16-bit operands are IEEE fp16 (the library's working format; bf16 weights are converted at init); for the TILED and
 * STREAMING kinds W must be in the working layout made by rlhf_gen_op_tile_weights (A is plain row-major).
 *   TILED     fp16 A and W; epilogue selects out: fp32 [M,N] store, fp32 [M,N] accumulate, fp16 [M,N] store, or
 *             SWIGLU where W is [2N, K] (gate rows then up rows) and out is fp16 [M,N] = silu(gate) * up.
 *             N % 256 == 0 (N % 128 for SWIGLU), K % 128 == 0.  With epilogue STORE_F32 and nsplit > 1: split-K
 *             form for a few hundred rows, out is fp32 [nsplit, M, N] partial sums as for STREAMING; nsplit must
 *             leave no split empty (ceil(K/32 / ceil(K/32 / nsplit)) == nsplit), else UNSUPPORTED.
 *   STREAMING fp16 A and W, M <= 256, N % 64 == 0, K % 128 == 0; out is fp32 [nsplit, M, N] partial sums whose
 *             sum over the first axis is the product.  nsplit in [1, K/128].  With epilogue SWIGLU instead: W is
 *             [2N, K] (gate rows then up rows), N % 32 == 0, no split, out is fp16 [M, N] = silu(gate) * up.
 *   FP32      fp32 A, W, out; epilogue STORE_F32 or RESID_F32.
 * a_pairs != 0 (TILED, and STREAMING up to 128 rows without SWIGLU): A is [M, 2K], each row the fp16 pair
 * [hi (K) | lo (K)] of a higher-precision activation, and out = (hi + lo) W^T. */
int rlhf_gen_op_gemm(void* stream, int kind, const void* A, const void* W, void* out, int32_t M, int32_t N, int32_t K,
                     int32_t epilogue, int32_t nsplit, int32_t a_pairs);

/* The prefill form of the two projections whose input travels as a pair hi + lo (the QKV and the output projection:
 * x W^T of a decoder layer with x carried beyond fp16 precision).  The low half is 2^-11 of the value it corrects, so
 * its product with W is taken in a 4-bit side format by the block-scaled MFMA, at a quarter of the cost of a second
 * fp16 pass: elements are e2m1 (sign; magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6), two per byte with the even k in the low
 * nibble; a group shares a power-of-two scale 2^(byte - 127), the smallest that brings the group's largest magnitude
 * to at most 6.
 *   tile_weights4: w_tiled [N, K] fp16 in the working layout -> w4 (N K / 2 bytes: the working layout of a matrix with
 *                  K / 4 16-bit columns, each holding four consecutive k) and w_scale [N] bytes, one group per row.
 *                  N % 16 == 0, K % 512 == 0.
 *   rmsnorm_lo4:   y = rmsnorm(x) * gain for x fp32 [M, d], gain bf16 [d], in the form the GEMM reads: row m of y
 *                  (pitch 4 d bytes) = [hi: d fp16 | lo4: d / 2 bytes | unused]; one scale byte per (row, 128 columns)
 *                  at row_scale[((t G + m / 128) 32 + m % 32) 4 + (m / 32) % 4] for column group t, with G =
 *                  scale_groups >= ceil(M / 128) (row_scale holds (d / 128) G 128 bytes).  d % 128 == 0, d <= 8192.
 *   gemm_lo4:      out fp32 [M, N] (=, or += with RESID_F32) hi W^T + lo4 W4^T for A in that row form.  N % 256 == 0,
 *                  K % 512 == 0, scale_groups >= 2 ceil(M / 256); bytes of row_scale that belong to rows >= M must
 *                  not be 255 (the format's NaN).
 * All pointers device memory.  Errors: INVALID, UNSUPPORTED (shape), DEVICE. */
int rlhf_gen_op_tile_weights4(void* stream, const void* w_tiled, void* w4, void* w_scale, int32_t N, int32_t K);
int rlhf_gen_op_rmsnorm_lo4(void* stream, const float* x, const void* gain_bf16, void* y, void* row_scale, int32_t scale_groups,
                            int32_t M, int32_t d, float eps);
int rlhf_gen_op_gemm_lo4(void* stream, const void* A, const void* W, const void* W4, const void* w_scale, const void* a_scale,
                         int32_t scale_groups, float* out, int32_t M, int32_t N, int32_t K, int32_t epilogue);

/* For callers that cannot allocate device memory (code under HIP graph capture, serving loops and harnesses that forbid
 * hipMalloc): the STREAMING product out = A W^T of rlhf_gen_op_gemm with its split-K partial sums summed inside the
 * library.  rlhf_gen_op_gemm(STREAMING) needs a caller-provided fp32 [nsplit, M, N] buffer for the partial sums; here they
 * go to a workspace of 32 MiB that is part of the library's device image (each GPU the library runs on holds it until
 * the process ends), and the call allocates nothing - no hipMalloc, no hipFree, no allocating library routine.
 *   A fp16 [M, K] (a_pairs != 0: [M, 2K] hi | lo pairs), W fp16 [N, K] in the working layout, out fp32 [M, N] (written
 *   completely); M <= 256 (128 with a_pairs), N % 64 == 0, K % 128 == 0, else UNSUPPORTED.  The split count is the one
 *   the rollout uses for this weight shape; *nsplit_out (host, may be NULL) receives it.  The planes are added in
 *   ascending order, as the rollout's consumer kernels add them.
 * Errors: E_INVALID if nsplit * M * N * 4 bytes exceed the 32 MiB workspace (message via rlhf_gen_last_error(NULL)).
 * Every call on a GPU uses that GPU's one workspace: calls that overlap in time on the same GPU (different streams or
 * threads) race and must be serialised by the caller.  The workspace keeps the previous call's contents; nothing in it
 * has to start at zero, since every element the summation reads is written by the same call first. */
int rlhf_gen_op_gemm_static(void* stream, const void* A, const void* W, float* out, int32_t M, int32_t N, int32_t K,
                            int32_t a_pairs, int32_t* nsplit_out);

/* Rotate q and k of fp32 qkv rows [M, (Hq + 2 Hkv) head_dim] by their positions and append k, v to the paged
 * cache.  row_pos [M] position of each row; row_seq [M] batch row (NULL = identity); cos_t / sin_t
 * [positions, head_dim/2] fp32 tables; block_table int32 [batch, max_blocks]; kv_pool = one layer's pool
 * ([Hkv, n_blocks, 8192] bytes of fp16 in 16-bit mode, [Hkv, n_blocks, 2, 16, head_dim] floats in fp32 mode);
 * q_out: half16 != 0: fp16 [M, Hq, 2, head_dim], the pair [hi | lo] of each rotated query head; else fp32
 * [M, Hq, head_dim]. */
int rlhf_gen_op_rope_append(void* stream, const float* qkv, const int32_t* row_pos, const int32_t* row_seq,
                            const float* cos_t, const float* sin_t, void* q_out, void* kv_pool,
                            const int32_t* block_table, int32_t max_blocks, int32_t n_blocks, int32_t M, int32_t Hq,
                            int32_t Hkv, int32_t head_dim, int32_t half16);

/* One query row per (sequence, query head) against the seq_len[b] + 1 newest-inclusive cached tokens (fp16 cache,
 * head_dim 128).  q fp16 [B, Hq, 2, 128] (hi | lo pairs), out fp16 [B, 2, Hq * 128] (hi block, then lo block). */
int rlhf_gen_op_attn_decode(void* stream, const void* q, const void* kv_pool, const int32_t* block_table,
                            int32_t max_blocks, int32_t n_blocks, const int32_t* seq_len, void* out, int32_t B, int32_t Hq,
                            int32_t Hkv);

/* Causal attention of packed query rows over the cache their own keys were appended to.  cu_seqlens [nseq + 1]
 * row offsets, seq_ids [nseq] batch rows (block-table rows), q [rows, Hq, 2, 128] and out [rows, 2, Hq * 128] fp16 pairs
 * as in the decode call, max_len = longest sequence. */
int rlhf_gen_op_attn_prefill(void* stream, const void* q, const void* kv_pool, const int32_t* block_table,
                             int32_t max_blocks, int32_t n_blocks, const int32_t* cu_seqlens, const int32_t* seq_ids, void* out,
                             int32_t nseq, int32_t max_len, int32_t Hq, int32_t Hkv);

/* The two attention calls with the low halves of out in the 4-bit side format of rlhf_gen_op_gemm_lo4 (the input form
 * of the output projection in prefill and in decode batches above 128 rows): row m of out (pitch 4 Hq 128 bytes) =
 * [hi: Hq 128 fp16 | lo4: Hq 64 bytes | unused], one scale byte per (row, head) in row_scale at the position
 * rlhf_gen_op_rmsnorm_lo4 documents (column group = head).  128 scale_groups must cover the rows. */
int rlhf_gen_op_attn_decode_lo4(void* stream, const void* q, const void* kv_pool, const int32_t* block_table,
                                int32_t max_blocks, int32_t n_blocks, const int32_t* seq_len, void* out, void* row_scale,
                                int32_t scale_groups, int32_t B, int32_t Hq, int32_t Hkv);
int rlhf_gen_op_attn_prefill_lo4(void* stream, const void* q, const void* kv_pool, const int32_t* block_table,
                                 int32_t max_blocks, int32_t n_blocks, const int32_t* cu_seqlens, const int32_t* seq_ids, void* out,
                                 void* row_scale, int32_t scale_groups, int32_t nseq, int32_t max_len, int32_t Hq, int32_t Hkv);

/* Sampler on fp32 logits [B, V]: token and log-prob per row for response index *step (device int32).
 * sp is a host struct.  scratch_tok: device int32 [B] (receives a copy of the tokens). */
int rlhf_gen_op_sample(void* stream, const float* logits, int32_t B, int32_t V, const rlhf_gen_sampling* sp,
                       const int32_t* step, int32_t* tok_out, float* logprob_out, int32_t* scratch_tok);

#ifdef __cplusplus
}
#endif
#endif /* RLHF_GEN_OPS_H */
