/*
 * rlhf_gen - one GPU's share of the RLHF generation stage on MI355X (gfx950).
 *
 * The operation is `Response <- Actor.generate(Query)` of the paper's Alg. 1 and
 * `ShadowActor.generate(Query)` of Alg. 2: a batched autoregressive rollout of a
 * Llama-style Actor (Sec. V-A, "LLM Backbones") that emits exactly R response tokens
 * per query (Sec. V-A, "Hyperparameters": minimum = maximum generation length) plus the
 * log-probability of every emitted token, which PPO consumes (Sec. II, the RLHF pipeline).
 * The paper names this stage as the bottleneck of a step (Sec. III-B).
 *
 * Plain C ABI: no exceptions, no C++ or framework types.  Every call returns an
 * rlhf_gen_status; a negative value means nothing useful was produced and
 * rlhf_gen_last_error() describes why.  A context is not thread-safe.
 *
 * Memory conventions
 *   "device" pointers are HIP device allocations on cfg.device, owned by the caller,
 *   row-major.  "host" pointers are ordinary process memory.  Weight matrices are
 *   [out_features, in_features] (y = x W^T), stored as cfg.dtype, BORROWED for the
 *   context's lifetime and never written (unless RLHF_GEN_FLAG_CONVERT_IN_PLACE is set).  The library owns the paged KV cache, block
 *   tables, activations and counters; all of it is allocated in rlhf_gen_init and
 *   nothing is allocated afterwards.
 *   Work is enqueued on cfg.stream.  prefill and decode_step return after enqueueing
 *   (prefill synchronises once at entry to validate the token ids); generate
 *   synchronises the stream before returning.
 */
#ifndef RLHF_GEN_H
#define RLHF_GEN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rlhf_gen_ctx rlhf_gen_ctx; /* opaque */

typedef enum {
  RLHF_GEN_OK = 0,
  RLHF_GEN_E_INVALID = -1,     /* bad argument: NULL, shape, token id out of range */
  RLHF_GEN_E_NOMEM = -2,       /* KV pool or device memory cannot hold the request */
  RLHF_GEN_E_STATE = -3,       /* call order: decode before prefill, past max_seq */
  RLHF_GEN_E_DEVICE = -4,      /* a HIP call failed */
  RLHF_GEN_E_UNSUPPORTED = -5  /* a shape the kernels do not cover */
} rlhf_gen_status;

enum { RLHF_GEN_DTYPE_FP32 = 0, RLHF_GEN_DTYPE_BF16 = 1 };

/* cfg.flags */
enum {
  RLHF_GEN_FLAG_SHUFFLE_BLOCKS = 1u, /* hand out KV blocks in a scrambled order (tests: results must not depend on placement) */
  RLHF_GEN_FLAG_NO_GRAPH = 2u,       /* generate launches every decode step kernel by kernel instead of replaying a captured graph */
  RLHF_GEN_FLAG_GENERIC_GEMM = 4u,   /* decode uses the large-tile GEMM instead of the weight-streaming one (cross-check) */
  RLHF_GEN_FLAG_FUSED_ROPE = 16u,    /* decode folds RoPE + KV append into the attention kernel (one launch fewer per layer;
                                        measured 2 % slower per step on MI355X at the 7B shape, so it is off by default) */
  RLHF_GEN_FLAG_CONVERT_IN_PLACE = 8u, /* bf16 mode: rewrite the caller's projection matrices and LM head in place into
                                         the fp16 working format (tiled layout) instead of allocating working copies
                                         (for models that fill the card; the buffers then no longer hold row-major
                                         bf16 and must not be reused as such); costs a 1024-row staging buffer */
  RLHF_GEN_FLAG_PREFILL_FP16_PAIRS = 32u /* bf16 mode: prefill and scoring contract the low halves of the QKV and output
                                         projections' inputs in fp16, as decode does, instead of the 4-bit side format
                                         (a second pass at full cost instead of a quarter; no 4-bit copies of those two
                                         matrices, which take 1/4 of their fp16 size; cross-check) */
};

/* Model and capacity description.  Architecture: pre-norm decoder, RMSNorm (eps inside the
 * square root), rotary embedding with half-split pairing (dimension i pairs with i + head_dim/2,
 * angle pos * rope_theta^(-2i/head_dim)), causal attention scaled by 1/sqrt(head_dim) where
 * query head j reads KV head j / (n_heads / n_kv_heads), SwiGLU MLP, no biases, untied LM head. */
typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_theta;
  int32_t dtype;          /* RLHF_GEN_DTYPE_*: storage type of the caller's weights.  bf16: the projection matrices are
                             converted once to fp16 working copies in a tiled layout (exact unless |w| < 2^-17), every MFMA operand,
                             activation and the KV cache is fp16 (bf16's 8 significant bits cannot meet the parity
                             tolerance over 32 layers), accumulation / residual / softmax / logits are fp32.  Four
                             activation tensors (the inputs of the QKV and output projections, the rotated queries, the
                             attention probabilities) travel as fp16 pairs hi + lo; where d_model and n_heads * head_dim
                             are multiples of 512, prefill and scoring contract the low halves of the two projection
                             inputs in a 4-bit format against 4-bit copies of wqkv and wo made at init (a quarter of
                             their fp16 size; RLHF_GEN_FLAG_PREFILL_FP16_PAIRS turns that off).  Like any
                             fp16 inference it assumes activations within +-65504 (they saturate there).  fp32 is a
                             plain-ALU path meant for small models */
  int32_t max_batch;      /* largest B any call will pass */
  int32_t max_seq;        /* most tokens one sequence holds in the cache: query length + response length - 1 (the last
                             token drawn is not fed back) */
  int32_t kv_block;       /* tokens per KV page; must be 16 */
  int32_t kv_pool_blocks; /* pages in the pool (shared by all sequences, one set per layer);
                             0 = max_batch * ceil(max_seq / kv_block) */
  int32_t device;         /* HIP device ordinal */
  void* stream;           /* hipStream_t, borrowed; NULL = the default stream */
  uint32_t flags;
} rlhf_gen_cfg;

/* Device pointers.  The per-layer members are HOST arrays of n_layers DEVICE pointers. */
typedef struct {
  const void* tok_emb;           /* [vocab, d_model] */
  const void* lm_head;           /* [vocab, d_model] */
  const void* final_norm;        /* [d_model] */
  const void* const* attn_norm;  /* each [d_model] */
  const void* const* wqkv;       /* each [(n_heads + 2 n_kv_heads) head_dim, d_model]: q rows, k rows, v rows */
  const void* const* wo;         /* each [d_model, n_heads head_dim] */
  const void* const* ffn_norm;   /* each [d_model] */
  const void* const* w_gate_up;  /* each [2 d_ffn, d_model]: gate rows, then up rows */
  const void* const* w_down;     /* each [d_model, d_ffn] */
} rlhf_gen_weights;

/* Sampling rule for one rollout.  The paper states none, so it is a parameter.
 * greedy != 0: argmax, lowest index on exact ties.  Otherwise z = logits / temperature,
 * p = softmax(z), nucleus = shortest prefix of the tokens ordered by (p descending, index
 * ascending) whose mass reaches top_p (top_p >= 1 keeps everything), p' = p renormalised on the
 * nucleus, token = first nucleus member in ascending index order whose running p' sum exceeds u.
 * u in [0,1) has 24 bits: u = (mix(seed ^ b*0x9E3779B97F4A7C15 ^ t*0xBF58476D1CE4E5B9) >> 40) / 2^24
 * with mix = the splitmix64 output function applied to its argument + 0x9E3779B97F4A7C15,
 * b the batch row and t the response index.
 * logprob_mode 0: log softmax(logits)[token] of the raw model distribution (what a later
 * Actor.forward over query+response returns, Alg. 1); 1: log p'[token]. */
typedef struct {
  float temperature;
  float top_p;
  uint64_t seed;
  int32_t greedy;
  int32_t logprob_mode;
} rlhf_gen_sampling;

/* Create a context for one Actor replica.  Validates cfg, allocates every buffer, zeroes the KV
 * pool.  weights/cfg are host structs; *out receives the context (NULL on failure, in which case
 * rlhf_gen_last_error(NULL) holds the reason).  Sec. V-A fixes only "Llama" and the lengths; the
 * architecture details are those listed at rlhf_gen_cfg. */
int rlhf_gen_init(const rlhf_gen_weights* weights, const rlhf_gen_cfg* cfg, rlhf_gen_ctx** out);

/* Prefill: run the Actor over B right-padded queries, fill the KV cache, and draw response token 0
 * of every sequence from the logits at its last query position (Alg. 1, the first step of
 * Actor.generate).  Replaces any previous batch held by the context.
 *   query_tokens  device int32 [B, Lmax]; row b holds lengths[b] token ids, then padding that is never read
 *   lengths       HOST int32 [B]; 1 <= lengths[b] <= min(Lmax, max_seq)
 *   sampling      host struct, copied; stays in force for the following decode steps
 *   tok_out       device int32 [B]; logprob_out device float [B]
 * Errors: E_INVALID (NULL, B or lengths out of range, a token id outside [0, vocab)),
 * E_NOMEM (KV pool too small). */
int rlhf_gen_prefill(rlhf_gen_ctx* ctx, const int32_t* query_tokens, const int32_t* lengths, int32_t B,
                     int32_t Lmax, const rlhf_gen_sampling* sampling, int32_t* tok_out, float* logprob_out);

/* One KV-cached decode step for the current batch: feed each sequence one token (the one drawn by
 * the previous call, or forced_tokens[b] if forced_tokens is not NULL - teacher forcing), append
 * its key/value to the cache, and draw the next response token and its log-prob.
 *   forced_tokens device int32 [B] or NULL
 *   tok_out       device int32 [B]; logprob_out device float [B]
 * The call does not wait for the device, so it cannot refuse a forced id outside [0, vocab) itself: the step runs with
 * the nearest valid id, the kernel raises a flag, and the mistake is reported as E_INVALID by the next
 * rlhf_gen_decode_step that finds the step completed (always, if the stream was synchronised in between) or by the next
 * rlhf_gen_get_logits, whichever comes first; the flag is then cleared.
 * Errors: E_STATE (no prefill yet, or a sequence would exceed max_seq), E_NOMEM (pool exhausted), E_INVALID (deferred,
 * see above). */
int rlhf_gen_decode_step(rlhf_gen_ctx* ctx, const int32_t* forced_tokens, int32_t* tok_out, float* logprob_out);

/* Whole rollout = prefill + (max_resp_len - 1) decode steps; every sequence gets exactly
 * max_resp_len tokens (no end-of-sequence stop; Sec. V-A).  Reserves all KV pages up front and
 * fails with E_NOMEM before computing if they do not fit.  Synchronises the stream before returning.
 *   resp_tokens   device int32 [B, max_resp_len]; resp_logprobs device float [B, max_resp_len] */
int rlhf_gen_generate(rlhf_gen_ctx* ctx, const int32_t* query_tokens, const int32_t* lengths, int32_t B,
                      int32_t Lmax, int32_t max_resp_len, const rlhf_gen_sampling* sampling,
                      int32_t* resp_tokens, float* resp_logprobs);

/* Micro-batched rollout.  The paper hides the hand-off between stages by micro-batching: the forward stage (and the
 * transfer that feeds it) of one micro-batch starts when its generation ends, not when the whole batch has been
 * generated, and the transfers run on a stream of their own beside the computation (Sec. IV-A: the Interleaving
 * strategy puts communication and computation on separate streams, the Disaggregated strategy pipelines micro-batches
 * to hide the idle time of the hand-off; Sec. IV-C, third recommendation of the second guideline).  This call generates rows [0, B) in micro-batches of micro_batch rows, one after
 * the other on cfg.stream, and tells the caller when each is finished:
 *   - after micro-batch i (rows row0 = i * micro_batch .. row0 + rows) is complete, done_events[i] (a hipEvent_t the
 *     caller created; done_events is a HOST array of ceil(B / micro_batch) entries, or NULL) is recorded on cfg.stream;
 *   - then on_ready(user, i, row0, rows, done_events[i]) (or NULL) is called on the calling thread, before micro-batch
 *     i + 1 is enqueued: work the callback enqueues on another stream behind hipStreamWaitEvent(stream, event) - a copy
 *     of the finished rows to the host or to a peer, a scoring pass on another context - overlaps with the generation of
 *     the following micro-batches.
 * Row b draws the same random numbers as in rlhf_gen_generate over the whole batch, and the kernels accumulate every
 * output element in an order that does not depend on the number of rows up to 128 rows per call (larger decode
 * batches take a tile GEMM with another summation order), so for B <= 128 the result equals rlhf_gen_generate's bit
 * for bit; for larger B it equals it within the rounding differences of the two GEMMs.  Only min(micro_batch, B) <= cfg.max_batch is required (the KV pool is reused by each
 * micro-batch), so a context can be sized for the micro-batch.  rlhf_gen_last_timing reports the sums over the
 * micro-batches.  Other arguments and errors as for rlhf_gen_generate; on an error the remaining micro-batches are
 * not generated. */
typedef void (*rlhf_gen_microbatch_fn)(void* user, int32_t index, int32_t row0, int32_t rows, void* done_event);
int rlhf_gen_generate_stream(rlhf_gen_ctx* ctx, const int32_t* query_tokens, const int32_t* lengths, int32_t B,
                             int32_t Lmax, int32_t max_resp_len, const rlhf_gen_sampling* sampling, int32_t* resp_tokens,
                             float* resp_logprobs, int32_t micro_batch, void* const* done_events,
                             rlhf_gen_microbatch_fn on_ready, void* user);

/* Micro-batched rollout inside ONE decode loop (continuous batching).  rlhf_gen_generate_stream generates its
 * micro-batches one after the other, so every micro-batch streams all the weights again at every step: at 16 rows per
 * micro-batch the whole batch takes twice as long as in one piece.  Here the micro-batches share the decode steps: rows
 * join the running batch a micro-batch at a time and leave it when they have their R tokens (exactly R per row, Sec. V-A),
 * so a decode step carries rows at different response indices and the weights are streamed once per step for all of
 * them.  Micro-batch i (rows i * micro_batch ...) is prefilled and admitted once stagger_steps decode steps have passed
 * since the previous admission (0: all at the start, which is rlhf_gen_generate with per-micro-batch completion events)
 * AND the KV pool has free pages for all of its rows to the end of their responses; until then the running rows keep
 * decoding and admission resumes when finished rows hand their pages back.  That second condition is the paper's rule
 * for sizing a run - the batch is what memory allows (Sec. V-A "Hyperparameters"; Sec. IV-C, raise the batch while below
 * 95 % of memory): with cfg.kv_pool_blocks set from rlhf_gen_plan_capacity the call keeps as many rows in flight as
 * the pool holds, whatever B is.  Micro-batch i completes stagger_steps decode steps after micro-batch i - 1 (later if
 * it had to wait for pages), which is the spacing the consumer of done_events / on_ready sees (Sec. IV-A: the next stage
 * works on one micro-batch while the following ones are generated).
 * Requirements beyond rlhf_gen_generate's: B <= cfg.max_batch (every row keeps its own state row; the pool may be smaller
 * than B rows' worth) and every single micro-batch must fit the pool (else E_NOMEM before any work).  Results: row b draws
 * the random numbers it draws in rlhf_gen_generate, and its arithmetic does not depend on its batch mates up to 128
 * rows in flight, so the output equals rlhf_gen_generate's bit for bit under that limit.  done_events / on_ready as in
 * rlhf_gen_generate_stream.  rlhf_gen_last_timing reports the prefill time (sum), the rest as decode time, and the
 * number of decode steps run; rlhf_gen_last_peak_rows the most rows that decoded together. */
int rlhf_gen_generate_continuous(rlhf_gen_ctx* ctx, const int32_t* query_tokens, const int32_t* lengths, int32_t B,
                                 int32_t Lmax, int32_t max_resp_len, const rlhf_gen_sampling* sampling,
                                 int32_t* resp_tokens, float* resp_logprobs, int32_t micro_batch, int32_t stagger_steps,
                                 void* const* done_events, rlhf_gen_microbatch_fn on_ready, void* user);
int32_t rlhf_gen_last_peak_rows(const rlhf_gen_ctx* ctx);

/* The admission schedule rlhf_gen_generate_continuous would follow, without a context or a GPU: for each of the
 * ceil(B / micro_batch) micro-batches the decode-step count at which it is admitted and at which it completes
 * (admit + max_resp_len - 1), and the most rows decoding together.  A pure function of its arguments: micro-batch i is
 * admitted at the first step boundary where stagger_steps steps have passed since the previous admission and
 * kv_pool_blocks pages minus those held by running rows cover ceil((lengths[b] + max_resp_len - 1) / 16) pages for each of
 * its rows (pages of micro-batches completing at that boundary count as free).  With rlhf_gen_plan_capacity this answers
 * "how many rows will be in flight, and when does each micro-batch reach the next stage" for a memory budget (Sec. IV-C).
 *   lengths HOST int32 [B]; admit_step / done_step HOST int32 [ceil(B / micro_batch)] or NULL; peak_rows HOST or NULL.
 * Errors: E_INVALID, E_NOMEM (a micro-batch needs more pages than the pool has). */
int rlhf_gen_plan_admission(const int32_t* lengths, int32_t B, int32_t max_resp_len, int32_t micro_batch,
                            int32_t stagger_steps, int32_t kv_pool_blocks, int32_t* admit_step, int32_t* done_step,
                            int32_t* peak_rows);

/* Teacher-forced scoring pass: the raw-model log-probability of every token of given responses, by one forward over
 * query ++ response per sequence - `ActorOutput <- Actor.forward(Query, Response)` of Alg. 1 (the same call scores the
 * Ref model).  logprobs_out[b, t] = log softmax(logits at position lengths[b] - 1 + t)[resp_tokens[b, t]]; for a
 * rollout produced by rlhf_gen_generate with logprob_mode 0 it reproduces the log-probs returned there (up to the
 * rounding of the 16-bit path).  The [rows, vocab] logits are produced and consumed in blocks of 1024 rows inside the
 * library and never written out.  Replaces the batch held by the context (a following decode_step fails with E_STATE).
 *   query_tokens device int32 [B, Lmax]; lengths HOST int32 [B]; resp_tokens device int32 [B, R];
 *   lengths[b] + R - 1 <= max_seq; logprobs_out device float [B, R], valid after the stream is synchronised.
 * Errors as for rlhf_gen_prefill; every query and response id, the last response token included, is validated before
 * the forward pass (E_INVALID). */
int rlhf_gen_score(rlhf_gen_ctx* ctx, const int32_t* query_tokens, const int32_t* lengths, int32_t B, int32_t Lmax,
                   const int32_t* resp_tokens, int32_t R, float* logprobs_out);

/* Low-rank adapters to fold into the weights at a refresh (the paper trains the Actor with LoRA adapters of
 * dimension 4, Sec. V-A "Hyperparameters"): the effective matrix is W + scale * B A. */
typedef struct {
  const void* a;  /* device bf16 [rank, in_features]; NULL = no adapter on this matrix */
  const void* b;  /* device bf16 [out_features, rank] */
  int32_t rank;   /* 1..64 (an adapter on a fused matrix such as wqkv stacks its parts: rank = sum of their ranks) */
} rlhf_gen_lora_pair;
typedef struct {
  float scale;                          /* alpha / rank of the usual parametrisation */
  const rlhf_gen_lora_pair* wqkv;       /* HOST arrays of n_layers entries, or NULL for "none on these matrices" */
  const rlhf_gen_lora_pair* wo;
  const rlhf_gen_lora_pair* w_gate_up;
  const rlhf_gen_lora_pair* w_down;
  rlhf_gen_lora_pair lm_head;
} rlhf_gen_lora;

/* Refresh the replica's weights from the trainer's current ones - the periodic parameter synchronisation of the
 * shadow Actor in Alg. 2 (parameters of the shadow models are synchronised with the training models after each round of PPO training, Sec. IV-A, Disaggregated strategy) - without
 * allocating.  weights has the meaning it has in rlhf_gen_init (same shapes and dtype; the pointers may be the ones
 * given at init, whose contents the caller has overwritten, or other buffers).  bf16 mode: every projection matrix
 * and the LM head is converted again into the fp16 working copies made at init (with
 * RLHF_GEN_FLAG_CONVERT_IN_PLACE: rewritten in place, so the buffers must hold bf16 again when this is called), and
 * where lora names an adapter the update W + scale * B A is formed in fp32 on the way (one rounding to fp16).
 * lora may be NULL.  fp32 mode: the pointers are adopted; adapters are E_UNSUPPORTED there.
 * The work is enqueued on cfg.stream; the sources may be reused once it has completed.  The batch held by the context
 * is dropped (its KV cache belongs to the old weights): the next call must be prefill, generate or score.
 * Captured decode graphs stay valid unless an address the kernels read directly changed (token embedding, norm gains,
 * any matrix in fp32 or in-place mode); then they are recorded again by the next rlhf_gen_generate.
 * Errors: E_INVALID (NULL pointers, rank out of range), E_UNSUPPORTED, E_DEVICE. */
int rlhf_gen_update_weights(rlhf_gen_ctx* ctx, const rlhf_gen_weights* weights, const rlhf_gen_lora* lora);

/* Capacity planning.  The paper sizes every run by memory: the batch is the largest that does not run out of memory
 * (Sec. V-A "Hyperparameters"), and its guideline is to raise the batch while memory is spare and stop before 95 % of
 * the capacity (Sec. IV-C).  This call answers that question for one replica without allocating: the largest
 * max_batch for which a context created from cfg (cfg.max_batch is ignored, cfg.kv_pool_blocks must be 0, cfg.max_seq
 * = query + response length of the longest sequence) fits into fraction * capacity_bytes - reserved_bytes.  The
 * footprint is computed by the same code that performs the allocations in rlhf_gen_init (KV pool of
 * max_batch * ceil(max_seq / 16) pages per layer, fp16 working copies of the matrices unless
 * RLHF_GEN_FLAG_CONVERT_IN_PLACE, the 4-bit copies of wqkv and wo, activations, logits, split-K workspace), as the sum
 * of the sizes requested.
 *   capacity_bytes   memory of the card; 0 = ask HIP for the total memory of cfg.device (the only case that touches a GPU)
 *   fraction         in (0, 1], e.g. 0.95
 *   reserved_bytes   memory others hold on the card; a negative value stands for "the caller's copy of this model in
 *                    cfg.dtype", which rlhf_gen_init borrows
 *   *max_batch_out   the answer, 0 if not even one sequence fits; *context_bytes_out (may be NULL) the device bytes
 *                    such a context allocates
 * Errors: E_INVALID, E_UNSUPPORTED (as rlhf_gen_init for the shape), E_DEVICE. */
int rlhf_gen_plan_capacity(const rlhf_gen_cfg* cfg, int64_t capacity_bytes, double fraction, int64_t reserved_bytes,
                           int32_t* max_batch_out, int64_t* context_bytes_out);

/* Device bytes the context requested from HIP in rlhf_gen_init (what rlhf_gen_plan_capacity predicts). */
int64_t rlhf_gen_context_bytes(const rlhf_gen_ctx* ctx);

/* Number of decode-step graphs this context has recorded so far.  rlhf_gen_generate replays one captured graph per
 * decode step; the graph depends only on the number of batch rows - the sampling rule, the seed and the output
 * buffers are read from device memory at run time - so a PPO loop that calls generate with a new seed and fresh
 * output buffers every round (Alg. 1: one Actor.generate per batch of queries) records once and replays thereafter.
 * Up to 64 graphs (batch widths; row windows of rlhf_gen_generate_continuous) are kept. */
int64_t rlhf_gen_graph_captures(const rlhf_gen_ctx* ctx);

/* Copy the fp32 logits [B, vocab] that the last prefill/decode step sampled from into a device
 * buffer (parity checks), and wait for the steps enqueued so far.  E_STATE if no step has run; E_INVALID if an
 * earlier rlhf_gen_decode_step was given a forced token id outside [0, vocab) (see there). */
int rlhf_gen_get_logits(rlhf_gen_ctx* ctx, float* out);

/* Timing of the last rlhf_gen_generate on this context, measured with HIP events on cfg.stream:
 * prefill_ms, decode_ms (all decode steps together) and the number of decode steps. */
int rlhf_gen_last_timing(const rlhf_gen_ctx* ctx, float* prefill_ms, float* decode_ms, int32_t* decode_steps);

/* Time of every decode step of the last rlhf_gen_generate (HIP events on cfg.stream, one after each step): ms_out
 * receives min(capacity, *n_out) values, step t = 1 first; *n_out the number of steps.  Host pointers, either may be
 * NULL.  After rlhf_gen_generate_stream: the steps of the last micro-batch. */
int rlhf_gen_last_step_ms(const rlhf_gen_ctx* ctx, float* ms_out, int32_t capacity, int32_t* n_out);

/* Per-kernel timing of the decode loop, for roofline reports.  With every > 0, rlhf_gen_generate runs decode
 * step t kernel by kernel (instead of replaying its graph) whenever t % every == 0 and brackets each kernel with
 * HIP events on cfg.stream; at most 16 steps per call are sampled.  every = 0 switches it off.  Counters
 * accumulate over calls until the next rlhf_gen_set_profile.  Only the bf16 weight-streaming decode path is
 * instrumented. */
enum {
  RLHF_GEN_PROF_EMBED = 0, RLHF_GEN_PROF_NORM, RLHF_GEN_PROF_GEMM_QKV, RLHF_GEN_PROF_ROPE, RLHF_GEN_PROF_ATTN,
  RLHF_GEN_PROF_GEMM_WO, RLHF_GEN_PROF_GEMM_GATE_UP, RLHF_GEN_PROF_SWIGLU, RLHF_GEN_PROF_GEMM_DOWN,
  RLHF_GEN_PROF_LM_HEAD, RLHF_GEN_PROF_SAMPLER, RLHF_GEN_PROF_CLASSES
};
int rlhf_gen_set_profile(rlhf_gen_ctx* ctx, int32_t every);
/* ms[RLHF_GEN_PROF_CLASSES]: summed kernel time per class over the sampled steps; launches[...]: kernels timed;
 * *attn_tokens: sum over sampled steps and sequences of the cached tokens one attention launch read per KV head;
 * *steps: sampled steps.  Host pointers, any may be NULL. */
int rlhf_gen_get_profile(const rlhf_gen_ctx* ctx, double* ms, int64_t* launches, int64_t* attn_tokens, int32_t* steps);

/* Message of the last failed call on ctx (or of the last failed rlhf_gen_init if ctx is NULL).
 * The pointer stays valid until the next call on the same context. */
const char* rlhf_gen_last_error(const rlhf_gen_ctx* ctx);

/* Free everything the context owns.  The caller's weights are untouched.  NULL is allowed. */
void rlhf_gen_destroy(rlhf_gen_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* RLHF_GEN_H */
