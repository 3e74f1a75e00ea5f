// Host side of the library: context, argument checks, KV page allocator, and the sequencing of the
// kernels for prefill and decode (Actor.generate of Alg. 1 / ShadowActor.generate of Alg. 2).
// Everything numerical happens in the kernels; this file only decides what to launch.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <string>
#include <utility>
#include <vector>

#include "../../include/rlhf_gen.h"
#include "../../include/rlhf_gen_ops.h"
#include "kernels.h"

namespace {

std::string g_init_error;

// A captured decode step depends on the batch rows it covers and on nothing else: the sampling rule, the seed and the
// output buffers are read from a block in device memory (SamplerArgs) that is rewritten before the first replay of a
// rollout, positions and response indices from per-row device arrays.  Key: (first row, number of rows).
typedef std::pair<int, int> GraphKey;
constexpr size_t MAX_CACHED_GRAPHS = 64;
constexpr int SARGS_RING = 32;

}  // namespace

void set_global_error(const char* msg) { g_init_error = msg ? msg : ""; }

struct rlhf_gen_ctx {
  rlhf_gen_cfg cfg{};
  bool bf16 = false;
  hipStream_t stream = nullptr;
  bool own_stream = false;
  const void *tok_emb = nullptr, *lm_head = nullptr, *final_norm = nullptr;
  std::vector<const void*> attn_norm, wqkv, wo, ffn_norm, w_gate_up, w_down;
  // caller's bf16 matrices; in bf16 mode the members above point at fp16 working copies instead
  std::vector<const void*> src_wqkv, src_wo, src_w_gate_up, src_w_down;
  // Prefill contracts the low halves of the two pair-input projections in the 4-bit side format (common.h): 4-bit
  // copies of wqkv and wo with a scale byte per row, and the scale bytes of the activation rows' low halves.
  bool lo4 = false;
  std::vector<char*> w4_qkv, w4_wo, ws_qkv, ws_wo;
  char* a_scale = nullptr;
  int scale_groups = 0;
  const void* src_lm_head = nullptr;

  // device memory owned by the context
  std::vector<void*> allocs;
  size_t dev_bytes = 0;   // sum of the device allocations requested
  bool dry_run = false;   // capacity planning: walk the allocation sequence without allocating
  char* conv_tmp = nullptr;  // in-place mode: staging buffer of the weight conversion (one slab of rows)
  char* kv_pool = nullptr;
  size_t layer_pool_bytes = 0;
  int n_blocks = 0, max_blocks = 0;
  // per batch row: pages, cached tokens, response index of the next token to draw, token to feed next
  int *d_table = nullptr, *d_seq_len = nullptr, *d_step = nullptr, *d_err = nullptr, *d_cur_tok = nullptr;
  SamplerArgs* d_sargs = nullptr;   // sampling rule and output buffers of the rollout in flight (read by captured graphs)
  SamplerArgs* h_sargs = nullptr;   // pinned staging copies of it (a ring: a copy may still be in flight when the next is written)
  int sargs_next = 0;
  float *d_cos = nullptr, *d_sin = nullptr;
  int *d_tok_seq = nullptr, *d_tok_pos = nullptr, *d_ids = nullptr, *d_cu = nullptr, *d_seq_ids = nullptr,
      *d_last_rows = nullptr;
  // scoring pass scratch: gathered rows, their response slots, and a block of logits
  int score_cap = 0;
  int *d_srows = nullptr, *d_sslot = nullptr, *h_srows = nullptr, *h_sslot = nullptr;
  void* ys = nullptr;
  float* slogits = nullptr;
  int act_rows = 0;  // row capacity of the activation buffers
  float *x = nullptr, *qkv = nullptr, *logits = nullptr, *part = nullptr;
  void *y = nullptr, *yl = nullptr, *qb = nullptr, *ab = nullptr, *hb = nullptr;
  int ks_qkv = 1, ks_wo = 1, ks_gu = 1, ks_down = 1;
  // split counts of the split-K tile GEMM that takes decode batches of 129..256 rows (tile_ok: every projection
  // has a width the 256-column tiles divide)
  bool tile_ok = false;
  int kt_qkv = 1, kt_wo = 1, kt_gu = 1, kt_down = 1;

  // pinned host staging
  int *h_tok_seq = nullptr, *h_tok_pos = nullptr, *h_cu = nullptr, *h_seq_ids = nullptr, *h_last_rows = nullptr,
      *h_table = nullptr, *h_lenbuf = nullptr, *h_misc = nullptr;

  // host state
  std::vector<int> h_len, n_alloc, free_list;
  int B = 0;
  // The per-row device state (block-table rows, lengths, response indices, next tokens) of the rows the kernels are
  // working on starts at row win_lo of those arrays: 0 everywhere except in rlhf_gen_generate_continuous, where rows
  // [win_lo, win_lo + B) of the whole batch are the ones currently decoding.  Activations and logits are always
  // indexed from 0; host-side row state (h_len, n_alloc, h_table) is indexed by batch row like the device arrays.
  int win_lo = 0;
  bool have_batch = false, have_logits = false;
  int h_step = 0;
  int reserve_extra = 0;  // tokens beyond the query that prefill must reserve pages for
  int row_offset = 0;     // batch row of row 0 of the current (micro-)batch, for the sampler's random stream
  SamplerArgs sp{};       // sampling rule in force (output fields filled per launch)
  std::string err;
  // decode_step cannot wait for the device: the flag the embedding kernel raises for an out-of-range forced token is
  // copied to pinned memory behind each step and looked at by the next call that finds the copy complete
  int* h_step_err = nullptr;
  hipEvent_t ev_step_err = nullptr;
  bool step_err_pending = false;

  // optional per-kernel timing of sampled decode steps (rlhf_gen_set_profile)
  int prof_every = 0;
  bool prof_on = false;            // the step being enqueued is a sampled one
  std::vector<hipEvent_t> prof_ev;  // event pool
  std::vector<int> prof_cls;        // prof_cls[i] = class of the kernel that ends at event i (-1: start marker)
  int prof_used = 0;
  long long prof_attn_tokens = 0;   // cached tokens read by the sampled attention launches (per layer, per KV head)
  int prof_steps = 0;
  double prof_ms[RLHF_GEN_PROF_CLASSES] = {0};
  long long prof_n[RLHF_GEN_PROF_CLASSES] = {0};

  std::map<GraphKey, hipGraphExec_t> graphs;
  long long graph_captures = 0;
  hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
  std::vector<hipEvent_t> step_ev;   // one event after every decode step of the last rollout
  std::vector<float> step_ms;
  float prefill_ms = 0.f, decode_ms = 0.f;
  int decode_steps = 0;
  int peak_rows = 0;   // most rows decoding together in the last rlhf_gen_generate_continuous
};

namespace {

int fail(rlhf_gen_ctx* c, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_init_error = buf;
  return code;
}

#define HIP_TRY(c, call)                                                                                 \
  do {                                                                                                   \
    hipError_t e_ = (call);                                                                              \
    if (e_ != hipSuccess) return fail(c, RLHF_GEN_E_DEVICE, "%s failed: %s", #call, hipGetErrorString(e_)); \
  } while (0)

template <typename T>
int dev_alloc(rlhf_gen_ctx* c, T** p, size_t bytes, bool zero) {
  void* q = nullptr;
  if (bytes == 0) bytes = 16;
  c->dev_bytes += bytes;
  if (c->dry_run) {
    *p = nullptr;
    return RLHF_GEN_OK;
  }
  hipError_t e = hipMalloc(&q, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(c, RLHF_GEN_E_NOMEM, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
  }
  c->allocs.push_back(q);
  if (zero) HIP_TRY(c, hipMemset(q, 0, bytes));
  *p = (T*)q;
  return RLHF_GEN_OK;
}

template <typename T>
int host_alloc(rlhf_gen_ctx* c, T** p, size_t bytes) {
  void* q = nullptr;
  if (c->dry_run) {
    *p = nullptr;
    return RLHF_GEN_OK;
  }
  HIP_TRY(c, hipHostMalloc(&q, bytes ? bytes : 16, hipHostMallocDefault));
  memset(q, 0, bytes ? bytes : 16);
  *p = (T*)q;
  return RLHF_GEN_OK;
}

size_t act_size(const rlhf_gen_ctx* c) { return c->bf16 ? 2 : 4; }

// per-row device state of the current window (see rlhf_gen_ctx::win_lo)
int* w_seq_len(const rlhf_gen_ctx* c) { return c->d_seq_len + c->win_lo; }
int* w_step(const rlhf_gen_ctx* c) { return c->d_step + c->win_lo; }
int* w_cur_tok(const rlhf_gen_ctx* c) { return c->d_cur_tok + c->win_lo; }
int* w_table(const rlhf_gen_ctx* c) { return c->d_table + (size_t)c->win_lo * c->max_blocks; }

void reset_free_list(rlhf_gen_ctx* c) {
  c->free_list.resize(c->n_blocks);
  // popped from the back: block 0 first unless shuffled
  for (int i = 0; i < c->n_blocks; ++i) c->free_list[i] = c->n_blocks - 1 - i;
  if (c->cfg.flags & RLHF_GEN_FLAG_SHUFFLE_BLOCKS) {
    uint64_t s = 0x2545F4914F6CDD1Dull;
    for (int i = c->n_blocks - 1; i > 0; --i) {
      s ^= s << 13; s ^= s >> 7; s ^= s << 17;
      int j = (int)(s % (uint64_t)(i + 1));
      std::swap(c->free_list[i], c->free_list[j]);
    }
  }
  std::fill(c->n_alloc.begin(), c->n_alloc.end(), 0);
}

int blocks_for(int tokens) { return (tokens + 15) / 16; }

// Give sequence b enough pages for `tokens` cached tokens.  Returns true if the table changed.
bool grow_seq(rlhf_gen_ctx* c, int b, int tokens) {
  bool changed = false;
  while (c->n_alloc[b] * 16 < tokens) {
    int blk = c->free_list.back();
    c->free_list.pop_back();
    c->h_table[(size_t)b * c->max_blocks + c->n_alloc[b]] = blk;
    c->n_alloc[b]++;
    changed = true;
  }
  return changed;
}

int check_launch(rlhf_gen_ctx* c, hipError_t e, const char* what) {
  if (e != hipSuccess) return fail(c, RLHF_GEN_E_DEVICE, "launch of %s failed: %s", what, hipGetErrorString(e));
  return RLHF_GEN_OK;
}
#define LAUNCH(c, call, what)                        \
  do {                                               \
    int r_ = check_launch(c, (call), what);          \
    if (r_ != RLHF_GEN_OK) return r_;                \
  } while (0)

// Record the end of a kernel of class `cls` (or a start marker, cls = -1) when the step is being profiled.
void prof_mark(rlhf_gen_ctx* c, int cls) {
  if (!c->prof_on || c->prof_used >= (int)c->prof_ev.size()) return;
  if (hipEventRecord(c->prof_ev[c->prof_used], c->stream) != hipSuccess) return;
  c->prof_cls[c->prof_used++] = cls;
}

struct RowSet {
  int M = 0;
  const int* ids = nullptr;      // device [M] token ids
  const int* row_pos = nullptr;  // device [M] position of each row's token
  const int* row_seq = nullptr;  // device [M] batch row, or NULL for identity
  // prefill only
  bool prefill = false;
  const int* cu = nullptr;       // device [nseq + 1] chunk-local row offsets
  const int* seq_ids = nullptr;  // device [nseq]
  int nseq = 0, max_len = 0;
};

int gemm_any(rlhf_gen_ctx* c, const void* A, const void* W, void* out, int M, int N, int K, int epi, int a_dual = 0) {
  if (c->bf16) {
    LAUNCH(c, launch_gemm_h16(c->stream, A, W, out, M, N, K, epi, a_dual), "gemm_h16");
  } else {
    if (epi == EPI_SWIGLU) return fail(c, RLHF_GEN_E_UNSUPPORTED, "no fused SwiGLU on the fp32 path");
    LAUNCH(c, launch_gemm_f32(c->stream, (const float*)A, (const float*)W, (float*)out, M, N, K, epi == EPI_RESID_F32),
           "gemm_f32");
  }
  return RLHF_GEN_OK;
}

// All layers for a set of token rows, activations in x/y/...; leaves the residual stream in c->x.
int forward_layers_generic(rlhf_gen_ctx* c, const RowSet& r) {
  const rlhf_gen_cfg& g = c->cfg;
  const int d = g.d_model, Hq = g.n_heads, Hkv = g.n_kv_heads, h = g.head_dim, F = g.d_ffn;
  const int qkv_w = (Hq + 2 * Hkv) * h;
  hipStream_t s = c->stream;
  LAUNCH(c, launch_embed(s, r.ids, c->tok_emb, c->bf16, c->x, r.M, d, g.vocab, c->d_err), "embed");
  for (int l = 0; l < g.n_layers; ++l) {
    char* pool = c->kv_pool + (size_t)l * c->layer_pool_bytes;
    // 16-bit mode: the inputs of the QKV and output projections travel as fp16 hi|lo pairs
    const bool lo4 = c->lo4 && r.prefill;   // (rows that attend through the decode kernel keep fp16 pairs)
    LAUNCH(c, launch_rmsnorm(s, c->x, nullptr, 0, 0, c->attn_norm[l], c->bf16, c->y, c->bf16, r.M, d, g.rms_eps, nullptr,
                             lo4 ? 2 : c->bf16, c->a_scale, c->scale_groups), "rmsnorm");
    int rc = RLHF_GEN_OK;
    if (c->bf16) {
      // 16-bit mode: rotation and cache append are the projection's epilogue (head_dim is 128 there)
      const RopeEpi re{r.row_pos, r.row_seq, c->d_cos, c->d_sin, c->qb, pool, w_table(c), c->max_blocks, c->n_blocks, Hq, Hkv};
      if (lo4) {
        LAUNCH(c, launch_gemm_h16_lo4(s, c->y, c->wqkv[l], c->w4_qkv[l], c->ws_qkv[l], c->a_scale, c->scale_groups, nullptr, r.M,
                                      qkv_w, d, EPI_QKV_ROPE, &re), "gemm_qkv_rope lo4");
      } else {
        LAUNCH(c, launch_gemm_h16_qkv_rope(s, c->y, c->wqkv[l], r.M, d, re), "gemm_qkv_rope");
      }
    } else {
      rc = gemm_any(c, c->y, c->wqkv[l], c->qkv, r.M, qkv_w, d, EPI_STORE_F32, 0);
      if (rc) return rc;
      LAUNCH(c, launch_rope_append(s, c->qkv, nullptr, 0, 0, r.row_pos, r.row_seq, c->d_cos, c->d_sin, c->qb, pool,
                                   w_table(c), c->max_blocks, c->n_blocks, r.M, Hq, Hkv, h, 0), "rope_append");
    }
    if (!c->bf16) {
      LAUNCH(c, launch_attn_f32(s, (const float*)c->qb, (const float*)pool, w_table(c), c->max_blocks, c->n_blocks, r.row_pos,
                                r.row_seq, (float*)c->ab, r.M, Hq, Hkv, h), "attn_f32");
    } else if (r.prefill) {
      LAUNCH(c, launch_attn_prefill_h16(s, c->qb, pool, w_table(c), c->max_blocks, c->n_blocks, r.cu, r.seq_ids, c->ab, r.nseq,
                                         r.max_len, Hq, Hkv, lo4 ? c->a_scale : nullptr, c->scale_groups), "attn_prefill");
    } else {
      LAUNCH(c, launch_attn_decode_h16(s, c->qb, pool, w_table(c), c->max_blocks, c->n_blocks, w_seq_len(c), c->ab, r.M, Hq, Hkv),
             "attn_decode");
    }
    if (lo4) {
      LAUNCH(c, launch_gemm_h16_lo4(s, c->ab, c->wo[l], c->w4_wo[l], c->ws_wo[l], c->a_scale, c->scale_groups, c->x, r.M, d,
                                    Hq * h, EPI_RESID_F32, nullptr), "gemm_wo lo4");
    } else {
      rc = gemm_any(c, c->ab, c->wo[l], c->x, r.M, d, Hq * h, EPI_RESID_F32, c->bf16);
      if (rc) return rc;
    }
    LAUNCH(c, launch_rmsnorm(s, c->x, nullptr, 0, 0, c->ffn_norm[l], c->bf16, c->y, c->bf16, r.M, d, g.rms_eps, nullptr, 0),
           "rmsnorm");
    if (c->bf16) {
      rc = gemm_any(c, c->y, c->w_gate_up[l], c->hb, r.M, F, d, EPI_SWIGLU);
      if (rc) return rc;
    } else {
      rc = gemm_any(c, c->y, c->w_gate_up[l], c->qkv, r.M, 2 * F, d, EPI_STORE_F32);
      if (rc) return rc;
      LAUNCH(c, launch_swiglu(s, c->qkv, 1, 0, c->hb, 0, r.M, F), "swiglu");
    }
    rc = gemm_any(c, c->hb, c->w_down[l], c->x, r.M, d, F, EPI_RESID_F32);
    if (rc) return rc;
  }
  return RLHF_GEN_OK;
}

// Decode step on the weight-streaming GEMM: every projection writes split-K partial sums, and the next
// small kernel (RoPE+append, RMSNorm+residual, SwiGLU) adds them up while doing its own work.
// Projection whose input travels as hi|lo pairs: the streaming kernel takes up to 128 such rows, taller batches go
// in slabs of 128 rows that share the split-K planes of `part` (the weights are then streamed once per slab).
static int skinny_pairs(rlhf_gen_ctx* c, const void* A, const void* W, int B, int Nw, int K, int nsplit, const char* what) {
  for (int r0 = 0; r0 < B; r0 += 128) {
    const int rows = std::min(128, B - r0);
    LAUNCH(c, launch_gemm_skinny_h16(c->stream, (const uint16_t*)A + (size_t)r0 * 2 * K, W, c->part + (size_t)r0 * Nw, rows, Nw,
                                     K, nsplit, 1, B), what);
  }
  return RLHF_GEN_OK;
}

// Batches of more than 128 rows are past the point where the weight stream bounds the projections (at 256 rows the
// MFMA time of a projection exceeds its weight-streaming time), and the streaming kernel, in which every wavefront
// reads the whole activation slice, falls behind: measured at 256 rows on the 7B shapes, QKV 115 -> 62 us,
// output projection 43 -> 28 us, gate/up 180 -> 74 + 12 us (un-fused, two splits), down 75 -> 42 us with the
// split-K form of the large-tile GEMM.  At 128 rows and below the streaming kernels are faster.
static bool decode_uses_tiles(const rlhf_gen_ctx* c, int B) { return c->tile_ok && B > 128; }

int forward_decode_streaming(rlhf_gen_ctx* c, int B) {
  const rlhf_gen_cfg& g = c->cfg;
  const int d = g.d_model, Hq = g.n_heads, Hkv = g.n_kv_heads, h = g.head_dim, F = g.d_ffn;
  const int qkv_w = (Hq + 2 * Hkv) * h;
  hipStream_t s = c->stream;
  const bool tiles = decode_uses_tiles(c, B);
  // the split-K tile GEMMs of the two pair-input projections take the 4-bit low halves of the prefill (the fused
  // RoPE + attention kernel writes fp16 pairs only)
  const bool lo4 = tiles && c->lo4 && !(c->cfg.flags & RLHF_GEN_FLAG_FUSED_ROPE);
  const int ks_qkv = tiles ? c->kt_qkv : c->ks_qkv, ks_wo = tiles ? c->kt_wo : c->ks_wo;
  const int ks_down = tiles ? c->kt_down : c->ks_down;
  prof_mark(c, -1);
  LAUNCH(c, launch_embed(s, w_cur_tok(c), c->tok_emb, 1, c->x, B, d, g.vocab, c->d_err), "embed");
  prof_mark(c, RLHF_GEN_PROF_EMBED);
  int pending = 0;  // split count of the down-projection partial sums not yet added to x
  for (int l = 0; l < g.n_layers; ++l) {
    char* pool = c->kv_pool + (size_t)l * c->layer_pool_bytes;
    LAUNCH(c, launch_rmsnorm(s, c->x, pending ? c->part : nullptr, pending, (size_t)B * d, c->attn_norm[l], 1, c->y, 1,
                             B, d, g.rms_eps, nullptr, lo4 ? 2 : 1, c->a_scale, c->scale_groups), "rmsnorm");
    prof_mark(c, RLHF_GEN_PROF_NORM);
    if (lo4) {
      LAUNCH(c, launch_gemm_h16_splitk_lo4(s, c->y, c->wqkv[l], c->w4_qkv[l], c->ws_qkv[l], c->a_scale, c->scale_groups, c->part, B,
                                           qkv_w, d, ks_qkv, B), "gemm_splitk qkv lo4");
    } else if (tiles) {
      LAUNCH(c, launch_gemm_h16_splitk(s, c->y, c->wqkv[l], c->part, B, qkv_w, d, 1, ks_qkv, B), "gemm_splitk qkv");
    } else if (int rc = skinny_pairs(c, c->y, c->wqkv[l], B, qkv_w, d, ks_qkv, "gemm_skinny qkv")) {
      return rc;
    }
    prof_mark(c, RLHF_GEN_PROF_GEMM_QKV);
    size_t st = (size_t)B * qkv_w;
    if (!(c->cfg.flags & RLHF_GEN_FLAG_FUSED_ROPE)) {
      LAUNCH(c, launch_rope_append(s, c->part, ks_qkv > 1 ? c->part + st : nullptr, ks_qkv - 1, st, w_seq_len(c),
                                   nullptr, c->d_cos, c->d_sin, c->qb, pool, w_table(c), c->max_blocks, c->n_blocks, B, Hq,
                                   Hkv, h, 1), "rope_append");
      prof_mark(c, RLHF_GEN_PROF_ROPE);
      LAUNCH(c, launch_attn_decode_h16(s, c->qb, pool, w_table(c), c->max_blocks, c->n_blocks, w_seq_len(c), c->ab, B, Hq,
                                       Hkv, lo4 ? c->a_scale : nullptr, c->scale_groups), "attn_decode");
    } else {
      LAUNCH(c, launch_attn_decode_fused_h16(s, c->part, ks_qkv, st, c->d_cos, c->d_sin, pool, w_table(c), c->max_blocks,
                                             c->n_blocks, w_seq_len(c), c->ab, B, Hq, Hkv), "attn_decode_fused");
    }
    prof_mark(c, RLHF_GEN_PROF_ATTN);
    if (lo4) {
      LAUNCH(c, launch_gemm_h16_splitk_lo4(s, c->ab, c->wo[l], c->w4_wo[l], c->ws_wo[l], c->a_scale, c->scale_groups, c->part, B, d,
                                           Hq * h, ks_wo, B), "gemm_splitk wo lo4");
    } else if (tiles) {
      LAUNCH(c, launch_gemm_h16_splitk(s, c->ab, c->wo[l], c->part, B, d, Hq * h, 1, ks_wo, B), "gemm_splitk wo");
    } else if (int rc = skinny_pairs(c, c->ab, c->wo[l], B, d, Hq * h, ks_wo, "gemm_skinny wo")) {
      return rc;
    }
    prof_mark(c, RLHF_GEN_PROF_GEMM_WO);
    LAUNCH(c, launch_rmsnorm(s, c->x, c->part, ks_wo, (size_t)B * d, c->ffn_norm[l], 1, c->y, 1, B, d, g.rms_eps,
                             nullptr, 0), "rmsnorm");
    prof_mark(c, RLHF_GEN_PROF_NORM);
    if (tiles) {
      // gate and up as plain partial sums (the fused SwiGLU epilogue cannot be split), combined by a small kernel
      LAUNCH(c, launch_gemm_h16_splitk(s, c->y, c->w_gate_up[l], c->part, B, 2 * F, d, 0, c->kt_gu, B), "gemm_splitk gate_up");
      LAUNCH(c, launch_swiglu(s, c->part, c->kt_gu, (size_t)B * 2 * F, c->hb, 1, B, F), "swiglu");
    } else {
      LAUNCH(c, launch_gemm_skinny_h16(s, c->y, c->w_gate_up[l], (float*)c->hb, B, 2 * F, d, 0, 0), "gemm_skinny gate_up");
    }
    prof_mark(c, RLHF_GEN_PROF_GEMM_GATE_UP);
    if (tiles) {
      LAUNCH(c, launch_gemm_h16_splitk(s, c->hb, c->w_down[l], c->part, B, d, F, 0, ks_down, B), "gemm_splitk down");
    } else {
      LAUNCH(c, launch_gemm_skinny_h16(s, c->hb, c->w_down[l], c->part, B, d, F, ks_down, 0), "gemm_skinny down");
    }
    prof_mark(c, RLHF_GEN_PROF_GEMM_DOWN);
    pending = ks_down;
  }
  LAUNCH(c, launch_rmsnorm(s, c->x, pending ? c->part : nullptr, pending, (size_t)B * d, c->final_norm, 1, c->yl, 1, B,
                           d, g.rms_eps, nullptr, 0), "final rmsnorm");
  prof_mark(c, RLHF_GEN_PROF_NORM);
  if (tiles && g.vocab % 256 == 0 && (size_t)g.vocab * d * 2 < ((size_t)1 << 32)) {
    LAUNCH(c, launch_gemm_h16(s, c->yl, c->lm_head, c->logits, B, g.vocab, d, EPI_STORE_F32, 0), "gemm lm_head");
  } else {
    LAUNCH(c, launch_gemm_skinny_h16(s, c->yl, c->lm_head, c->logits, B, g.vocab, d, 1, 0), "gemm_skinny lm_head");
  }
  prof_mark(c, RLHF_GEN_PROF_LM_HEAD);
  return RLHF_GEN_OK;
}

bool use_streaming(const rlhf_gen_ctx* c, int B) {
  // the weight-streaming GEMM takes up to 256 rows (hi|lo activation pairs in slabs of 128); larger batches use the
  // tiled GEMM
  return c->bf16 && !(c->cfg.flags & RLHF_GEN_FLAG_GENERIC_GEMM) && B <= 256;
}

// Kernels of one decode step, in order, ending with the sampler and the counter update.
// `from_dev`: the sampler reads its arguments from c->d_sargs (graph capture and everything else inside a rollout);
// otherwise they are passed by value with the given outputs (single decode steps, whose buffers change per call).
int enqueue_decode_body(rlhf_gen_ctx* c, int* tok_out, float* lp_out, int stride, int use_col, bool from_dev) {
  const rlhf_gen_cfg& g = c->cfg;
  const int B = c->B;
  int rc;
  if (use_streaming(c, B)) {
    rc = forward_decode_streaming(c, B);
    if (rc) return rc;
  } else {
    RowSet r;
    r.M = B;
    r.ids = w_cur_tok(c);
    r.row_pos = w_seq_len(c);
    rc = forward_layers_generic(c, r);
    if (rc) return rc;
    LAUNCH(c, launch_rmsnorm(c->stream, c->x, nullptr, 0, 0, c->final_norm, c->bf16, c->yl, c->bf16, B, g.d_model,
                             g.rms_eps, nullptr, 0), "final rmsnorm");
    rc = gemm_any(c, c->yl, c->lm_head, c->logits, B, g.vocab, g.d_model, EPI_STORE_F32);
    if (rc) return rc;
  }
  SamplerArgs a = c->sp;
  a.out_stride = stride; a.use_step_col = use_col; a.step_stride = 1; a.tok_out = tok_out; a.lp_out = lp_out;
  LAUNCH(c, launch_sampler(c->stream, c->logits, B, g.vocab, a, from_dev ? c->d_sargs : nullptr, w_step(c), w_cur_tok(c),
                           w_seq_len(c), w_step(c)), "sampler");   // (and the step's bookkeeping)
  prof_mark(c, RLHF_GEN_PROF_SAMPLER);
  return RLHF_GEN_OK;
}

int check_sampling(rlhf_gen_ctx* c, const rlhf_gen_sampling* sp) {
  if (!sp) return fail(c, RLHF_GEN_E_INVALID, "sampling is NULL");
  if (!sp->greedy) {
    if (!(sp->temperature > 0.f) || !isfinite(sp->temperature))
      return fail(c, RLHF_GEN_E_INVALID, "temperature must be a positive finite number (got %g)", sp->temperature);
    if (!(sp->top_p > 0.f)) return fail(c, RLHF_GEN_E_INVALID, "top_p must be positive (got %g)", sp->top_p);
  }
  if (sp->logprob_mode != 0 && sp->logprob_mode != 1)
    return fail(c, RLHF_GEN_E_INVALID, "logprob_mode must be 0 or 1 (got %d)", sp->logprob_mode);
  return RLHF_GEN_OK;
}

// Prefill of B queries into batch rows [c->win_lo, c->win_lo + B): query_tokens / lengths / the outputs point at the first
// of these rows.  fresh: the context holds nothing else (every page is free again); otherwise rows outside the range
// keep their cache pages and state, and the new rows take pages from what is left.
int prefill_impl(rlhf_gen_ctx* c, const int32_t* query_tokens, const int32_t* lengths, int32_t B, int32_t Lmax,
                 const rlhf_gen_sampling* sampling, int32_t* tok_out, float* lp_out, int out_stride, bool fresh = true) {
  const rlhf_gen_cfg& g = c->cfg;
  const int lo = c->win_lo;
  if (!query_tokens || !lengths || !tok_out || !lp_out) return fail(c, RLHF_GEN_E_INVALID, "NULL pointer argument");
  int rc = check_sampling(c, sampling);
  if (rc) return rc;
  if (B < 1 || lo + B > g.max_batch)
    return fail(c, RLHF_GEN_E_INVALID, "B = %d outside [1, max_batch = %d]", lo + B, g.max_batch);
  if (Lmax < 1) return fail(c, RLHF_GEN_E_INVALID, "Lmax = %d must be positive", Lmax);
  long need_blocks = 0;
  for (int b = 0; b < B; ++b) {
    if (lengths[b] < 1 || lengths[b] > Lmax)
      return fail(c, RLHF_GEN_E_INVALID, "lengths[%d] = %d outside [1, Lmax = %d]", b, lengths[b], Lmax);
    if (lengths[b] + 1 + c->reserve_extra > g.max_seq + 1)
      return fail(c, RLHF_GEN_E_INVALID, "sequence %d: %d query + %d further tokens exceed max_seq = %d", b, lengths[b],
                  c->reserve_extra, g.max_seq);
    need_blocks += blocks_for(lengths[b] + c->reserve_extra);
  }
  if (need_blocks > (fresh ? (long)c->n_blocks : (long)c->free_list.size()))
    return fail(c, RLHF_GEN_E_NOMEM, "KV pool has %ld free pages, the batch needs %ld",
                fresh ? (long)c->n_blocks : (long)c->free_list.size(), need_blocks);

  HIP_TRY(c, hipSetDevice(g.device));
  HIP_TRY(c, hipStreamSynchronize(c->stream));  // staging buffers are free again
  c->have_batch = false;
  c->have_logits = false;
  c->B = B;
  c->sp.temperature = sampling->temperature;
  c->sp.top_p = sampling->top_p;
  c->sp.seed = sampling->seed;
  c->sp.greedy = sampling->greedy;
  c->sp.logprob_mode = sampling->logprob_mode;
  c->sp.row0 = c->row_offset + lo;
  if (fresh) reset_free_list(c);
  int T = 0;
  for (int b = 0; b < B; ++b) {
    c->h_len[lo + b] = lengths[b];
    grow_seq(c, lo + b, lengths[b] + c->reserve_extra);
    for (int p = 0; p < lengths[b]; ++p) {
      c->h_tok_seq[T] = b;
      c->h_tok_pos[T] = p;
      ++T;
    }
    c->h_lenbuf[b] = lengths[b];
    c->h_seq_ids[b] = b;
  }
  hipStream_t s = c->stream;
  HIP_TRY(c, hipMemcpyAsync(w_table(c), c->h_table + (size_t)lo * c->max_blocks, sizeof(int) * (size_t)B * c->max_blocks,
                            hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipMemcpyAsync(c->d_tok_seq, c->h_tok_seq, sizeof(int) * T, hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipMemcpyAsync(c->d_tok_pos, c->h_tok_pos, sizeof(int) * T, hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipMemcpyAsync(w_seq_len(c), c->h_lenbuf, sizeof(int) * B, hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipMemcpyAsync(c->d_seq_ids, c->h_seq_ids, sizeof(int) * B, hipMemcpyHostToDevice, s));
  c->h_misc[0] = 0;
  c->h_misc[1] = 1;
  if (fresh) HIP_TRY(c, hipMemcpyAsync(c->d_err, &c->h_misc[0], sizeof(int), hipMemcpyHostToDevice, s));
  c->step_err_pending = false;   // (the stream was synchronised above: no copy of the flag is in flight)
  *c->h_step_err = 0;
  LAUNCH(c, launch_fill_int(s, w_step(c), B, 0), "fill");
  LAUNCH(c, launch_pack_tokens(s, query_tokens, Lmax, c->d_tok_seq, c->d_tok_pos, T, g.vocab, c->d_ids, c->d_err),
         "pack_tokens");
  HIP_TRY(c, hipMemcpyAsync(&c->h_misc[2], c->d_err, sizeof(int), hipMemcpyDeviceToHost, s));
  HIP_TRY(c, hipStreamSynchronize(s));
  if (c->h_misc[2]) return fail(c, RLHF_GEN_E_INVALID, "a query token id lies outside [0, vocab = %d)", g.vocab);

  // chunks of whole sequences that fit the activation buffers
  std::vector<int> chunk_begin;
  {
    int rows = 0;
    chunk_begin.push_back(0);
    for (int b = 0; b < B; ++b) {
      if (rows + lengths[b] > c->act_rows) {
        chunk_begin.push_back(b);
        rows = 0;
      }
      rows += lengths[b];
    }
    chunk_begin.push_back(B);
  }
  // chunk-local row offsets and last-token rows, all chunks at once
  int cu_fill = 0;
  std::vector<int> cu_at(chunk_begin.size() - 1);
  for (size_t ci = 0; ci + 1 < chunk_begin.size(); ++ci) {
    cu_at[ci] = cu_fill;
    int rows = 0;
    c->h_cu[cu_fill++] = 0;
    for (int b = chunk_begin[ci]; b < chunk_begin[ci + 1]; ++b) {
      rows += lengths[b];
      c->h_cu[cu_fill++] = rows;
      c->h_last_rows[b] = rows - 1;
    }
  }
  HIP_TRY(c, hipMemcpyAsync(c->d_cu, c->h_cu, sizeof(int) * cu_fill, hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipMemcpyAsync(c->d_last_rows, c->h_last_rows, sizeof(int) * B, hipMemcpyHostToDevice, s));

  int row0 = 0;
  for (size_t ci = 0; ci + 1 < chunk_begin.size(); ++ci) {
    int b0 = chunk_begin[ci], b1 = chunk_begin[ci + 1];
    RowSet r;
    r.prefill = true;
    r.nseq = b1 - b0;
    r.M = 0;
    r.max_len = 0;
    for (int b = b0; b < b1; ++b) {
      r.M += lengths[b];
      r.max_len = std::max(r.max_len, (int)lengths[b]);
    }
    r.ids = c->d_ids + row0;
    r.row_pos = c->d_tok_pos + row0;
    r.row_seq = c->d_tok_seq + row0;
    r.cu = c->d_cu + cu_at[ci];
    r.seq_ids = c->d_seq_ids + b0;
    rc = forward_layers_generic(c, r);
    if (rc) return rc;
    // final norm of each sequence's last row, gathered into rows b0..b1 of yl
    LAUNCH(c, launch_rmsnorm(s, c->x, nullptr, 0, 0, c->final_norm, c->bf16,
                             (char*)c->yl + (size_t)b0 * g.d_model * act_size(c), c->bf16, r.nseq, g.d_model, g.rms_eps,
                             c->d_last_rows + b0, 0), "final rmsnorm");
    row0 += r.M;
  }
  rc = gemm_any(c, c->yl, c->lm_head, c->logits, B, g.vocab, g.d_model, EPI_STORE_F32);
  if (rc) return rc;
  {
    SamplerArgs a = c->sp;
    a.out_stride = out_stride; a.use_step_col = 1; a.step_stride = 1; a.tok_out = tok_out; a.lp_out = lp_out;
    LAUNCH(c, launch_sampler(s, c->logits, B, g.vocab, a, nullptr, w_step(c), w_cur_tok(c)), "sampler");
  }
  LAUNCH(c, launch_fill_int(s, w_step(c), B, 1), "fill");
  c->h_step = 1;
  c->have_batch = true;
  c->have_logits = true;
  return RLHF_GEN_OK;
}

// Teacher-forced forward over query ++ response[0 .. R-2] and log-softmax gather at the R positions that predict the
// response tokens.  Uses the same kernels as prefill; replaces the batch held by the context.
int score_impl(rlhf_gen_ctx* c, const int32_t* query_tokens, const int32_t* lengths, int32_t B, int32_t Lmax,
               const int32_t* resp_tokens, int32_t R, float* lp_out) {
  const rlhf_gen_cfg& g = c->cfg;
  if (!query_tokens || !lengths || !resp_tokens || !lp_out) return fail(c, RLHF_GEN_E_INVALID, "NULL pointer argument");
  if (B < 1 || B > g.max_batch) return fail(c, RLHF_GEN_E_INVALID, "B = %d outside [1, max_batch = %d]", B, g.max_batch);
  if (Lmax < 1 || R < 1) return fail(c, RLHF_GEN_E_INVALID, "Lmax and R must be positive");
  long need_blocks = 0;
  for (int b = 0; b < B; ++b) {
    if (lengths[b] < 1 || lengths[b] > Lmax)
      return fail(c, RLHF_GEN_E_INVALID, "lengths[%d] = %d outside [1, Lmax = %d]", b, lengths[b], Lmax);
    if (lengths[b] + R - 1 > g.max_seq)
      return fail(c, RLHF_GEN_E_INVALID, "sequence %d: %d query + %d response tokens exceed max_seq = %d", b, lengths[b], R,
                  g.max_seq);
    need_blocks += blocks_for(lengths[b] + R - 1);
  }
  if (need_blocks > c->n_blocks)
    return fail(c, RLHF_GEN_E_NOMEM, "KV pool has %d pages, the batch needs %ld", c->n_blocks, need_blocks);
  HIP_TRY(c, hipSetDevice(g.device));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  c->have_batch = false;
  c->have_logits = false;
  c->B = B;
  c->win_lo = 0;
  reset_free_list(c);
  int T = 0;
  for (int b = 0; b < B; ++b) {
    const int fed = lengths[b] + R - 1;
    c->h_len[b] = fed;
    grow_seq(c, b, fed);
    for (int p = 0; p < fed; ++p) {
      c->h_tok_seq[T] = b;
      c->h_tok_pos[T] = p;
      ++T;
    }
    c->h_lenbuf[b] = lengths[b];
    c->h_seq_ids[b] = b;
  }
  hipStream_t s = c->stream;
  HIP_TRY(c, hipMemcpyAsync(c->d_table, c->h_table, sizeof(int) * (size_t)g.max_batch * c->max_blocks,
                            hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipMemcpyAsync(c->d_tok_seq, c->h_tok_seq, sizeof(int) * T, hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipMemcpyAsync(c->d_tok_pos, c->h_tok_pos, sizeof(int) * T, hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipMemcpyAsync(c->d_seq_len, c->h_lenbuf, sizeof(int) * B, hipMemcpyHostToDevice, s));  // query lengths
  HIP_TRY(c, hipMemcpyAsync(c->d_seq_ids, c->h_seq_ids, sizeof(int) * B, hipMemcpyHostToDevice, s));
  c->h_misc[0] = 0;
  HIP_TRY(c, hipMemcpyAsync(c->d_err, &c->h_misc[0], sizeof(int), hipMemcpyHostToDevice, s));
  LAUNCH(c, launch_pack_tokens2(s, query_tokens, Lmax, resp_tokens, R, c->d_seq_len, c->d_tok_seq, c->d_tok_pos, T,
                                g.vocab, c->d_ids, c->d_err), "pack_tokens2");
  HIP_TRY(c, hipMemcpyAsync(&c->h_misc[2], c->d_err, sizeof(int), hipMemcpyDeviceToHost, s));
  HIP_TRY(c, hipStreamSynchronize(s));
  if (c->h_misc[2]) return fail(c, RLHF_GEN_E_INVALID, "a token id lies outside [0, vocab = %d)", g.vocab);

  std::vector<int> chunk_begin;
  {
    int rows = 0;
    chunk_begin.push_back(0);
    for (int b = 0; b < B; ++b) {
      const int fed = lengths[b] + R - 1;
      if (rows + fed > c->act_rows) {
        chunk_begin.push_back(b);
        rows = 0;
      }
      rows += fed;
    }
    chunk_begin.push_back(B);
  }
  // per chunk: local row offsets; for every response slot (b, t) the chunk-local row that predicts it
  int cu_fill = 0, sfill = 0;
  std::vector<int> cu_at(chunk_begin.size() - 1), s_at(chunk_begin.size());
  for (size_t ci = 0; ci + 1 < chunk_begin.size(); ++ci) {
    cu_at[ci] = cu_fill;
    s_at[ci] = sfill;
    int rows = 0;
    c->h_cu[cu_fill++] = 0;
    for (int b = chunk_begin[ci]; b < chunk_begin[ci + 1]; ++b) {
      for (int t = 0; t < R; ++t) {
        c->h_srows[sfill] = rows + lengths[b] - 1 + t;
        c->h_sslot[sfill] = b * R + t;
        ++sfill;
      }
      rows += lengths[b] + R - 1;
      c->h_cu[cu_fill++] = rows;
    }
  }
  s_at[chunk_begin.size() - 1] = sfill;
  HIP_TRY(c, hipMemcpyAsync(c->d_cu, c->h_cu, sizeof(int) * cu_fill, hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipMemcpyAsync(c->d_srows, c->h_srows, sizeof(int) * sfill, hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipMemcpyAsync(c->d_sslot, c->h_sslot, sizeof(int) * sfill, hipMemcpyHostToDevice, s));

  int row0 = 0;
  for (size_t ci = 0; ci + 1 < chunk_begin.size(); ++ci) {
    int b0 = chunk_begin[ci], b1 = chunk_begin[ci + 1];
    RowSet r;
    r.prefill = true;
    r.nseq = b1 - b0;
    for (int b = b0; b < b1; ++b) {
      r.M += lengths[b] + R - 1;
      r.max_len = std::max(r.max_len, (int)lengths[b] + R - 1);
    }
    r.ids = c->d_ids + row0;
    r.row_pos = c->d_tok_pos + row0;
    r.row_seq = c->d_tok_seq + row0;
    r.cu = c->d_cu + cu_at[ci];
    r.seq_ids = c->d_seq_ids + b0;
    int rc = forward_layers_generic(c, r);
    if (rc) return rc;
    // LM head + log-softmax gather over the chunk's scoring rows, score_cap rows at a time (logits never leave the scratch)
    for (int q0 = s_at[ci]; q0 < s_at[ci + 1]; q0 += c->score_cap) {
      const int n = std::min(c->score_cap, s_at[ci + 1] - q0);
      LAUNCH(c, launch_rmsnorm(s, c->x, nullptr, 0, 0, c->final_norm, c->bf16, c->ys, c->bf16, n, g.d_model, g.rms_eps,
                               c->d_srows + q0, 0), "final rmsnorm");
      rc = gemm_any(c, c->ys, c->lm_head, c->slogits, n, g.vocab, g.d_model, EPI_STORE_F32);
      if (rc) return rc;
      LAUNCH(c, launch_logprob_gather(s, c->slogits, n, g.vocab, c->d_sslot + q0, resp_tokens, lp_out, c->d_err),
             "logprob_gather");
    }
    row0 += r.M;
  }
  return RLHF_GEN_OK;
}

int decode_checks(rlhf_gen_ctx* c) {
  if (!c->have_batch) return fail(c, RLHF_GEN_E_STATE, "decode_step before a successful prefill");
  long need = 0;
  for (int b = c->win_lo; b < c->win_lo + c->B; ++b) {
    if (c->h_len[b] + 1 > c->cfg.max_seq)
      return fail(c, RLHF_GEN_E_STATE, "sequence %d already holds %d tokens (max_seq = %d)", b, c->h_len[b], c->cfg.max_seq);
    if (c->n_alloc[b] * 16 < c->h_len[b] + 1) need++;
  }
  if (need > (long)c->free_list.size())
    return fail(c, RLHF_GEN_E_NOMEM, "KV pool exhausted: %ld more pages needed, %zu free", need, c->free_list.size());
  if (need) {
    HIP_TRY(c, hipStreamSynchronize(c->stream));  // the pinned table may still be in flight
    for (int b = c->win_lo; b < c->win_lo + c->B; ++b) grow_seq(c, b, c->h_len[b] + 1);
    HIP_TRY(c, hipMemcpyAsync(c->d_table, c->h_table, sizeof(int) * (size_t)c->cfg.max_batch * c->max_blocks,
                              hipMemcpyHostToDevice, c->stream));
  }
  return RLHF_GEN_OK;
}

void after_step(rlhf_gen_ctx* c) {
  for (int b = c->win_lo; b < c->win_lo + c->B; ++b) c->h_len[b]++;
  c->h_step++;
}

void drop_graph(rlhf_gen_ctx* c) {
  for (auto& kv : c->graphs) (void)hipGraphExecDestroy(kv.second);
  c->graphs.clear();
}

// The decode step for batch rows [c->win_lo, c->win_lo + B) as an executable graph: recorded once, then reused by every rollout of that
// width (nothing a rollout changes - seed, temperature, top-p, output buffers - is baked into it).
int decode_graph(rlhf_gen_ctx* c, int B, hipGraphExec_t* out) {
  const GraphKey key(c->win_lo, B);
  auto it = c->graphs.find(key);
  if (it != c->graphs.end()) {
    *out = it->second;
    return RLHF_GEN_OK;
  }
  if (c->graphs.size() >= MAX_CACHED_GRAPHS) drop_graph(c);
  hipGraph_t graph = nullptr;
  HIP_TRY(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
  int rc = enqueue_decode_body(c, nullptr, nullptr, 0, 0, true);
  hipError_t e = hipStreamEndCapture(c->stream, &graph);
  if (rc) {
    if (graph) (void)hipGraphDestroy(graph);
    return rc;
  }
  if (e != hipSuccess) return fail(c, RLHF_GEN_E_DEVICE, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
  hipGraphExec_t exec = nullptr;
  e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (e != hipSuccess) return fail(c, RLHF_GEN_E_DEVICE, "hipGraphInstantiate failed: %s", hipGetErrorString(e));
  c->graphs[key] = exec;
  c->graph_captures++;
  *out = exec;
  return RLHF_GEN_OK;
}

// Sampling rule, random-stream row and output rows of the decode window [c->win_lo, c->win_lo + c->B) into the device
// block that the (captured) sampler reads.  tok_base / lp_base: row 0 of the whole batch's [rows, R] outputs.
int push_sampler_args(rlhf_gen_ctx* c, int R, int32_t* tok_base, float* lp_base) {
  if (c->sargs_next == SARGS_RING) {   // every staging slot has been handed to a copy: let them all finish
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->sargs_next = 0;
  }
  SamplerArgs* h = c->h_sargs + c->sargs_next++;
  *h = c->sp;
  h->row0 = c->row_offset + c->win_lo;
  h->out_stride = R; h->use_step_col = 1; h->step_stride = 1;
  h->tok_out = tok_base + (size_t)c->win_lo * R;
  h->lp_out = lp_base + (size_t)c->win_lo * R;
  HIP_TRY(c, hipMemcpyAsync(c->d_sargs, h, sizeof(SamplerArgs), hipMemcpyHostToDevice, c->stream));
  return RLHF_GEN_OK;
}

// Result of the asynchronous check that decode_step leaves behind (see rlhf_gen_ctx::h_step_err).  `wait`: block
// until the copy has landed (callers that synchronise anyway); otherwise only look if it already has.
int take_step_error(rlhf_gen_ctx* c, bool wait) {
  if (!c->step_err_pending) return RLHF_GEN_OK;
  if (wait) {
    HIP_TRY(c, hipEventSynchronize(c->ev_step_err));
  } else {
    hipError_t q = hipEventQuery(c->ev_step_err);
    if (q == hipErrorNotReady) return RLHF_GEN_OK;
    if (q != hipSuccess) return fail(c, RLHF_GEN_E_DEVICE, "hipEventQuery failed: %s", hipGetErrorString(q));
  }
  c->step_err_pending = false;
  if (*c->h_step_err) {
    *c->h_step_err = 0;
    c->h_misc[0] = 0;
    HIP_TRY(c, hipMemcpyAsync(c->d_err, &c->h_misc[0], sizeof(int), hipMemcpyHostToDevice, c->stream));
    return fail(c, RLHF_GEN_E_INVALID,
                "a forced token id of an earlier decode step lay outside [0, vocab = %d); that step used the nearest valid id",
                c->cfg.vocab);
  }
  return RLHF_GEN_OK;
}

}  // namespace

extern "C" {

// Shape and capacity checks shared by rlhf_gen_init and the capacity planner.
static int validate_cfg(const rlhf_gen_cfg* cfg) {
  const rlhf_gen_cfg& g = *cfg;
  if (g.n_layers < 1 || g.d_model < 1 || g.n_heads < 1 || g.n_kv_heads < 1 || g.head_dim < 1 || g.d_ffn < 1 || g.vocab < 1)
    return fail(nullptr, RLHF_GEN_E_INVALID, "model dimensions must be positive");
  if (g.n_heads % g.n_kv_heads) return fail(nullptr, RLHF_GEN_E_INVALID, "n_heads must be a multiple of n_kv_heads");
  if (g.head_dim & 1) return fail(nullptr, RLHF_GEN_E_INVALID, "head_dim must be even");
  if (g.max_batch < 1 || g.max_seq < 2) return fail(nullptr, RLHF_GEN_E_INVALID, "max_batch >= 1 and max_seq >= 2 required");
  if (g.kv_block != 16) return fail(nullptr, RLHF_GEN_E_UNSUPPORTED, "kv_block must be 16 (got %d)", g.kv_block);
  if (g.dtype != RLHF_GEN_DTYPE_FP32 && g.dtype != RLHF_GEN_DTYPE_BF16)
    return fail(nullptr, RLHF_GEN_E_INVALID, "dtype must be 0 (fp32) or 1 (bf16)");
  if (!(g.rms_eps > 0.f) || !(g.rope_theta > 0.f)) return fail(nullptr, RLHF_GEN_E_INVALID, "rms_eps and rope_theta must be positive");
  if (g.kv_pool_blocks < 0) return fail(nullptr, RLHF_GEN_E_INVALID, "kv_pool_blocks must not be negative");
  if (g.d_model > 8192 || (g.d_model & 3)) return fail(nullptr, RLHF_GEN_E_UNSUPPORTED, "d_model must be a multiple of 4, at most 8192");
  const int qkv_w = (g.n_heads + 2 * g.n_kv_heads) * g.head_dim;
  if (g.dtype == RLHF_GEN_DTYPE_BF16) {
    if (g.head_dim != 128) return fail(nullptr, RLHF_GEN_E_UNSUPPORTED, "bf16 path needs head_dim 128 (got %d)", g.head_dim);
    if (g.n_heads / g.n_kv_heads > 16) return fail(nullptr, RLHF_GEN_E_UNSUPPORTED, "bf16 path supports at most 16 query heads per KV head");
    if (g.d_model % 256 || qkv_w % 256 || g.vocab % 256 || g.d_ffn % 128 || (g.n_heads * g.head_dim) % 128)
      return fail(nullptr, RLHF_GEN_E_UNSUPPORTED,
                  "bf16 path needs d_model, (n_heads + 2 n_kv_heads) head_dim and vocab to be multiples of 256 and d_ffn of 128");
  } else {
    if (g.head_dim != 32 && g.head_dim != 64 && g.head_dim != 128)
      return fail(nullptr, RLHF_GEN_E_UNSUPPORTED, "fp32 path supports head_dim 32, 64 or 128");
  }
  return RLHF_GEN_OK;
}

// One weight matrix [rows, cols] from the caller's bf16 row-major storage into the fp16 tiled working layout at dst,
// optionally with an adapter folded in.  dst == src (in-place mode) goes through the staging buffer in slabs of
// whole 16-row blocks: a slab's tiled image occupies exactly the bytes of its row-major rows.
constexpr int CONV_SLAB_ROWS = 1024;
static int convert_matrix(rlhf_gen_ctx* c, const void* src, void* dst, int rows, int cols, const rlhf_gen_lora_pair* pr,
                          float scale) {
  const void* A = pr ? pr->a : nullptr;
  const void* Bm = pr ? pr->b : nullptr;
  const int rank = pr ? pr->rank : 0;
  hipError_t e = hipSuccess;
  if (dst != src) {
    e = launch_to_h16_tiled(c->stream, src, 0, dst, rows, cols, A, Bm, rank, scale, 0);
  } else {
    if (!c->conv_tmp) return fail(c, RLHF_GEN_E_STATE, "in-place conversion without a staging buffer");
    for (int r0 = 0; r0 < rows && e == hipSuccess; r0 += CONV_SLAB_ROWS) {
      const int nr = std::min(CONV_SLAB_ROWS, rows - r0);
      char* slab = (char*)const_cast<void*>(src) + (size_t)r0 * cols * 2;
      e = launch_to_h16_tiled(c->stream, slab, 0, c->conv_tmp, nr, cols, A, Bm, rank, scale, r0);
      if (e == hipSuccess) e = hipMemcpyAsync(slab, c->conv_tmp, (size_t)nr * cols * 2, hipMemcpyDeviceToDevice, c->stream);
    }
  }
  if (e != hipSuccess) return fail(c, RLHF_GEN_E_DEVICE, "weight conversion failed: %s", hipGetErrorString(e));
  return RLHF_GEN_OK;
}

// 4-bit copies of layer l's pair-input projections, from their fp16 working copies.
static int convert_w4(rlhf_gen_ctx* c, int l) {
  const rlhf_gen_cfg& g = c->cfg;
  const int qkv_w = (g.n_heads + 2 * g.n_kv_heads) * g.head_dim, attn_w = g.n_heads * g.head_dim;
  LAUNCH(c, launch_to_w4_tiled(c->stream, c->wqkv[l], c->w4_qkv[l], c->ws_qkv[l], qkv_w, g.d_model), "to_w4_tiled qkv");
  LAUNCH(c, launch_to_w4_tiled(c->stream, c->wo[l], c->w4_wo[l], c->ws_wo[l], g.d_model, attn_w), "to_w4_tiled wo");
  return RLHF_GEN_OK;
}

// Every device and pinned-host allocation of a context, in one place.  With c->dry_run set nothing is allocated or
// launched and c->dev_bytes ends up as the context's device footprint.
static int allocate_all(rlhf_gen_ctx* c) {
  const rlhf_gen_cfg& g = c->cfg;
  const int qkv_w = (g.n_heads + 2 * g.n_kv_heads) * g.head_dim;
  auto bail = [&](int code) { return code; };
  c->max_blocks = blocks_for(g.max_seq);
  c->n_blocks = g.kv_pool_blocks ? g.kv_pool_blocks : g.max_batch * c->max_blocks;
  const size_t page_bytes = c->bf16 ? 8192 : (size_t)2 * 16 * g.head_dim * 4;
  c->layer_pool_bytes = (size_t)c->n_blocks * g.n_kv_heads * page_bytes;
  c->h_len.assign(g.max_batch, 0);
  c->n_alloc.assign(g.max_batch, 0);
  // activation rows: a prefill chunk holds whole sequences, so at least max_seq rows; 16384 keeps the
  // large GEMMs in their efficient regime while bounding the scratch
  c->act_rows = std::max(std::max(g.max_seq, g.max_batch), 16384);
  c->act_rows = (int)std::min<long long>(c->act_rows, std::max<long long>((long long)g.max_batch * g.max_seq, g.max_batch));
  c->act_rows = (c->act_rows + 255) / 256 * 256;
  const size_t rows = c->act_rows, as = act_size(c);
  const size_t total_tok = (size_t)g.max_batch * g.max_seq;
  const int half = g.head_dim / 2;
  int rc = RLHF_GEN_OK;
#define A_(expr) do { rc = (expr); if (rc) return bail(rc); } while (0)
  if (c->bf16) {
    // fp16 working copies of the projection matrices (or an in-place rewrite if the caller allows it)
    const bool in_place = (g.flags & RLHF_GEN_FLAG_CONVERT_IN_PLACE) != 0;
    if (in_place) {
      const int widest = std::max(std::max(g.d_model, g.d_ffn), g.n_heads * g.head_dim);
      A_(dev_alloc(c, &c->conv_tmp, (size_t)CONV_SLAB_ROWS * widest * 2, false));
    }
    auto convert = [&](const void* src, const void** dst, int rows, int cols) -> int {
      void* d = const_cast<void*>(src);
      if (!in_place) {
        char* fresh = nullptr;
        int r = dev_alloc(c, &fresh, (size_t)rows * cols * 2, false);
        if (r) return r;
        d = fresh;
      }
      *dst = d;
      return c->dry_run ? RLHF_GEN_OK : convert_matrix(c, src, d, rows, cols, nullptr, 0.f);
    };
    // the 4-bit low-half phase of the prefill GEMMs needs k extents that are multiples of 512 and whole 256-column tiles
    const int attn_w = g.n_heads * g.head_dim;
    c->lo4 = !(g.flags & RLHF_GEN_FLAG_PREFILL_FP16_PAIRS) && g.d_model % 512 == 0 && attn_w % 512 == 0 && qkv_w % 256 == 0 &&
             g.d_model % 256 == 0;
    c->w4_qkv.assign(g.n_layers, nullptr); c->w4_wo = c->ws_qkv = c->ws_wo = c->w4_qkv;
    for (int l = 0; l < g.n_layers; ++l) {
      A_(convert(c->src_wqkv[l], &c->wqkv[l], qkv_w, g.d_model));
      A_(convert(c->src_wo[l], &c->wo[l], g.d_model, attn_w));
      A_(convert(c->src_w_gate_up[l], &c->w_gate_up[l], 2 * g.d_ffn, g.d_model));
      A_(convert(c->src_w_down[l], &c->w_down[l], g.d_model, g.d_ffn));
      if (c->lo4) {
        A_(dev_alloc(c, &c->w4_qkv[l], (size_t)qkv_w * g.d_model / 2, false));
        A_(dev_alloc(c, &c->ws_qkv[l], (size_t)qkv_w, false));
        A_(dev_alloc(c, &c->w4_wo[l], (size_t)g.d_model * attn_w / 2, false));
        A_(dev_alloc(c, &c->ws_wo[l], (size_t)g.d_model, false));
        if (!c->dry_run) A_(convert_w4(c, l));
      }
    }
    A_(convert(c->src_lm_head, &c->lm_head, g.vocab, g.d_model));
  }
  A_(dev_alloc(c, &c->kv_pool, c->layer_pool_bytes * g.n_layers, true));
  A_(dev_alloc(c, &c->d_table, sizeof(int) * (size_t)g.max_batch * c->max_blocks, true));
  A_(dev_alloc(c, &c->d_seq_len, sizeof(int) * g.max_batch, true));
  A_(dev_alloc(c, &c->d_step, sizeof(int) * g.max_batch, true));
  A_(dev_alloc(c, &c->d_sargs, sizeof(SamplerArgs), true));
  A_(dev_alloc(c, &c->d_err, sizeof(int), true));
  A_(dev_alloc(c, &c->d_cur_tok, sizeof(int) * g.max_batch, true));
  A_(dev_alloc(c, &c->d_cos, sizeof(float) * (size_t)(g.max_seq + 1) * half, false));
  A_(dev_alloc(c, &c->d_sin, sizeof(float) * (size_t)(g.max_seq + 1) * half, false));
  A_(dev_alloc(c, &c->d_tok_seq, sizeof(int) * total_tok, true));
  A_(dev_alloc(c, &c->d_tok_pos, sizeof(int) * total_tok, true));
  A_(dev_alloc(c, &c->d_ids, sizeof(int) * total_tok, true));
  A_(dev_alloc(c, &c->d_cu, sizeof(int) * (2 * (size_t)g.max_batch + 2), true));
  A_(dev_alloc(c, &c->d_seq_ids, sizeof(int) * g.max_batch, true));
  A_(dev_alloc(c, &c->d_last_rows, sizeof(int) * g.max_batch, true));
  A_(dev_alloc(c, &c->x, 4 * rows * g.d_model, true));
  // fp32 q|k|v (and gate|up) rows of the fp32 path; the 16-bit path never materialises them
  A_(dev_alloc(c, &c->qkv, c->bf16 ? 16 : 4 * rows * std::max(qkv_w, 2 * g.d_ffn), true));
  A_(dev_alloc(c, &c->y, 2 * as * rows * g.d_model, true));              // room for hi|lo pairs
  A_(dev_alloc(c, &c->yl, as * ((size_t)g.max_batch + 256) * g.d_model, true));
  A_(dev_alloc(c, &c->qb, 2 * as * rows * g.n_heads * g.head_dim, true));
  A_(dev_alloc(c, &c->ab, 2 * as * rows * g.n_heads * g.head_dim, true));
  if (c->lo4) {
    // scale bytes of the activation rows' 4-bit low halves: one per (row, 128 columns), zero-filled (rows past the end of
    // a chunk are multiplied into output rows that are never stored)
    c->scale_groups = (int)(rows / 128);
    A_(dev_alloc(c, &c->a_scale, rows * (size_t)(std::max(g.d_model, g.n_heads * g.head_dim) / 128), true));
  }
  A_(dev_alloc(c, &c->hb, as * rows * g.d_ffn, true));
  A_(dev_alloc(c, &c->logits, 4 * (size_t)g.max_batch * g.vocab, true));
  c->score_cap = 1024;
  A_(dev_alloc(c, &c->d_srows, sizeof(int) * total_tok, true));
  A_(dev_alloc(c, &c->d_sslot, sizeof(int) * total_tok, true));
  A_(dev_alloc(c, &c->ys, as * ((size_t)c->score_cap + 256) * g.d_model, true));
  A_(dev_alloc(c, &c->slogits, 4 * (size_t)c->score_cap * g.vocab, true));
  if (c->bf16) {
    const int Bm = std::min(g.max_batch, 256);
    c->ks_qkv = gemm_skinny_pick_split(Bm, qkv_w, g.d_model, 1);
    c->ks_wo = gemm_skinny_pick_split(Bm, g.d_model, g.n_heads * g.head_dim, 1);
    c->ks_gu = gemm_skinny_pick_split(Bm, 2 * g.d_ffn, g.d_model);
    c->ks_down = gemm_skinny_pick_split(Bm, g.d_model, g.d_ffn);
    size_t pe = std::max(std::max((size_t)c->ks_qkv * qkv_w, (size_t)c->ks_wo * g.d_model),
                         std::max((size_t)c->ks_gu * 2 * g.d_ffn, (size_t)c->ks_down * g.d_model));
    const int attn_w = g.n_heads * g.head_dim;
    c->tile_ok = Bm > 128 && qkv_w % 256 == 0 && g.d_model % 256 == 0 && (2 * g.d_ffn) % 256 == 0 && attn_w % 128 == 0 &&
                 g.d_ffn % 128 == 0 && (size_t)2 * g.d_ffn * g.d_model * 2 < ((size_t)1 << 32) &&
                 (size_t)g.d_model * g.d_ffn * 2 < ((size_t)1 << 32) && (size_t)qkv_w * g.d_model * 2 < ((size_t)1 << 32);
    if (c->tile_ok) {
      const int l4 = c->lo4 && !(g.flags & RLHF_GEN_FLAG_FUSED_ROPE);
      c->kt_qkv = gemm_tiled_pick_split(Bm, qkv_w, g.d_model, 8, l4);   // (the fused RoPE + attention kernel takes up to 8 planes)
      c->kt_qkv = gemm_tiled_pick_split(Bm, qkv_w, g.d_model, 8, l4);   // (the fused RoPE + attention kernel takes up to 8 planes)
      c->kt_wo = gemm_tiled_pick_split(Bm, g.d_model, attn_w, 16, l4);
      c->kt_gu = gemm_tiled_pick_split(Bm, 2 * g.d_ffn, g.d_model);
      c->kt_down = gemm_tiled_pick_split(Bm, g.d_model, g.d_ffn);
      pe = std::max(pe, std::max(std::max((size_t)c->kt_qkv * qkv_w, (size_t)c->kt_wo * g.d_model),
                                 std::max((size_t)c->kt_gu * 2 * g.d_ffn, (size_t)c->kt_down * g.d_model)));
    }
    A_(dev_alloc(c, &c->part, 4 * pe * Bm, true));
  }
  A_(host_alloc(c, &c->h_tok_seq, sizeof(int) * total_tok));
  A_(host_alloc(c, &c->h_tok_pos, sizeof(int) * total_tok));
  A_(host_alloc(c, &c->h_cu, sizeof(int) * (2 * (size_t)g.max_batch + 2)));
  A_(host_alloc(c, &c->h_seq_ids, sizeof(int) * g.max_batch));
  A_(host_alloc(c, &c->h_last_rows, sizeof(int) * g.max_batch));
  A_(host_alloc(c, &c->h_table, sizeof(int) * (size_t)g.max_batch * c->max_blocks));
  A_(host_alloc(c, &c->h_lenbuf, sizeof(int) * g.max_batch));
  A_(host_alloc(c, &c->h_misc, sizeof(int) * 8));
  A_(host_alloc(c, &c->h_step_err, sizeof(int)));
  A_(host_alloc(c, &c->h_sargs, sizeof(SamplerArgs) * SARGS_RING));
  A_(host_alloc(c, &c->h_srows, sizeof(int) * total_tok));
  A_(host_alloc(c, &c->h_sslot, sizeof(int) * total_tok));
#undef A_
  return RLHF_GEN_OK;
}

int rlhf_gen_init(const rlhf_gen_weights* w, const rlhf_gen_cfg* cfg, rlhf_gen_ctx** out) {
  if (out) *out = nullptr;
  if (!w || !cfg || !out) return fail(nullptr, RLHF_GEN_E_INVALID, "NULL argument to rlhf_gen_init");
  {
    int vrc = validate_cfg(cfg);
    if (vrc) return vrc;
  }
  const rlhf_gen_cfg& g = *cfg;
  if (!w->tok_emb || !w->lm_head || !w->final_norm || !w->attn_norm || !w->wqkv || !w->wo || !w->ffn_norm ||
      !w->w_gate_up || !w->w_down)
    return fail(nullptr, RLHF_GEN_E_INVALID, "NULL weight pointer");
  for (int l = 0; l < g.n_layers; ++l)
    if (!w->attn_norm[l] || !w->wqkv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->w_gate_up[l] || !w->w_down[l])
      return fail(nullptr, RLHF_GEN_E_INVALID, "NULL weight pointer in layer %d", l);

  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || g.device < 0 || g.device >= ndev) {
    (void)hipGetLastError();
    return fail(nullptr, RLHF_GEN_E_DEVICE, "HIP device %d is not available (%d devices)", g.device, ndev);
  }
  rlhf_gen_ctx* c = new rlhf_gen_ctx();
  c->cfg = g;
  c->bf16 = g.dtype == RLHF_GEN_DTYPE_BF16;
  c->stream = (hipStream_t)g.stream;
  c->tok_emb = w->tok_emb;
  c->lm_head = w->lm_head;
  c->final_norm = w->final_norm;
  for (int l = 0; l < g.n_layers; ++l) {
    c->attn_norm.push_back(w->attn_norm[l]);
    c->wqkv.push_back(w->wqkv[l]);
    c->wo.push_back(w->wo[l]);
    c->ffn_norm.push_back(w->ffn_norm[l]);
    c->w_gate_up.push_back(w->w_gate_up[l]);
    c->w_down.push_back(w->w_down[l]);
  }
  c->src_wqkv = c->wqkv; c->src_wo = c->wo; c->src_w_gate_up = c->w_gate_up; c->src_w_down = c->w_down;
  c->src_lm_head = c->lm_head;
  auto bail = [&](int code) {
    g_init_error = c->err;
    rlhf_gen_destroy(c);
    return code;
  };
  if (hipSetDevice(g.device) != hipSuccess) {
    (void)hipGetLastError();
    c->err = "hipSetDevice failed";
    return bail(RLHF_GEN_E_DEVICE);
  }
  if (!c->stream) {
    // the legacy default stream cannot be captured into a graph: use a stream of our own (default priority)
    if (hipStreamCreate(&c->stream) != hipSuccess) {
      c->err = "hipStreamCreate failed";
      c->stream = nullptr;
      return bail(RLHF_GEN_E_DEVICE);
    }
    c->own_stream = true;
  }
  if (gemm_configure() != hipSuccess || sampler_configure() != hipSuccess || static_scratch_prepare() != hipSuccess) {
    (void)hipGetLastError();
    c->err = "kernel attribute setup failed";
    return bail(RLHF_GEN_E_DEVICE);
  }
  {
    int arc = allocate_all(c);
    if (arc) return bail(arc);
  }
  const int half = g.head_dim / 2;
  {
    // rotation tables in double, rounded once to fp32: angle = pos * theta^(-2i/h)
    std::vector<float> cs((size_t)(g.max_seq + 1) * half), sn((size_t)(g.max_seq + 1) * half);
    for (int p = 0; p <= g.max_seq; ++p)
      for (int i = 0; i < half; ++i) {
        double ang = (double)p * pow((double)g.rope_theta, -2.0 * i / g.head_dim);
        cs[(size_t)p * half + i] = (float)cos(ang);
        sn[(size_t)p * half + i] = (float)sin(ang);
      }
    if (hipMemcpy(c->d_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(c->d_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice) != hipSuccess) {
      c->err = "upload of the rotation tables failed";
      return bail(RLHF_GEN_E_DEVICE);
    }
  }
  for (int i = 0; i < 3; ++i)
    if (hipEventCreate(&c->ev[i]) != hipSuccess) {
      c->err = "hipEventCreate failed";
      return bail(RLHF_GEN_E_DEVICE);
    }
  if (hipEventCreateWithFlags(&c->ev_step_err, hipEventDisableTiming) != hipSuccess) {
    c->err = "hipEventCreate failed";
    return bail(RLHF_GEN_E_DEVICE);
  }
  reset_free_list(c);
  if (hipDeviceSynchronize() != hipSuccess) {
    c->err = "device synchronisation after init failed";
    return bail(RLHF_GEN_E_DEVICE);
  }
  *out = c;
  return RLHF_GEN_OK;
}

int rlhf_gen_prefill(rlhf_gen_ctx* c, const int32_t* query_tokens, const int32_t* lengths, int32_t B, int32_t Lmax,
                     const rlhf_gen_sampling* sampling, int32_t* tok_out, float* logprob_out) {
  if (!c) return RLHF_GEN_E_INVALID;
  c->reserve_extra = 0;
  c->win_lo = 0;
  return prefill_impl(c, query_tokens, lengths, B, Lmax, sampling, tok_out, logprob_out, 1);
}

int rlhf_gen_decode_step(rlhf_gen_ctx* c, const int32_t* forced_tokens, int32_t* tok_out, float* logprob_out) {
  if (!c) return RLHF_GEN_E_INVALID;
  if (!tok_out || !logprob_out) return fail(c, RLHF_GEN_E_INVALID, "NULL output pointer");
  HIP_TRY(c, hipSetDevice(c->cfg.device));
  int rc = take_step_error(c, false);
  if (rc) return rc;
  rc = decode_checks(c);
  if (rc) return rc;
  if (forced_tokens)
    HIP_TRY(c, hipMemcpyAsync(c->d_cur_tok, forced_tokens, sizeof(int) * c->B, hipMemcpyDeviceToDevice, c->stream));
  rc = enqueue_decode_body(c, tok_out, logprob_out, 1, 0, false);
  if (rc) return rc;
  after_step(c);
  if (forced_tokens) {
    // the embedding kernel has flagged ids outside the vocabulary; fetch the flag behind the step without waiting
    if (c->step_err_pending) HIP_TRY(c, hipEventSynchronize(c->ev_step_err));   // one pinned word: the previous copy must have landed
    HIP_TRY(c, hipMemcpyAsync(c->h_step_err, c->d_err, sizeof(int), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipEventRecord(c->ev_step_err, c->stream));
    c->step_err_pending = true;
  }
  return RLHF_GEN_OK;
}

static int generate_impl(rlhf_gen_ctx* c, const int32_t* query_tokens, const int32_t* lengths, int32_t B, int32_t Lmax,
                         int32_t R, const rlhf_gen_sampling* sampling, int32_t* resp_tokens, float* resp_logprobs) {
  if (R < 1) return fail(c, RLHF_GEN_E_INVALID, "max_resp_len = %d must be positive", R);
  HIP_TRY(c, hipSetDevice(c->cfg.device));
  c->win_lo = 0;
  c->reserve_extra = R - 1;
  hipStream_t s = c->stream;
  HIP_TRY(c, hipStreamSynchronize(s));
  c->sargs_next = 0;
  HIP_TRY(c, hipEventRecord(c->ev[0], s));
  int rc = prefill_impl(c, query_tokens, lengths, B, Lmax, sampling, resp_tokens, resp_logprobs, R);
  c->reserve_extra = 0;
  if (rc) return rc;
  HIP_TRY(c, hipEventRecord(c->ev[1], s));
  // the decode steps read the sampling rule and the output buffers from device memory
  rc = push_sampler_args(c, R, resp_tokens, resp_logprobs);
  if (rc) return rc;
  const bool use_graph = !(c->cfg.flags & RLHF_GEN_FLAG_NO_GRAPH) && R > 2;
  hipGraphExec_t graph_exec = nullptr;
  if (use_graph) {
    rc = decode_graph(c, B, &graph_exec);
    if (rc) return rc;
  }
  for (int t = 1; t < R; ++t) {
    rc = decode_checks(c);  // pages were reserved by prefill: never allocates here
    if (rc) return rc;
    const bool sampled = c->prof_every > 0 && t % c->prof_every == 0 && use_streaming(c, B) &&
                         c->prof_used + 16 * c->cfg.n_layers + 16 <= (int)c->prof_ev.size();
    if (use_graph && !sampled) {
      HIP_TRY(c, hipGraphLaunch(graph_exec, s));
    } else {
      c->prof_on = sampled;
      rc = enqueue_decode_body(c, nullptr, nullptr, 0, 0, true);
      c->prof_on = false;
      if (rc) return rc;
      if (sampled) {
        for (int b = 0; b < B; ++b) c->prof_attn_tokens += c->h_len[b] + 1;
        c->prof_steps++;
      }
    }
    after_step(c);
    if ((int)c->step_ev.size() < t) {
      hipEvent_t e = nullptr;
      HIP_TRY(c, hipEventCreate(&e));
      c->step_ev.push_back(e);
    }
    HIP_TRY(c, hipEventRecord(c->step_ev[t - 1], s));
  }
  HIP_TRY(c, hipEventRecord(c->ev[2], s));
  HIP_TRY(c, hipMemcpyAsync(&c->h_misc[2], c->d_err, sizeof(int), hipMemcpyDeviceToHost, s));
  HIP_TRY(c, hipStreamSynchronize(s));
  HIP_TRY(c, hipEventElapsedTime(&c->prefill_ms, c->ev[0], c->ev[1]));
  HIP_TRY(c, hipEventElapsedTime(&c->decode_ms, c->ev[1], c->ev[2]));
  c->decode_steps = R - 1;
  c->step_ms.assign(R - 1, 0.f);
  for (int t = 1; t < R; ++t)
    HIP_TRY(c, hipEventElapsedTime(&c->step_ms[t - 1], t == 1 ? c->ev[1] : c->step_ev[t - 2], c->step_ev[t - 1]));
  for (int i = 1; i < c->prof_used; ++i) {
    if (c->prof_cls[i] < 0) continue;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->prof_ev[i - 1], c->prof_ev[i]) == hipSuccess) {
      c->prof_ms[c->prof_cls[i]] += ms;
      c->prof_n[c->prof_cls[i]]++;
    }
  }
  c->prof_used = 0;
  if (c->h_misc[2]) return fail(c, RLHF_GEN_E_INVALID, "a token id outside [0, vocab) reached the embedding");
  return RLHF_GEN_OK;
}

int rlhf_gen_generate(rlhf_gen_ctx* c, const int32_t* query_tokens, const int32_t* lengths, int32_t B, int32_t Lmax,
                      int32_t R, const rlhf_gen_sampling* sampling, int32_t* resp_tokens, float* resp_logprobs) {
  if (!c) return RLHF_GEN_E_INVALID;
  c->row_offset = 0;
  return generate_impl(c, query_tokens, lengths, B, Lmax, R, sampling, resp_tokens, resp_logprobs);
}

int rlhf_gen_generate_stream(rlhf_gen_ctx* c, const int32_t* query_tokens, const int32_t* lengths, int32_t B, int32_t Lmax,
                             int32_t R, const rlhf_gen_sampling* sampling, int32_t* resp_tokens, float* resp_logprobs,
                             int32_t micro_batch, void* const* done_events, rlhf_gen_microbatch_fn on_ready, void* user) {
  if (!c) return RLHF_GEN_E_INVALID;
  if (!query_tokens || !lengths || !resp_tokens || !resp_logprobs) return fail(c, RLHF_GEN_E_INVALID, "NULL argument");
  if (B < 1 || Lmax < 1) return fail(c, RLHF_GEN_E_INVALID, "B = %d and Lmax = %d must be positive", B, Lmax);
  if (micro_batch < 1) return fail(c, RLHF_GEN_E_INVALID, "micro_batch = %d must be positive", micro_batch);
  micro_batch = std::min(micro_batch, B);
  if (micro_batch > c->cfg.max_batch)
    return fail(c, RLHF_GEN_E_INVALID, "micro-batches of %d rows exceed max_batch = %d", micro_batch, c->cfg.max_batch);
  HIP_TRY(c, hipSetDevice(c->cfg.device));
  float pre = 0.f, dec = 0.f;
  int steps = 0, rc = RLHF_GEN_OK, index = 0;
  for (int row0 = 0; row0 < B; row0 += micro_batch, ++index) {
    const int rows = std::min(micro_batch, B - row0);
    c->row_offset = row0;
    rc = generate_impl(c, query_tokens + (size_t)row0 * Lmax, lengths + row0, rows, Lmax, R, sampling,
                       resp_tokens + (size_t)row0 * R, resp_logprobs + (size_t)row0 * R);
    c->row_offset = 0;
    if (rc) return rc;
    pre += c->prefill_ms; dec += c->decode_ms; steps += c->decode_steps;
    void* ev = done_events ? done_events[index] : nullptr;
    if (ev) HIP_TRY(c, hipEventRecord((hipEvent_t)ev, c->stream));
    if (on_ready) on_ready(user, index, row0, rows, ev);
  }
  c->prefill_ms = pre; c->decode_ms = dec; c->decode_steps = steps;
  return RLHF_GEN_OK;
}

// When each micro-batch joins and leaves the running batch: a pure function of the lengths, the response length, the
// micro-batch size, the stagger and the number of KV pages, in units of decode steps.  Micro-batch i is admitted at the
// first step boundary at which (a) stagger steps have passed since the previous admission and (b) the pool has free
// pages for all of its rows to the end of their responses (pages of micro-batches that complete at that boundary count
// as free); it completes R - 1 decode steps later.  Shared by rlhf_gen_plan_admission and the rollout that executes it.
static int plan_admission(rlhf_gen_ctx* c, const int32_t* lengths, int B, int R, int micro_batch, int stagger, long pool_blocks,
                          std::vector<long>& admit, std::vector<long>& done, std::vector<long>& pages, int* peak_rows) {
  const int n_mb = (B + micro_batch - 1) / micro_batch;
  admit.assign(n_mb, 0); done.assign(n_mb, 0); pages.assign(n_mb, 0);
  for (int b = 0; b < B; ++b) {
    if (lengths[b] < 1) return fail(c, RLHF_GEN_E_INVALID, "lengths[%d] = %d must be positive", b, lengths[b]);
    pages[b / micro_batch] += blocks_for(lengths[b] + R - 1);
  }
  for (int i = 0; i < n_mb; ++i)
    if (pages[i] > pool_blocks)   // it could never be admitted
      return fail(c, RLHF_GEN_E_NOMEM, "KV pool has %ld pages, micro-batch %d alone needs %ld", pool_blocks, i, pages[i]);
  long free_pages = pool_blocks, step = 0, last_admit = 0;
  int front = 0, next = 0, peak = 0;
  while (front < n_mb) {
    for (bool moved = true; moved;) {
      moved = false;
      while (front < next && done[front] <= step) { free_pages += pages[front++]; moved = true; }
      while (next < n_mb && (next == 0 || step - last_admit >= stagger) && pages[next] <= free_pages) {
        admit[next] = step; done[next] = step + (R - 1); free_pages -= pages[next]; last_admit = step; ++next; moved = true;
      }
    }
    if (front == n_mb) break;
    const int rows = std::min(B, next * micro_batch) - front * micro_batch;
    peak = std::max(peak, rows);
    // the next boundary at which something changes: the front micro-batch completes, or the stagger lets the next one
    // in (with nothing running the pool is empty, so only the stagger holds the next one back)
    long next_event = front < next ? done[front] : last_admit + stagger;
    if (front < next && next < n_mb && pages[next] <= free_pages) next_event = std::min(next_event, last_admit + stagger);
    step = std::max(step + 1, next_event);
  }
  if (peak_rows) *peak_rows = peak;
  return RLHF_GEN_OK;
}

int rlhf_gen_plan_admission(const int32_t* lengths, int32_t B, int32_t max_resp_len, int32_t micro_batch, int32_t stagger_steps,
                            int32_t kv_pool_blocks, int32_t* admit_step, int32_t* done_step, int32_t* peak_rows) {
  if (!lengths || B < 1 || max_resp_len < 1 || micro_batch < 1 || stagger_steps < 0 || kv_pool_blocks < 1)
    return fail(nullptr, RLHF_GEN_E_INVALID, "rlhf_gen_plan_admission: NULL lengths or a size out of range");
  micro_batch = std::min(micro_batch, B);
  std::vector<long> admit, done, pages;
  int peak = 0;
  int rc = plan_admission(nullptr, lengths, B, max_resp_len, micro_batch, stagger_steps, kv_pool_blocks, admit, done, pages, &peak);
  if (rc) return rc;
  for (size_t i = 0; i < admit.size(); ++i) {
    if (admit_step) admit_step[i] = (int32_t)admit[i];
    if (done_step) done_step[i] = (int32_t)done[i];
  }
  if (peak_rows) *peak_rows = peak;
  return RLHF_GEN_OK;
}

int rlhf_gen_generate_continuous(rlhf_gen_ctx* c, const int32_t* query_tokens, const int32_t* lengths, int32_t B, int32_t Lmax,
                                 int32_t R, const rlhf_gen_sampling* sampling, int32_t* resp_tokens, float* resp_logprobs,
                                 int32_t micro_batch, int32_t stagger_steps, void* const* done_events,
                                 rlhf_gen_microbatch_fn on_ready, void* user) {
  if (!c) return RLHF_GEN_E_INVALID;
  const rlhf_gen_cfg& g = c->cfg;
  if (!query_tokens || !lengths || !resp_tokens || !resp_logprobs) return fail(c, RLHF_GEN_E_INVALID, "NULL argument");
  if (B < 1 || Lmax < 1 || R < 1) return fail(c, RLHF_GEN_E_INVALID, "B = %d, Lmax = %d and max_resp_len = %d must be positive", B, Lmax, R);
  if (B > g.max_batch)
    return fail(c, RLHF_GEN_E_INVALID, "B = %d exceeds max_batch = %d (every row of the batch keeps its own state row)", B, g.max_batch);
  if (micro_batch < 1 || stagger_steps < 0)
    return fail(c, RLHF_GEN_E_INVALID, "micro_batch = %d must be positive and stagger_steps = %d non-negative", micro_batch, stagger_steps);
  micro_batch = std::min(micro_batch, B);
  int rc = check_sampling(c, sampling);
  if (rc) return rc;
  for (int b = 0; b < B; ++b) {
    if (lengths[b] < 1 || lengths[b] > Lmax)
      return fail(c, RLHF_GEN_E_INVALID, "lengths[%d] = %d outside [1, Lmax = %d]", b, lengths[b], Lmax);
    if (lengths[b] + R - 1 > g.max_seq)
      return fail(c, RLHF_GEN_E_INVALID, "sequence %d: %d query + %d further tokens exceed max_seq = %d", b, lengths[b], R - 1, g.max_seq);
  }
  const int n_mb = (B + micro_batch - 1) / micro_batch;
  std::vector<long> admit, done, pages;
  int peak_rows = 0;
  rc = plan_admission(c, lengths, B, R, micro_batch, stagger_steps, c->n_blocks, admit, done, pages, &peak_rows);
  if (rc) return rc;
  HIP_TRY(c, hipSetDevice(g.device));
  hipStream_t s = c->stream;
  HIP_TRY(c, hipStreamSynchronize(s));
  c->sargs_next = 0;
  c->row_offset = 0;
  c->have_batch = c->have_logits = false;
  reset_free_list(c);
  c->h_misc[0] = 0;
  HIP_TRY(c, hipMemcpyAsync(c->d_err, &c->h_misc[0], sizeof(int), hipMemcpyHostToDevice, s));
  HIP_TRY(c, hipEventRecord(c->ev[0], s));
  const bool use_graph = !(g.flags & RLHF_GEN_FLAG_NO_GRAPH);
  float prefill_ms = 0.f;
  int front = 0, next = 0;   // micro-batches [front, next) are decoding
  long step = 0;             // decode steps enqueued so far
  auto row_of = [&](int mb) { return std::min(B, mb * micro_batch); };
  auto bail = [&](int code) { c->win_lo = 0; c->B = 0; c->have_batch = false; return code; };
  while (front < n_mb) {
    for (bool moved = true; moved;) {
      moved = false;
      while (front < next && done[front] <= step) {   // micro-batches at the front of the window that have all R tokens
        for (int b = row_of(front); b < row_of(front + 1); ++b) {   // their pages go back to the pool
          for (int k = 0; k < c->n_alloc[b]; ++k) c->free_list.push_back(c->h_table[(size_t)b * c->max_blocks + k]);
          c->n_alloc[b] = 0;
        }
        void* ev = done_events ? done_events[front] : nullptr;
        if (ev && hipEventRecord((hipEvent_t)ev, s) != hipSuccess) return bail(fail(c, RLHF_GEN_E_DEVICE, "hipEventRecord failed"));
        if (on_ready) on_ready(user, front, row_of(front), row_of(front + 1) - row_of(front), ev);
        ++front;
        moved = true;
      }
      while (next < n_mb && admit[next] <= step) {    // admissions due at this step boundary
        if (pages[next] > (long)c->free_list.size()) return bail(fail(c, RLHF_GEN_E_STATE, "admission plan and page pool disagree"));
        const int r0 = row_of(next), rows = row_of(next + 1) - r0;
        c->win_lo = r0;
        c->reserve_extra = R - 1;
        if (hipEventRecord(c->ev[1], s) != hipSuccess) return bail(fail(c, RLHF_GEN_E_DEVICE, "hipEventRecord failed"));
        rc = prefill_impl(c, query_tokens + (size_t)r0 * Lmax, lengths + r0, rows, Lmax, sampling, resp_tokens + (size_t)r0 * R,
                          resp_logprobs + (size_t)r0 * R, R, /*fresh=*/false);
        c->reserve_extra = 0;
        if (rc) return bail(rc);
        // (the next prefill synchronises the stream anyway; waiting here makes this one's time readable)
        float ms = 0.f;
        if (hipEventRecord(c->ev[2], s) != hipSuccess || hipEventSynchronize(c->ev[2]) != hipSuccess ||
            hipEventElapsedTime(&ms, c->ev[1], c->ev[2]) != hipSuccess)
          return bail(fail(c, RLHF_GEN_E_DEVICE, "timing the prefill of micro-batch %d failed", next));
        prefill_ms += ms;
        c->sargs_next = 0;
        ++next;
        moved = true;
      }
    }
    if (front == n_mb) break;
    // decode rows [front, next) up to the next boundary at which the plan changes the window
    if (front == next) {   // nothing is decoding and the stagger holds the next micro-batch back: skip to its admission
      step = admit[next];
      continue;
    }
    const long until = next < n_mb ? std::min(done[front], admit[next]) : done[front];
    const long run = until - step;
    if (run < 1) return bail(fail(c, RLHF_GEN_E_STATE, "admission plan stalled at step %ld", step));
    c->win_lo = row_of(front);
    c->B = row_of(next) - row_of(front);
    rc = push_sampler_args(c, R, resp_tokens, resp_logprobs);
    if (rc) return bail(rc);
    hipGraphExec_t graph_exec = nullptr;
    if (use_graph && run > 1 && (rc = decode_graph(c, c->B, &graph_exec))) return bail(rc);
    for (long k = 0; k < run; ++k) {
      if (graph_exec) {
        const hipError_t e = hipGraphLaunch(graph_exec, s);
        if (e != hipSuccess) return bail(fail(c, RLHF_GEN_E_DEVICE, "hipGraphLaunch failed: %s", hipGetErrorString(e)));
      } else if ((rc = enqueue_decode_body(c, nullptr, nullptr, 0, 0, true))) {
        return bail(rc);
      }
      after_step(c);
    }
    step = until;
  }
  c->win_lo = 0;
  c->B = 0;
  c->have_batch = c->have_logits = false;   // every row has its R tokens: there is nothing left to step
  HIP_TRY(c, hipEventRecord(c->ev[2], s));
  HIP_TRY(c, hipMemcpyAsync(&c->h_misc[2], c->d_err, sizeof(int), hipMemcpyDeviceToHost, s));
  HIP_TRY(c, hipStreamSynchronize(s));
  float total = 0.f;
  HIP_TRY(c, hipEventElapsedTime(&total, c->ev[0], c->ev[2]));
  c->prefill_ms = prefill_ms;
  c->decode_ms = total - prefill_ms;
  c->decode_steps = (int)step;
  c->step_ms.clear();
  c->peak_rows = peak_rows;
  if (c->h_misc[2]) return fail(c, RLHF_GEN_E_INVALID, "a token id outside [0, vocab) reached the embedding");
  return RLHF_GEN_OK;
}

int rlhf_gen_score(rlhf_gen_ctx* c, const int32_t* query_tokens, const int32_t* lengths, int32_t B, int32_t Lmax,
                   const int32_t* resp_tokens, int32_t R, float* logprobs_out) {
  if (!c) return RLHF_GEN_E_INVALID;
  return score_impl(c, query_tokens, lengths, B, Lmax, resp_tokens, R, logprobs_out);
}

int rlhf_gen_get_logits(rlhf_gen_ctx* c, float* out) {
  if (!c) return RLHF_GEN_E_INVALID;
  if (!out) return fail(c, RLHF_GEN_E_INVALID, "NULL output pointer");
  if (!c->have_logits) return fail(c, RLHF_GEN_E_STATE, "no step has produced logits yet");
  HIP_TRY(c, hipMemcpyAsync(out, c->logits, sizeof(float) * (size_t)c->B * c->cfg.vocab, hipMemcpyDeviceToDevice, c->stream));
  return take_step_error(c, true);
}

int rlhf_gen_last_timing(const rlhf_gen_ctx* c, float* prefill_ms, float* decode_ms, int32_t* decode_steps) {
  if (!c) return RLHF_GEN_E_INVALID;
  if (prefill_ms) *prefill_ms = c->prefill_ms;
  if (decode_ms) *decode_ms = c->decode_ms;
  if (decode_steps) *decode_steps = c->decode_steps;
  return RLHF_GEN_OK;
}

int rlhf_gen_last_step_ms(const rlhf_gen_ctx* c, float* ms_out, int32_t capacity, int32_t* n_out) {
  if (!c) return RLHF_GEN_E_INVALID;
  const int n = (int)c->step_ms.size();
  if (n_out) *n_out = n;
  if (ms_out)
    for (int i = 0; i < n && i < capacity; ++i) ms_out[i] = c->step_ms[i];
  return RLHF_GEN_OK;
}

int rlhf_gen_set_profile(rlhf_gen_ctx* c, int32_t every) {
  if (!c) return RLHF_GEN_E_INVALID;
  if (every < 0) return fail(c, RLHF_GEN_E_INVALID, "every must not be negative");
  HIP_TRY(c, hipSetDevice(c->cfg.device));
  c->prof_every = every;
  c->prof_used = 0;
  c->prof_attn_tokens = 0;
  c->prof_steps = 0;
  for (int i = 0; i < RLHF_GEN_PROF_CLASSES; ++i) { c->prof_ms[i] = 0; c->prof_n[i] = 0; }
  if (every > 0 && c->prof_ev.empty()) {
    const int want = 16 * (16 * c->cfg.n_layers + 16);  // up to 16 sampled steps per generate
    c->prof_ev.reserve(want);
    for (int i = 0; i < want; ++i) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) break;
      c->prof_ev.push_back(e);
    }
    c->prof_cls.assign(c->prof_ev.size(), -1);
  }
  return RLHF_GEN_OK;
}

int rlhf_gen_get_profile(const rlhf_gen_ctx* c, double* ms, int64_t* launches, int64_t* attn_tokens, int32_t* steps) {
  if (!c) return RLHF_GEN_E_INVALID;
  for (int i = 0; i < RLHF_GEN_PROF_CLASSES; ++i) {
    if (ms) ms[i] = c->prof_ms[i];
    if (launches) launches[i] = c->prof_n[i];
  }
  if (attn_tokens) *attn_tokens = c->prof_attn_tokens;
  if (steps) *steps = c->prof_steps;
  return RLHF_GEN_OK;
}

const char* rlhf_gen_last_error(const rlhf_gen_ctx* c) { return c ? c->err.c_str() : g_init_error.c_str(); }

int64_t rlhf_gen_context_bytes(const rlhf_gen_ctx* c) { return c ? (int64_t)c->dev_bytes : 0; }

int64_t rlhf_gen_graph_captures(const rlhf_gen_ctx* c) { return c ? (int64_t)c->graph_captures : 0; }

int32_t rlhf_gen_last_peak_rows(const rlhf_gen_ctx* c) { return c ? c->peak_rows : 0; }

int rlhf_gen_plan_capacity(const rlhf_gen_cfg* cfg, int64_t capacity_bytes, double fraction, int64_t reserved_bytes,
                           int32_t* max_batch_out, int64_t* context_bytes_out) {
  if (!cfg || !max_batch_out) return fail(nullptr, RLHF_GEN_E_INVALID, "NULL argument to rlhf_gen_plan_capacity");
  if (!(fraction > 0.0) || fraction > 1.0) return fail(nullptr, RLHF_GEN_E_INVALID, "fraction must be in (0, 1]");
  if (capacity_bytes < 0) return fail(nullptr, RLHF_GEN_E_INVALID, "capacity_bytes must not be negative");
  rlhf_gen_cfg g = *cfg;
  g.max_batch = 1;
  int rc = validate_cfg(&g);
  if (rc) return rc;
  if (g.kv_pool_blocks != 0)
    return fail(nullptr, RLHF_GEN_E_INVALID, "the planner sizes the KV pool itself: kv_pool_blocks must be 0");
  if (capacity_bytes == 0) {
    size_t free_b = 0, total_b = 0;
    if (hipSetDevice(g.device) != hipSuccess || hipMemGetInfo(&free_b, &total_b) != hipSuccess) {
      (void)hipGetLastError();
      return fail(nullptr, RLHF_GEN_E_DEVICE, "cannot query the memory of HIP device %d", g.device);
    }
    capacity_bytes = (int64_t)total_b;
  }
  if (reserved_bytes < 0) {
    // the caller's own copy of the model in cfg.dtype
    const size_t es = g.dtype == RLHF_GEN_DTYPE_BF16 ? 2 : 4;
    const size_t qkv_w = (size_t)(g.n_heads + 2 * g.n_kv_heads) * g.head_dim;
    const size_t per_layer = qkv_w * g.d_model + (size_t)g.d_model * g.n_heads * g.head_dim + (size_t)3 * g.d_ffn * g.d_model +
                             (size_t)2 * g.d_model;
    reserved_bytes = (int64_t)(es * (per_layer * g.n_layers + (size_t)2 * g.vocab * g.d_model + g.d_model));
  }
  const double budget = fraction * (double)capacity_bytes - (double)reserved_bytes;
  auto footprint = [&](int B) -> int64_t {
    rlhf_gen_ctx tmp;
    tmp.cfg = g;
    tmp.cfg.max_batch = B;
    tmp.bf16 = g.dtype == RLHF_GEN_DTYPE_BF16;
    tmp.dry_run = true;
    tmp.src_wqkv.assign(g.n_layers, nullptr); tmp.src_wo = tmp.src_w_gate_up = tmp.src_w_down = tmp.src_wqkv;
    tmp.wqkv = tmp.wo = tmp.w_gate_up = tmp.w_down = tmp.src_wqkv;
    if (allocate_all(&tmp)) return INT64_MAX;
    return (int64_t)tmp.dev_bytes;
  };
  // the footprint grows with B: bisect for the largest batch within the budget
  const int blocks = (g.max_seq + 15) / 16;
  int hi = (int)std::min<long long>(1 << 20, std::min<long long>((1ll << 30) / g.max_seq, (1ll << 30) / blocks));
  int lo = 0;  // largest batch known to fit (0: none)
  if ((double)footprint(1) <= budget) {
    lo = 1;
    if ((double)footprint(hi) <= budget) lo = hi;
    while (hi - lo > 1 && lo != hi) {
      int mid = lo + (hi - lo) / 2;
      if ((double)footprint(mid) <= budget) lo = mid; else hi = mid;
    }
  }
  *max_batch_out = lo;
  if (context_bytes_out) *context_bytes_out = lo ? footprint(lo) : 0;
  return RLHF_GEN_OK;
}

int rlhf_gen_update_weights(rlhf_gen_ctx* c, const rlhf_gen_weights* w, const rlhf_gen_lora* lora) {
  if (!c) return RLHF_GEN_E_INVALID;
  if (!w) return fail(c, RLHF_GEN_E_INVALID, "NULL weights");
  const rlhf_gen_cfg& g = c->cfg;
  if (!w->tok_emb || !w->lm_head || !w->final_norm || !w->attn_norm || !w->wqkv || !w->wo || !w->ffn_norm ||
      !w->w_gate_up || !w->w_down)
    return fail(c, RLHF_GEN_E_INVALID, "NULL weight pointer");
  for (int l = 0; l < g.n_layers; ++l)
    if (!w->attn_norm[l] || !w->wqkv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->w_gate_up[l] || !w->w_down[l])
      return fail(c, RLHF_GEN_E_INVALID, "NULL weight pointer in layer %d", l);
  // adapters: validate everything before the first kernel is enqueued
  auto pair_of = [&](const rlhf_gen_lora_pair* arr, int l) -> const rlhf_gen_lora_pair* {
    return (lora && arr && arr[l].a) ? &arr[l] : nullptr;
  };
  bool any_lora = false;
  if (lora) {
    const rlhf_gen_lora_pair* arrs[4] = {lora->wqkv, lora->wo, lora->w_gate_up, lora->w_down};
    for (int l = 0; l <= g.n_layers; ++l)
      for (int m = 0; m < (l < g.n_layers ? 4 : 1); ++m) {
        const rlhf_gen_lora_pair* pr = l < g.n_layers ? pair_of(arrs[m], l) : (lora->lm_head.a ? &lora->lm_head : nullptr);
        if (!pr) continue;
        if (!pr->b) return fail(c, RLHF_GEN_E_INVALID, "adapter with A but no B");
        if (pr->rank < 1 || pr->rank > 64) return fail(c, RLHF_GEN_E_INVALID, "adapter rank must be in 1..64 (got %d)", pr->rank);
        any_lora = true;
      }
    if (any_lora && !(lora->scale == lora->scale)) return fail(c, RLHF_GEN_E_INVALID, "adapter scale is NaN");
  }
  if (any_lora && !c->bf16)
    return fail(c, RLHF_GEN_E_UNSUPPORTED, "the fp32 path reads the caller's matrices in place and cannot fold adapters");
  HIP_TRY(c, hipSetDevice(g.device));

  bool moved = c->tok_emb != w->tok_emb || c->final_norm != w->final_norm;
  for (int l = 0; l < g.n_layers; ++l) moved = moved || c->attn_norm[l] != w->attn_norm[l] || c->ffn_norm[l] != w->ffn_norm[l];
  const int qkv_w = (g.n_heads + 2 * g.n_kv_heads) * g.head_dim;
  if (c->bf16) {
    const bool in_place = (g.flags & RLHF_GEN_FLAG_CONVERT_IN_PLACE) != 0;
    auto refresh = [&](const void* src, const void** work, int rows, int cols, const rlhf_gen_lora_pair* pr) -> int {
      void* dst = in_place ? const_cast<void*>(src) : const_cast<void*>(*work);
      int r = convert_matrix(c, src, dst, rows, cols, pr, lora ? lora->scale : 0.f);
      if (r) return r;
      if (*work != dst) moved = true;
      *work = dst;
      return RLHF_GEN_OK;
    };
    int rc;
    for (int l = 0; l < g.n_layers; ++l) {
      if ((rc = refresh(w->wqkv[l], &c->wqkv[l], qkv_w, g.d_model, pair_of(lora ? lora->wqkv : nullptr, l)))) return rc;
      if ((rc = refresh(w->wo[l], &c->wo[l], g.d_model, g.n_heads * g.head_dim, pair_of(lora ? lora->wo : nullptr, l)))) return rc;
      if ((rc = refresh(w->w_gate_up[l], &c->w_gate_up[l], 2 * g.d_ffn, g.d_model, pair_of(lora ? lora->w_gate_up : nullptr, l)))) return rc;
      if ((rc = refresh(w->w_down[l], &c->w_down[l], g.d_model, g.d_ffn, pair_of(lora ? lora->w_down : nullptr, l)))) return rc;
      c->src_wqkv[l] = w->wqkv[l]; c->src_wo[l] = w->wo[l]; c->src_w_gate_up[l] = w->w_gate_up[l]; c->src_w_down[l] = w->w_down[l];
      if (c->lo4 && (rc = convert_w4(c, l))) return rc;
    }
    if ((rc = refresh(w->lm_head, &c->lm_head, g.vocab, g.d_model, (lora && lora->lm_head.a) ? &lora->lm_head : nullptr))) return rc;
    c->src_lm_head = w->lm_head;
  } else {
    moved = moved || c->lm_head != w->lm_head;
    for (int l = 0; l < g.n_layers; ++l) {
      moved = moved || c->wqkv[l] != w->wqkv[l] || c->wo[l] != w->wo[l] || c->w_gate_up[l] != w->w_gate_up[l] ||
              c->w_down[l] != w->w_down[l];
      c->wqkv[l] = w->wqkv[l]; c->wo[l] = w->wo[l]; c->w_gate_up[l] = w->w_gate_up[l]; c->w_down[l] = w->w_down[l];
    }
    c->lm_head = w->lm_head;
  }
  c->tok_emb = w->tok_emb;
  c->final_norm = w->final_norm;
  for (int l = 0; l < g.n_layers; ++l) { c->attn_norm[l] = w->attn_norm[l]; c->ffn_norm[l] = w->ffn_norm[l]; }
  // a captured decode graph holds the addresses it was recorded with: it survives unless one of them changed
  if (moved) drop_graph(c);
  // whatever the KV cache holds was computed with the old weights
  c->have_batch = false;
  c->have_logits = false;
  return RLHF_GEN_OK;
}

void rlhf_gen_destroy(rlhf_gen_ctx* c) {
  if (!c) return;
  (void)hipSetDevice(c->cfg.device);
  if (c->stream || !c->allocs.empty()) (void)hipStreamSynchronize(c->stream);
  drop_graph(c);
  for (void* p : c->allocs) (void)hipFree(p);
  int* pinned[] = {c->h_tok_seq, c->h_tok_pos, c->h_cu, c->h_seq_ids, c->h_last_rows, c->h_table, c->h_lenbuf, c->h_misc,
                   c->h_srows, c->h_sslot};
  for (int* p : pinned)
    if (p) (void)hipHostFree(p);
  for (int i = 0; i < 3; ++i)
    if (c->ev[i]) (void)hipEventDestroy(c->ev[i]);
  if (c->ev_step_err) (void)hipEventDestroy(c->ev_step_err);
  if (c->h_step_err) (void)hipHostFree(c->h_step_err);
  if (c->h_sargs) (void)hipHostFree(c->h_sargs);
  for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->step_ev) (void)hipEventDestroy(e);
  if (c->own_stream && c->stream) (void)hipStreamDestroy(c->stream);
  delete c;
}

// ---- single-operation entry points (kernel parity tests) ----------------------------------------
int rlhf_gen_op_probe_stream_read(void* stream, const void* buf, int64_t bytes, int32_t nontemporal, void* scratch) {
  if (!buf || !scratch || bytes < 8192) return RLHF_GEN_E_INVALID;
  return launch_probe_stream_read((hipStream_t)stream, buf, (size_t)bytes, nontemporal, scratch) == hipSuccess ? RLHF_GEN_OK
                                                                                                             : RLHF_GEN_E_DEVICE;
}

int rlhf_gen_op_probe_mfma_loop(void* stream, const void* operands, int32_t workgroups, int32_t iters, void* scratch) {
  if (!operands || !scratch || workgroups < 1 || iters < 1) return RLHF_GEN_E_INVALID;
  return launch_probe_mfma_loop((hipStream_t)stream, operands, workgroups, iters, scratch) == hipSuccess ? RLHF_GEN_OK
                                                                                                         : RLHF_GEN_E_DEVICE;
}

int rlhf_gen_op_tile_weights(void* stream, const void* w_rowmajor, void* w_tiled, int32_t N, int32_t K) {
  if (!w_rowmajor || !w_tiled || w_rowmajor == w_tiled || N < 16 || K < 128 || N % 16 || K % 128) return RLHF_GEN_E_INVALID;
  hipError_t e = launch_to_h16_tiled((hipStream_t)stream, w_rowmajor, 1, w_tiled, N, K, nullptr, nullptr, 0, 0.f, 0);
  return e == hipSuccess ? RLHF_GEN_OK : RLHF_GEN_E_DEVICE;
}

int rlhf_gen_op_gemm(void* stream, int kind, const void* A, const void* W, void* out, int32_t M, int32_t N, int32_t K,
                     int32_t epilogue, int32_t nsplit, int32_t a_pairs) {
  hipStream_t s = (hipStream_t)stream;
  hipError_t e;
  if (!A || !W || !out || M < 1 || N < 1 || K < 1) return RLHF_GEN_E_INVALID;
  static bool configured = false;
  if (!configured) {
    if (gemm_configure() != hipSuccess) return RLHF_GEN_E_DEVICE;
    configured = true;
  }
  if (kind == RLHF_GEN_GEMM_TILED)
    e = (nsplit > 1 && epilogue == EPI_STORE_F32) ? launch_gemm_h16_splitk(s, A, W, (float*)out, M, N, K, a_pairs, nsplit, 0)
                                                  : launch_gemm_h16(s, A, W, out, M, N, K, epilogue, a_pairs);
  else if (kind == RLHF_GEN_GEMM_STREAMING)
    e = launch_gemm_skinny_h16(s, A, W, (float*)out, M, epilogue == EPI_SWIGLU ? 2 * N : N, K,
                               epilogue == EPI_SWIGLU ? 0 : nsplit, a_pairs);
  else if (kind == RLHF_GEN_GEMM_FP32) e = launch_gemm_f32(s, (const float*)A, (const float*)W, (float*)out, M, N, K, epilogue == EPI_RESID_F32);
  else return RLHF_GEN_E_INVALID;
  if (e == hipErrorInvalidValue) return RLHF_GEN_E_UNSUPPORTED;
  return e == hipSuccess ? RLHF_GEN_OK : RLHF_GEN_E_DEVICE;
}

int rlhf_gen_op_tile_weights4(void* stream, const void* w_tiled, void* w4, void* w_scale, int32_t N, int32_t K) {
  if (!w_tiled || !w4 || !w_scale || N < 16 || K < 512 || N % 16 || K % 512) return RLHF_GEN_E_INVALID;
  hipError_t e = launch_to_w4_tiled((hipStream_t)stream, w_tiled, w4, w_scale, N, K);
  return e == hipSuccess ? RLHF_GEN_OK : RLHF_GEN_E_DEVICE;
}

int rlhf_gen_op_rmsnorm_lo4(void* stream, const float* x, const void* gain_bf16, void* y, void* row_scale, int32_t scale_groups,
                            int32_t M, int32_t d, float eps) {
  if (!x || !gain_bf16 || !y || !row_scale || M < 1 || d < 128 || d > 8192 || d % 128 || scale_groups < (M + 127) / 128)
    return RLHF_GEN_E_INVALID;
  // (the kernel writes x back only when it adds partial sums, which this call never passes)
  hipError_t e = launch_rmsnorm((hipStream_t)stream, const_cast<float*>(x), nullptr, 0, 0, gain_bf16, 1, y, 1, M, d, eps, nullptr, 2,
                                row_scale, scale_groups);
  if (e == hipErrorInvalidValue) return RLHF_GEN_E_UNSUPPORTED;
  return e == hipSuccess ? RLHF_GEN_OK : RLHF_GEN_E_DEVICE;
}

int rlhf_gen_op_gemm_lo4(void* stream, const void* A, const void* W, const void* W4, const void* w_scale, const void* a_scale,
                         int32_t scale_groups, float* out, int32_t M, int32_t N, int32_t K, int32_t epilogue) {
  if (!A || !W || !W4 || !w_scale || !a_scale || !out || M < 1 || N < 1 || K < 1) return RLHF_GEN_E_INVALID;
  if (epilogue != EPI_STORE_F32 && epilogue != EPI_RESID_F32) return RLHF_GEN_E_INVALID;
  static bool configured = false;
  if (!configured) {
    if (gemm_configure() != hipSuccess) return RLHF_GEN_E_DEVICE;
    configured = true;
  }
  hipError_t e = launch_gemm_h16_lo4((hipStream_t)stream, A, W, W4, w_scale, a_scale, scale_groups, out, M, N, K, epilogue, nullptr);
  if (e == hipErrorInvalidValue) return RLHF_GEN_E_UNSUPPORTED;
  return e == hipSuccess ? RLHF_GEN_OK : RLHF_GEN_E_DEVICE;
}

int rlhf_gen_op_rope_append(void* stream, const float* qkv, const int32_t* row_pos, const int32_t* row_seq,
                            const float* cos_t, const float* sin_t, void* q_out, void* kv_pool,
                            const int32_t* block_table, int32_t max_blocks, int32_t n_blocks, int32_t M, int32_t Hq,
                            int32_t Hkv, int32_t head_dim, int32_t half16) {
  if (!qkv || !row_pos || !cos_t || !sin_t || !q_out || !kv_pool || !block_table) return RLHF_GEN_E_INVALID;
  hipError_t e = launch_rope_append((hipStream_t)stream, qkv, nullptr, 0, 0, row_pos, row_seq, cos_t, sin_t, q_out, kv_pool,
                                    block_table, max_blocks, n_blocks, M, Hq, Hkv, head_dim, half16);
  if (e == hipErrorInvalidValue) return RLHF_GEN_E_UNSUPPORTED;
  return e == hipSuccess ? RLHF_GEN_OK : RLHF_GEN_E_DEVICE;
}

int rlhf_gen_op_attn_decode(void* stream, const void* q, const void* kv_pool, const int32_t* block_table,
                            int32_t max_blocks, int32_t n_blocks, const int32_t* seq_len, void* out, int32_t B, int32_t Hq,
                            int32_t Hkv) {
  if (!q || !kv_pool || !block_table || !seq_len || !out) return RLHF_GEN_E_INVALID;
  hipError_t e = launch_attn_decode_h16((hipStream_t)stream, q, kv_pool, block_table, max_blocks, n_blocks, seq_len, out, B, Hq, Hkv);
  if (e == hipErrorInvalidValue) return RLHF_GEN_E_UNSUPPORTED;
  return e == hipSuccess ? RLHF_GEN_OK : RLHF_GEN_E_DEVICE;
}

int rlhf_gen_op_attn_prefill(void* stream, const void* q, const void* kv_pool, const int32_t* block_table,
                             int32_t max_blocks, int32_t n_blocks, const int32_t* cu_seqlens, const int32_t* seq_ids, void* out,
                             int32_t nseq, int32_t max_len, int32_t Hq, int32_t Hkv) {
  if (!q || !kv_pool || !block_table || !cu_seqlens || !seq_ids || !out) return RLHF_GEN_E_INVALID;
  hipError_t e = launch_attn_prefill_h16((hipStream_t)stream, q, kv_pool, block_table, max_blocks, n_blocks, cu_seqlens, seq_ids, out,
                                          nseq, max_len, Hq, Hkv);
  if (e == hipErrorInvalidValue) return RLHF_GEN_E_UNSUPPORTED;
  return e == hipSuccess ? RLHF_GEN_OK : RLHF_GEN_E_DEVICE;
}

int rlhf_gen_op_attn_decode_lo4(void* stream, const void* q, const void* kv_pool, const int32_t* block_table,
                                int32_t max_blocks, int32_t n_blocks, const int32_t* seq_len, void* out, void* row_scale,
                                int32_t scale_groups, int32_t B, int32_t Hq, int32_t Hkv) {
  if (!q || !kv_pool || !block_table || !seq_len || !out || !row_scale || scale_groups < 1) return RLHF_GEN_E_INVALID;
  hipError_t e = launch_attn_decode_h16((hipStream_t)stream, q, kv_pool, block_table, max_blocks, n_blocks, seq_len, out, B, Hq, Hkv,
                                         row_scale, scale_groups);
  if (e == hipErrorInvalidValue) return RLHF_GEN_E_UNSUPPORTED;
  return e == hipSuccess ? RLHF_GEN_OK : RLHF_GEN_E_DEVICE;
}

int rlhf_gen_op_attn_prefill_lo4(void* stream, const void* q, const void* kv_pool, const int32_t* block_table,
                                 int32_t max_blocks, int32_t n_blocks, const int32_t* cu_seqlens, const int32_t* seq_ids, void* out,
                                 void* row_scale, int32_t scale_groups, int32_t nseq, int32_t max_len, int32_t Hq, int32_t Hkv) {
  if (!q || !kv_pool || !block_table || !cu_seqlens || !seq_ids || !out || !row_scale || scale_groups < 1) return RLHF_GEN_E_INVALID;
  if ((int64_t)nseq * max_len > (int64_t)128 * scale_groups) return RLHF_GEN_E_INVALID;   // (an upper bound of the number of rows)
  hipError_t e = launch_attn_prefill_h16((hipStream_t)stream, q, kv_pool, block_table, max_blocks, n_blocks, cu_seqlens, seq_ids, out,
                                          nseq, max_len, Hq, Hkv, row_scale, scale_groups);
  if (e == hipErrorInvalidValue) return RLHF_GEN_E_UNSUPPORTED;
  return e == hipSuccess ? RLHF_GEN_OK : RLHF_GEN_E_DEVICE;
}

int rlhf_gen_op_sample(void* stream, const float* logits, int32_t B, int32_t V, const rlhf_gen_sampling* sp,
                       const int32_t* step, int32_t* tok_out, float* logprob_out, int32_t* scratch_tok) {
  if (!logits || !sp || !step || !tok_out || !logprob_out || !scratch_tok || B < 1 || V < 1) return RLHF_GEN_E_INVALID;
  static bool configured = false;
  if (!configured) {
    if (sampler_configure() != hipSuccess) return RLHF_GEN_E_DEVICE;
    configured = true;
  }
  SamplerArgs p{};
  p.temperature = sp->temperature; p.top_p = sp->top_p; p.seed = sp->seed; p.greedy = sp->greedy; p.logprob_mode = sp->logprob_mode;
  p.out_stride = 1; p.tok_out = tok_out; p.lp_out = logprob_out;   // one response index for all rows, results in column 0
  hipError_t e = launch_sampler((hipStream_t)stream, logits, B, V, p, nullptr, step, scratch_tok);
  return e == hipSuccess ? RLHF_GEN_OK : RLHF_GEN_E_DEVICE;
}

}  // extern "C"
