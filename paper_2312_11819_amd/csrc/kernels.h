// Host-callable launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

enum GemmEpilogue {
  EPI_STORE_F32 = 0,   // out fp32 [M, N] = acc
  EPI_RESID_F32 = 1,   // out fp32 [M, N] += acc
  EPI_SWIGLU = 2,      // W is [2F, K] (gate rows then up rows), N = F: out [M, F] = silu(gate) * up
  EPI_STORE_ACT = 3,   // out [M, N] in the activation type (fp16 on the MFMA path)
  EPI_QKV_ROPE = 4     // W is the fused q|k|v projection: rotate q and k by the row's position, write the query pairs and
                       // append k / v to the paged cache (launch_gemm_h16_qkv_rope); nothing else is stored
};

// ---- 16-bit MFMA path (fp16 operands, fp32 accumulation) ----
// Large-tile GEMM: out = A[M,K] (fp16) * W[N,K]^T (fp16).  Needs N % 256 == 0 (F % 128 == 0 for SWIGLU),
// K % 128 == 0, W in the tiled working layout (common.h); rows of A beyond M are never read.  a_dual: A is [M, 2K], each row = [hi (K) | lo (K)], and
// out = (hi + lo) W^T.
hipError_t launch_gemm_h16(hipStream_t s, const void* A, const void* W, void* out, int M, int N, int K, int epi,
                           int a_dual);
// The QKV projection of prefill with the rotary embedding and the cache append as its epilogue: the fp32 q|k|v rows are
// never written (at 16384 rows of the 7B shape that is 0.8 GB out and back in per layer, plus a kernel of 1.5 M
// workgroups).  A wavefront's 128 output columns are one head, and a lane holds dimensions 2c, 2c + 1 and their partners
// 64 + 2c, 64 + 2c + 1 of it, so the rotation happens in registers.  A fp16 [M, 2K] hi|lo pairs, W the [(Hq + 2 Hkv) 128, K]
// matrix in the working layout; row_pos [M] position of each row, row_seq [M] its block-table row (NULL = identity);
// q_out fp16 [M, Hq, 2, 128].
struct RopeEpi {
  const int* row_pos;
  const int* row_seq;
  const float* cos_t;      // [positions, 64]
  const float* sin_t;
  void* q_out;
  void* kv_pool_layer;
  const int* block_table;
  int max_blocks, n_blocks, Hq, Hkv;
};
hipError_t launch_gemm_h16_qkv_rope(hipStream_t s, const void* A, const void* W, int M, int K, const RopeEpi& re);
// The large-tile GEMM with the low halves of A in the 4-bit side format (common.h): A rows are [hi (K) | lo4 (K / 2
// bytes) | unused] at a pitch of 2 K halves, a_scale their scale bytes (fp4_row_scale_offset order over scale_groups
// 128-row groups, scale_groups >= 2 ceil(M / 256)), W the tiled fp16 matrix, W4 / w_scale its 4-bit copy
// (launch_to_w4_tiled).  out = hi W^T + lo4 W4^T with epi EPI_STORE_F32 / EPI_RESID_F32, or the QKV form (EPI_QKV_ROPE,
// re as in launch_gemm_h16_qkv_rope, out unused).  K % 512 == 0, N % 256 == 0.
hipError_t launch_gemm_h16_lo4(hipStream_t s, const void* A, const void* W, const void* W4, const void* w_scale,
                               const void* a_scale, int scale_groups, void* out, int M, int N, int K, int epi, const RopeEpi* re);
// Split-K form of the large-tile GEMM for a few hundred rows: fp32 partial sums part[ks][plane_rows][N], ks < nsplit
// (no split may be empty: take nsplit from gemm_tiled_pick_split), N % 256 == 0, K % 128 == 0; the consumer adds the planes.
hipError_t launch_gemm_h16_splitk(hipStream_t s, const void* A, const void* W, float* part, int M, int N, int K, int a_dual,
                                  int nsplit, int plane_rows = 0);
int gemm_tiled_pick_split(int M, int N, int K, int max_splits = 16, int lo4 = 0);
// The same with the low halves of A in the 4-bit side format (launch_gemm_h16_lo4); nsplit from
// gemm_tiled_pick_split(..., lo4 = 1): the splits begin at multiples of 128 columns.  K % 512 == 0.
hipError_t launch_gemm_h16_splitk_lo4(hipStream_t s, const void* A, const void* W, const void* W4, const void* w_scale,
                                      const void* a_scale, int scale_groups, float* part, int M, int N, int K, int nsplit,
                                      int plane_rows = 0);
// Weight-streaming GEMM for M <= 256 rows: writes fp32 partial sums part[ks][M][Nw] (Nw = rows of W)
// for ks < nsplit; the consumer kernel adds them.  nsplit = 0 selects the fused SwiGLU form: W = [2F, K]
// (gate rows, then up rows; Nw = 2F), no split, and `part` receives fp16 [M, F] = silu(gate) * up.
// plane_rows (0 = M): rows per split-K plane of `part`, for callers that fill a taller output in row slabs.
// W is in the tiled working layout (common.h); with a_dual M is at most 128.
hipError_t launch_gemm_skinny_h16(hipStream_t s, const void* A, const void* W, float* part, int M, int Nw, int K,
                                  int nsplit, int a_dual, int plane_rows = 0);
int gemm_skinny_pick_split(int M, int Nw, int K, int a_dual = 0);
// Per-device one-time kernel attribute setup; call before the first launch and outside any stream capture.
hipError_t gemm_configure();
hipError_t sampler_configure();   // likewise for the sampler's LDS row cache

// ---- elementwise / small kernels (act_bf16 != 0: 16-bit (fp16) activations, else fp32) ----
hipError_t launch_pack_tokens(hipStream_t s, const int* query_tokens, int Lmax, const int* tok_seq, const int* tok_pos,
                              int T, int vocab, int* ids_out, int* err_flag);
hipError_t launch_pack_tokens2(hipStream_t s, const int* query_tokens, int Lmax, const int* resp_tokens, int R,
                               const int* qlen, const int* tok_seq, const int* tok_pos, int T, int vocab, int* ids_out,
                               int* err_flag);
hipError_t launch_embed(hipStream_t s, const int* ids, const void* table, int w_bf16, float* x, int M, int d, int vocab,
                        int* err_flag);
// x[m] += sum_{s<nsplit} part[s][m][:] (if part), then y = rmsnorm(x) * gain.  rows[m] (optional) selects
// source rows of x (gather); then x is not updated.  dual (16-bit activations only): 1 = y rows are [hi (d) | lo (d)]
// fp16 pairs; 2 = [hi (d) | 4-bit low halves (d / 2 bytes) | unused] at the same row pitch, with one scale byte per
// (row, 128 columns) written to row_scale in the order of fp4_row_scale_offset(row, group, scale_groups) (common.h).
hipError_t launch_rmsnorm(hipStream_t s, float* x, const float* part, int nsplit, size_t part_stride,
                          const void* gain, int w_bf16, void* y, int act_bf16, int M, int d, float eps, const int* rows,
                          int dual, void* row_scale = nullptr, int scale_groups = 0);
// qkv fp32 [M, (Hq+2Hkv)h] (+ optional partial sums) -> rotated q and the paged KV cache.  16-bit mode: q_out is
// [M, Hq, 2, h] fp16 (hi | lo pair per head); fp32 mode: [M, Hq, h] floats.
hipError_t launch_rope_append(hipStream_t s, const float* qkv, const float* part, int nsplit, size_t part_stride,
                              const int* row_pos, const int* row_seq, const float* cos_t, const float* sin_t,
                              void* q_out, void* kv_pool_layer, const int* block_table, int max_blocks, int n_blocks,
                              int M, int Hq, int Hkv, int h, int act_bf16);
// h[m][f] = silu(sum gate) * (sum up) from fp32 [M, 2F] (+ partial sums).
hipError_t launch_swiglu(hipStream_t s, const float* gu, int nsplit, size_t part_stride, void* h_out, int act_bf16,
                         int M, int F);
// seq_len[b] += 1 and step[b] += 1 for b < B (every row carries its own response index); the decode step lets the sampler do it
hipError_t launch_advance(hipStream_t s, int* seq_len, int* step, int B);
// bf16 -> fp16 copy of n elements (working copies of the weight matrices).
// dst (tiled working layout, see common.h) = fp16(src + scale * B[row0.., :] A): src row-major [rows, cols], bf16 or
// (src_is_h16) fp16; A bf16 [rank, cols] and B bf16 [.., rank] may be NULL (plain conversion).  rows % 16 == 0,
// cols % 128 == 0; src and dst must not overlap.
hipError_t launch_to_h16_tiled(hipStream_t s, const void* src, int src_is_h16, void* dst, int rows, int cols, const void* A,
                               const void* B, int rank, float scale, int row0);
// 4-bit (e2m1) copy of a tiled fp16 matrix, rows * cols / 2 bytes in the tiled order of a matrix with cols / 4 16-bit
// columns, and one scale byte per row (common.h); cols % 512 == 0.
hipError_t launch_to_w4_tiled(hipStream_t s, const void* src_tiled_h16, void* dst, void* row_scale, int rows, int cols);

// One layer's pool is [Hkv][n_blocks] pages: the pages a sequence gets from consecutive block ids are contiguous per
// KV head, so a workgroup streams one contiguous region and different workgroups spread over the memory channels.
// ---- attention over the paged cache (16-bit mode: q [rows, Hq, 2, 128] hi|lo pairs, out [rows, 2, Hq*128] hi|lo) ----
// (row_scale != NULL: the low halves of out in the 4-bit side format, as launch_attn_prefill_h16 writes them)
hipError_t launch_attn_decode_h16(hipStream_t s, const void* q, const void* kv_pool_layer, const int* block_table,
                                   int max_blocks, int n_blocks, const int* seq_len, void* out, int B, int Hq, int Hkv,
                                   void* row_scale = nullptr, int scale_groups = 0);
// Decode attention that starts from the QKV projection's partial sums: adds them, applies RoPE, appends the new
// key/value to the cache and attends (no separate rope_append launch).
hipError_t launch_attn_decode_fused_h16(hipStream_t s, const float* qkv_part, int nsplit, size_t part_stride,
                                        const float* cos_t, const float* sin_t, void* kv_pool_layer,
                                        const int* block_table, int max_blocks, int n_blocks, const int* seq_len, void* out,
                                        int B, int Hq, int Hkv);
// out rows are [hi (Hq*128) | lo (Hq*128)] fp16 pairs; with row_scale the low halves take the 4-bit side format
// instead ([hi | lo4 (Hq*64 bytes) | unused], one scale byte per (row, head), see launch_rmsnorm).
hipError_t launch_attn_prefill_h16(hipStream_t s, const void* q, const void* kv_pool_layer, const int* block_table,
                                    int max_blocks, int n_blocks, const int* cu_seqlens, const int* seq_ids, void* out, int nseq,
                                    int max_len, int Hq, int Hkv, void* row_scale = nullptr, int scale_groups = 0);
// fp32 path: one wavefront per (row, query head); row_pos[m] = position of the row's token.
hipError_t launch_attn_f32(hipStream_t s, const float* q, const float* kv_pool_layer, const int* block_table,
                           int max_blocks, int n_blocks, const int* row_pos, const int* row_seq, float* out, int M, int Hq, int Hkv,
                           int h);

// ---- fp32 GEMM (plain ALU) ----
hipError_t launch_gemm_f32(hipStream_t s, const float* A, const float* W, float* out, int M, int N, int K, int accumulate);

// ---- sampler / log-prob gather ----
hipError_t launch_logprob_gather(hipStream_t s, const float* logits, int rows, int V, const int* slot,
                                 const int* resp_tokens, float* out, int* err_flag);
// Everything the sampler needs besides the logits.  Passed by value for ordinary launches, or read from device memory
// (args_dev != NULL) so that a captured decode graph serves every rollout: seed, temperature, top-p and the output
// buffers then change without re-recording anything.
struct SamplerArgs {
  float temperature, top_p;
  uint64_t seed;
  int greedy, logprob_mode;
  int row0;          // batch row of logits row 0 (a micro-batch keeps the random stream of its rows in the full batch)
  int out_stride;    // elements between consecutive rows of tok_out / lp_out
  int use_step_col;  // results go to column t (the row's response index) of the row instead of column 0
  int step_stride;   // 1: step_ptr[b] is the response index of row b; 0: step_ptr[0] for every row
  int* tok_out;
  float* lp_out;
};
// One workgroup per row of logits [B, V].  Response index of row b: t = step_ptr[b * step_stride]; results go to
// tok_out[b * out_stride + (use_step_col ? t : 0)]; cur_tok[b] receives the token too.  advance_seq_len / advance_step
// (both or neither; advance_step must then be step_ptr with step_stride 1): the step's bookkeeping is done here as well,
// seq_len[b] += 1 and step[b] = t + 1, which saves the decode step a launch.
hipError_t launch_sampler(hipStream_t s, const float* logits, int B, int V, const SamplerArgs& args, const SamplerArgs* args_dev,
                          const int* step_ptr, int* cur_tok, int* advance_seq_len = nullptr, int* advance_step = nullptr);
hipError_t launch_fill_int(hipStream_t s, int* p, int n, int value);

// Message that rlhf_gen_last_error(NULL) returns (entry points that have no context to attach it to).
void set_global_error(const char* msg);
// Device address of the library's static workspace for the current device, resolved once per device (rlhf_gen_static.hip).
hipError_t static_scratch_prepare();

// Hardware probes (k_probe.hip).  stream_read: reads bytes / 8192 chunks of 8 KB from buf (plain or nontemporal 16-byte
// loads), scratch >= 1 KB.  mfma_loop: `workgroups` x 4 wavefronts each issue 8 * iters v_mfma_f32_32x32x16_f16
// (32768 flop each) on operands taken from a 16 KB buffer; scratch >= 1 KB.
hipError_t launch_probe_stream_read(hipStream_t s, const void* buf, size_t bytes, int nontemporal, void* scratch);
hipError_t launch_probe_mfma_loop(hipStream_t s, const void* operands, int workgroups, int iters, void* scratch);
