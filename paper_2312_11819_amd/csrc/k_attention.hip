// Attention over the paged fp16 KV cache on the matrix cores (head_dim 128, 16-token pages).
//
// Both kernels work on tiles of 16 query rows that share one KV head.  For one page they form
// S^T = K Q^T (keys as the MFMA row operand, so lane l ends up holding the scores of tokens
// 4 (l >> 4) .. +4 against query row l & 15), run the online softmax on those registers, and feed the
// probabilities straight back as the column operand of O^T += V^T P^T; the page layout (common.h) is
// exactly the operand layout, so keys and values go from HBM to the MFMA through eight coalesced 16 B
// loads per lane with no shuffles and no LDS.
//   decode : the 16 rows are the query heads of one KV group at the newest position (rows beyond the group
//            size are zero padding); eight (or four) wavefronts split the pages of one (sequence, KV head) and
//            merge their partial (max, sum, O) through LDS.
//   prefill: the 16 rows are 16 consecutive positions of one query head; a wavefront walks the pages up to
//            its diagonal page and masks inside it.
// HBM-bound in decode: every cached byte is read once per step per KV head; the MFMA work is negligible.
#include <math.h>

#include "common.h"
#include "kernels.h"

namespace {

struct AttnState {
  f32x4_t o[8];  // O^T tile: o[db][i] = O[row l&15][dim 16 db + 4 (l>>4) + i]
  float m;       // running max (log2 domain) of row l & 15
  float l;       // this lane's share of the running sum
};

// STREAM: the page is read once by the whole grid (decode); prefill re-reads pages from several query tiles.
template <bool STREAM>
__device__ __forceinline__ void load_page(const char* page, int lane, uint4 kf[4], uint4 vf[4]) {
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    kf[kk] = STREAM ? load_stream16(page + kk * 1024 + lane * 16) : *(const uint4*)(page + kk * 1024 + lane * 16);
#pragma unroll
  for (int j = 0; j < 4; ++j)
    vf[j] = STREAM ? load_stream16(page + 4096 + j * 1024 + lane * 16) : *(const uint4*)(page + 4096 + j * 1024 + lane * 16);
}

// tok0: index of the page's first token; limit: number of tokens visible to this lane's query row.
// qf[0..3]: high parts of the query fragments, qf[4..7]: low parts (queries are fp16 pairs).
// The two halves of a page's work: scores from the key half, then the softmax update and the value half.
__device__ __forceinline__ f32x4_t attn_scores(const uint4 kf[4], const uint4 qf[8]) {
  f32x4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) s = mfma_16x16x32(kf[kk], qf[4 + kk], s);
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) s = mfma_16x16x32(kf[kk], qf[kk], s);
  return s;
}

template <bool MASK>
__device__ __forceinline__ void attn_update(f32x4_t s, const uint4 vf[4], AttnState& st, float scale_log2, int tok0,
                                            int limit, int g) {
  float sv[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    sv[i] = s[i] * scale_log2;
    if (MASK && tok0 + 4 * g + i >= limit) sv[i] = -INFINITY;
  }
  float mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  float mnew = fmaxf(st.m, mx);
  float alpha, p[4];
  if (mnew == -INFINITY) {  // nothing visible yet for this row
    alpha = 1.f;
    p[0] = p[1] = p[2] = p[3] = 0.f;
  } else {
    alpha = exp2f(st.m - mnew);
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = exp2f(sv[i] - mnew);
  }
  st.l = st.l * alpha + (p[0] + p[1]) + (p[2] + p[3]);
  st.m = mnew;
#pragma unroll
  for (int db = 0; db < 8; ++db) st.o[db] *= alpha;
  // probabilities as fp16 pairs: two MFMAs per value tile
  h16_t ph[4], pl[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) split_h16(p[i], ph[i], pl[i]);
  const uint2 pb = make_uint2((uint32_t)ph[0] | ((uint32_t)ph[1] << 16), (uint32_t)ph[2] | ((uint32_t)ph[3] << 16));
  const uint2 pc = make_uint2((uint32_t)pl[0] | ((uint32_t)pl[1] << 16), (uint32_t)pl[2] | ((uint32_t)pl[3] << 16));
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    st.o[2 * j] = mfma_16x16x16(make_uint2(vf[j].x, vf[j].y), pc, st.o[2 * j]);
    st.o[2 * j + 1] = mfma_16x16x16(make_uint2(vf[j].z, vf[j].w), pc, st.o[2 * j + 1]);
    st.o[2 * j] = mfma_16x16x16(make_uint2(vf[j].x, vf[j].y), pb, st.o[2 * j]);
    st.o[2 * j + 1] = mfma_16x16x16(make_uint2(vf[j].z, vf[j].w), pb, st.o[2 * j + 1]);
  }
}

template <bool MASK>
__device__ __forceinline__ void attn_page(const uint4 kf[4], const uint4 vf[4], const uint4 qf[8], AttnState& st,
                                          float scale_log2, int tok0, int limit, int g) {
  attn_update<MASK>(attn_scores(kf, qf), vf, st, scale_log2, tok0, limit, g);
}

__device__ __forceinline__ void init_state(AttnState& st) {
#pragma unroll
  for (int db = 0; db < 8; ++db) st.o[db] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
  st.m = -INFINITY;
  st.l = 0.f;
}

// grid (Hkv, B), 64 NWV threads.  out [B, 2, Hq*128] fp16 (hi | lo).  seq_len[b] = tokens cached BEFORE this step.
//   FUSED = false: q [B, Hq, 2, 128] fp16 (hi | lo per head) is given and the step's own key/value has already been
//     appended, so seq_len[b] + 1 tokens are read from the cache.
//   FUSED = true: the kernel starts from the QKV projection's split-K partial sums (qkv_part[s][b][qkv_w], s < nsplit):
//     it adds them, rotates q and k by the position, writes the new key/value into the cache page for later steps,
//     attends over the seq_len[b] cached tokens from HBM and folds the new token in from LDS at the merge.  This
//     removes the separate RoPE/append kernel from the decode step.
struct FusedArgs {
  const float* qkv_part;
  int nsplit;
  size_t part_stride;
  int qkv_w;
  const float* cos_t;
  const float* sin_t;
};

// NWV wavefronts per workgroup share a sequence's pages (page p goes to wavefront p % NWV); ROWS >= Hq / Hkv query rows.
// Measured on MI355X with the bare read pattern of this kernel (no arithmetic, same residency of 8 wavefronts per
// compute unit): four wavefronts with the next page prefetched while the current one is consumed reach 6.4-6.7 TB/s,
// eight wavefronts that each fetch a page, consume it and only then fetch the next reach 7.0-7.1 TB/s - the eight
// page loads of a workgroup then cover 64 KB of consecutive bytes and nothing else of that sequence is in flight.
// PREFETCH selects the former (kept for the fused form and for groups of more than 8 query heads).
template <bool FUSED, int NWV, int ROWS, bool PREFETCH>
__global__ __launch_bounds__(64 * NWV) void attn_decode_kernel(const h16_t* __restrict__ q, char* __restrict__ pool,
                                                          const int* __restrict__ block_table, int max_blocks, int n_blocks,
                                                          const int* __restrict__ seq_len, h16_t* __restrict__ out,
                                                          int Hq, int Hkv, float scale_log2, FusedArgs fa,
                                                          unsigned char* __restrict__ row_scale, int scale_groups) {
  __shared__ float m_s[NWV][16];
  __shared__ float l_s[NWV][16];
  __shared__ float o_s[NWV][ROWS][132];
  __shared__ __attribute__((aligned(16))) h16_t q_s[FUSED ? 16 : 1][256];  // [row][hi 128 | lo 128]
  __shared__ h16_t kn_s[FUSED ? 128 : 1], vn_s[FUSED ? 128 : 1];
  __shared__ float snew_s[16];
  const int kvh = blockIdx.x, b = blockIdx.y;
  const int group = Hq / Hkv;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, t = lane & 15, g = lane >> 4;
  // A workgroup's start is a chain of dependent loads: sequence length, then block-table entry, then page.  The
  // entry of this wavefront's first page (page w) does not need the length, so it is fetched alongside it and the
  // first page load follows one round trip earlier.  If the sequence has no page w the entry may be anything: it is
  // clamped to a valid page, and what comes back is never used (the wavefront has no pages then).
  const int* bt = block_table + (size_t)b * max_blocks;
  int first_blk = bt[min(w, max_blocks - 1)];
  const int pos = seq_len[b];                  // position of the step's token = tokens already cached
  first_blk = min(max(first_blk, 0), n_blocks - 1);
  uint4 qf[8];
  uint4 ka[4], va[4], kb[4], vb[4];
  load_page<true>(pool + ((size_t)kvh * n_blocks + first_blk) * KV_PAGE_BYTES, lane, ka, va);
  const int L = FUSED ? pos : pos + 1;         // tokens read from the cache
  const int npages = (L + 15) >> 4;
  // block-table entries of this wavefront's first 64 pages (lane i: page w + NWV i)
  const int last = npages - 1;
  const int my_blk0 = npages > 0 ? bt[min(w + NWV * lane, last)] : 0;
  if (FUSED) {
    const float* row = fa.qkv_part + (size_t)b * fa.qkv_w;
    const float* cs = fa.cos_t + (size_t)pos * 64;
    const float* sn = fa.sin_t + (size_t)pos * 64;
    char* page = pool + ((size_t)kvh * n_blocks + bt[pos >> 4]) * KV_PAGE_BYTES;
    const int slot = pos & 15;
    // tasks: (group + 2) vectors of 128 (the group's query heads, the key, the value), 64 dimension pairs each
    for (int task = threadIdx.x; task < (group + 2) * 64; task += 64 * NWV) {
      const int vec = task >> 6, i = task & 63;
      int col;  // column of dimension i of this vector in the fused qkv row
      if (vec < group) col = (kvh * group + vec) * 128 + i;
      else if (vec == group) col = (Hq + kvh) * 128 + i;
      else col = (Hq + Hkv + kvh) * 128 + i;
      // up to 8 partial sums, all loads in flight at once, added in split order
      float av[8], bv[8];
#pragma unroll
      for (int s8 = 0; s8 < 8; ++s8) {
        const size_t so = (size_t)min(s8, fa.nsplit - 1) * fa.part_stride;
        av[s8] = row[so + col];
        bv[s8] = row[so + col + 64];
      }
      float a = 0.f, bb = 0.f;
#pragma unroll
      for (int s8 = 0; s8 < 8; ++s8)
        if (s8 < fa.nsplit) { a += av[s8]; bb += bv[s8]; }
      if (vec <= group) {  // queries and the key are rotated
        const float c = cs[i], sv = sn[i];
        const float r0 = a * c - bb * sv, r1 = bb * c + a * sv;
        a = r0;
        bb = r1;
      }
      if (vec < group) {
        split_h16(a, q_s[vec][i], q_s[vec][128 + i]);
        split_h16(bb, q_s[vec][i + 64], q_s[vec][128 + i + 64]);
      } else if (vec == group) {
        const h16_t k0 = f32_to_h16(a), k1 = f32_to_h16(bb);
        kn_s[i] = k0;
        kn_s[i + 64] = k1;
        *(h16_t*)(page + kpage_offset(slot, i)) = k0;
        *(h16_t*)(page + kpage_offset(slot, i + 64)) = k1;
      } else {
        const h16_t v0 = f32_to_h16(a), v1 = f32_to_h16(bb);
        vn_s[i] = v0;
        vn_s[i + 64] = v1;
        *(h16_t*)(page + vpage_offset(slot, i)) = v0;
        *(h16_t*)(page + vpage_offset(slot, i + 64)) = v1;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      qf[kk] = make_uint4(0, 0, 0, 0);
      if (t < group) qf[kk] = *(const uint4*)(&q_s[t][(kk >> 2) * 128 + 8 * (4 * (kk & 3) + g)]);
    }
    // score of the new token against each query row (same fp16 values a later step will read from the cache)
    for (int r = w; r < group; r += NWV) {
      float acc = 0.f;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int d = 2 * lane + e;
        acc += (h16_to_f32(q_s[r][d]) + h16_to_f32(q_s[r][128 + d])) * h16_to_f32(kn_s[d]);
      }
      acc = wave_sum(acc);
      if (lane == 0) snew_s[r] = acc * scale_log2;
    }
  } else {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      qf[kk] = make_uint4(0, 0, 0, 0);
      if (t < group)
        qf[kk] = *(const uint4*)(q + ((size_t)b * Hq + kvh * group + t) * 256 + (kk >> 2) * 128 + 8 * (4 * (kk & 3) + g));
    }
  }
  AttnState st;
  init_state(st);
  // This wavefront takes pages w, w + NWV, w + 2 NWV, ...  Their block-table entries are fetched up front, 64 at a time
  // (lane i holds the entry of page w + NWV i), and broadcast from registers inside the loop.  Page loads are issued
  // with no branch around them (an index past the end re-reads the last page), so that the loads of the next page
  // stay in flight while the current one is consumed.
  for (int base = w; base < npages; base += 64 * NWV) {
    int my_blk = my_blk0;
    if (base != w) {  // beyond 64 NWV pages: next batch of 64 pages per wavefront
      my_blk = bt[min(base + NWV * lane, last)];
      load_page<true>(pool + ((size_t)kvh * n_blocks + __shfl(my_blk, 0)) * KV_PAGE_BYTES, lane, ka, va);
    }
    const int cnt = min(64, (npages - base + NWV - 1) / NWV);  // pages of this wavefront in this batch
    if (PREFETCH) {
      int i = 0;
      for (; i + 2 <= cnt; i += 2) {
        load_page<true>(pool + ((size_t)kvh * n_blocks + __shfl(my_blk, i + 1)) * KV_PAGE_BYTES, lane, kb, vb);
        attn_page<true>(ka, va, qf, st, scale_log2, (base + NWV * i) * 16, L, g);
        load_page<true>(pool + ((size_t)kvh * n_blocks + __shfl(my_blk, min(i + 2, cnt - 1))) * KV_PAGE_BYTES, lane, ka, va);
        attn_page<true>(kb, vb, qf, st, scale_log2, (base + NWV * (i + 1)) * 16, L, g);
      }
      if (i < cnt) attn_page<true>(ka, va, qf, st, scale_log2, (base + NWV * i) * 16, L, g);
    } else {
      // one page in flight per wavefront: the key half of the next page is requested as soon as the scores of
      // this one have been issued, its value half after the value MFMAs
      for (int i = 0; i < cnt; ++i) {
        const f32x4_t sc = attn_scores(ka, qf);
        const bool more = i + 1 < cnt;
        const char* next = pool + ((size_t)kvh * n_blocks + __shfl(my_blk, min(i + 1, cnt - 1))) * KV_PAGE_BYTES;
        if (more) {
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) ka[kk] = load_stream16(next + kk * 1024 + lane * 16);
        }
        attn_update<true>(sc, va, st, scale_log2, (base + NWV * i) * 16, L, g);
        if (more) {
#pragma unroll
          for (int j = 0; j < 4; ++j) va[j] = load_stream16(next + 4096 + j * 1024 + lane * 16);
        }
      }
    }
  }
  float lt = st.l;
  lt += __shfl_xor(lt, 16);
  lt += __shfl_xor(lt, 32);
  if (g == 0) { m_s[w][t] = st.m; l_s[w][t] = lt; }
  if (t < group) {
#pragma unroll
    for (int db = 0; db < 8; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) o_s[w][t][db * 16 + 4 * g + i] = st.o[db][i];
  }
  __syncthreads();
  if (!FUSED && row_scale) {
    // low halves in the 4-bit side format (row = [hi (Hq*128) | lo4 (Hq*64 bytes) | unused], one scale per (row, head)):
    // a wavefront merges whole heads, two adjacent dimensions per lane, so that the head's largest low half is a
    // wavefront reduction and a lane's two codes make one byte
    for (int r = w; r < group; r += NWV) {
      float M = m_s[0][r];
#pragma unroll
      for (int ww = 1; ww < NWV; ++ww) M = fmaxf(M, m_s[ww][r]);
      float n0 = 0.f, n1 = 0.f, den = 0.f;
#pragma unroll
      for (int ww = 0; ww < NWV; ++ww) {
        const float mw = m_s[ww][r];
        const float a = (mw == -INFINITY) ? 0.f : exp2f(mw - M);
        n0 += a * o_s[ww][r][2 * lane];
        n1 += a * o_s[ww][r][2 * lane + 1];
        den += a * l_s[ww][r];
      }
      const float v0 = n0 / den, v1 = n1 / den;
      const h16_t h0 = f32_to_h16(v0), h1 = f32_to_h16(v1);
      const float l0 = v0 - h16_to_f32(h0), l1 = v1 - h16_to_f32(h1);
      const uint32_t sb = fp4_scale_byte(wave_max(fmaxf(fabsf(l0), fabsf(l1))));
      const float is = fp4_inv_scale(sb);
      const int head = kvh * group + r;
      char* orow = (char*)out + (size_t)b * 4 * Hq * 128;
      *(uint32_t*)(orow + 2 * (head * 128 + 2 * lane)) = (uint32_t)h0 | ((uint32_t)h1 << 16);
      *(unsigned char*)(orow + 2 * Hq * 128 + head * 64 + lane) = (unsigned char)(fp4_code(l0 * is) | (fp4_code(l1 * is) << 4));
      if (lane == 0) row_scale[fp4_row_scale_offset(b, head, scale_groups)] = (unsigned char)sb;
    }
    return;
  }
  for (int idx = threadIdx.x; idx < group * 128; idx += 64 * NWV) {
    int r = idx >> 7, dim = idx & 127;
    float M = m_s[0][r];
#pragma unroll
    for (int ww = 1; ww < NWV; ++ww) M = fmaxf(M, m_s[ww][r]);
    if (FUSED) M = fmaxf(M, snew_s[r]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int ww = 0; ww < NWV; ++ww) {
      float mw = m_s[ww][r];
      float a = (mw == -INFINITY) ? 0.f : exp2f(mw - M);
      num += a * o_s[ww][r][dim];
      den += a * l_s[ww][r];
    }
    if (FUSED) {  // the new token: weight exp2(s_new - M), value from LDS
      float a = exp2f(snew_s[r] - M);
      num += a * h16_to_f32(vn_s[dim]);
      den += a;
    }
    h16_t* orow = out + (size_t)b * 2 * Hq * 128 + (kvh * group + r) * 128 + dim;
    split_h16(num / den, orow[0], orow[Hq * 128]);
  }
}

// grid (ceil(max_len / 64), Hq, nseq), 256 threads: wavefront w owns positions p0 .. p0+15 of sequence
// seq_ids[blockIdx.z] with p0 = 16 (4 blockIdx.x + w).  q / out are packed over tokens (row cu_seqlens[z] + pos)
// in the same hi | lo layouts as the decode kernel.
__global__ __launch_bounds__(256) void attn_prefill_kernel(const h16_t* __restrict__ q, const char* __restrict__ pool,
                                                           const int* __restrict__ block_table, int max_blocks, int n_blocks,
                                                           const int* __restrict__ cu_seqlens,
                                                           const int* __restrict__ seq_ids, h16_t* __restrict__ out,
                                                           int Hq, int Hkv, float scale_log2,
                                                           unsigned char* __restrict__ row_scale, int scale_groups) {
  const int z = blockIdx.z, head = blockIdx.y;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, t = lane & 15, g = lane >> 4;
  const int row0 = cu_seqlens[z], len = cu_seqlens[z + 1] - row0;
  const int p0 = 16 * (4 * blockIdx.x + w);
  if (p0 >= len) return;
  const int b = seq_ids[z];
  const int kvh = head / (Hq / Hkv);
  const bool valid = p0 + t < len;
  uint4 qf[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    qf[kk] = make_uint4(0, 0, 0, 0);
    if (valid)
      qf[kk] = *(const uint4*)(q + ((size_t)(row0 + p0 + t) * Hq + head) * 256 + (kk >> 2) * 128 + 8 * (4 * (kk & 3) + g));
  }
  AttnState st;
  init_state(st);
  const int* bt = block_table + (size_t)b * max_blocks;
  const int pd = p0 >> 4;  // diagonal page = last page this tile reads
  // Pages 0 .. pd in order.  As in the decode kernel the block-table entries are fetched 64 at a time (lane i holds
  // the entry of page base + i) and broadcast from registers, and the page loads are issued with no branch around
  // them (an index past the end re-reads the last page), so the next page is in flight while this one is consumed.
  const int my_blk0 = bt[min(lane, pd)];
  uint4 ka[4], va[4], kb[4], vb[4];
  load_page<false>(pool + ((size_t)kvh * n_blocks + __shfl(my_blk0, 0)) * KV_PAGE_BYTES, lane, ka, va);
#define PREFILL_PAGE(KF, VF, P)                                                              \
  if ((P) == pd)                                                                             \
    attn_page<true>(KF, VF, qf, st, scale_log2, (P) * 16, p0 + t + 1, g);                    \
  else                                                                                       \
    attn_page<false>(KF, VF, qf, st, scale_log2, (P) * 16, 0, g);
  for (int base = 0; base <= pd; base += 64) {
    int my_blk = my_blk0;
    if (base != 0) {
      my_blk = bt[min(base + lane, pd)];
      load_page<false>(pool + ((size_t)kvh * n_blocks + __shfl(my_blk, 0)) * KV_PAGE_BYTES, lane, ka, va);
    }
    const int cnt = min(64, pd + 1 - base);
    int i = 0;
    for (; i + 2 <= cnt; i += 2) {
      load_page<false>(pool + ((size_t)kvh * n_blocks + __shfl(my_blk, i + 1)) * KV_PAGE_BYTES, lane, kb, vb);
      PREFILL_PAGE(ka, va, base + i)
      load_page<false>(pool + ((size_t)kvh * n_blocks + __shfl(my_blk, min(i + 2, cnt - 1))) * KV_PAGE_BYTES, lane, ka, va);
      PREFILL_PAGE(kb, vb, base + i + 1)
    }
    if (i < cnt) PREFILL_PAGE(ka, va, base + i)
  }
#undef PREFILL_PAGE
  float lt = st.l;
  lt += __shfl_xor(lt, 16);
  lt += __shfl_xor(lt, 32);
  if (valid && row_scale) {
    // low halves in the 4-bit side format: row = [hi (Hq*128) | lo4 (Hq*64 bytes) | unused], one scale per (row, head);
    // the head's 128 dimensions of this row are spread over the four lanes t, t + 16, t + 32, t + 48
    const float inv = 1.f / lt;
    const int m = row0 + p0 + t;
    char* orow = (char*)out + (size_t)m * 4 * Hq * 128;
    float am = 0.f;
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      h16_t hi[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float v = st.o[db][i] * inv;
        hi[i] = f32_to_h16(v);
        st.o[db][i] = v - h16_to_f32(hi[i]);
        am = fmaxf(am, fabsf(st.o[db][i]));
      }
      *(uint2*)(orow + 2 * (head * 128 + db * 16 + 4 * g)) =
          make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
    }
    am = fmaxf(am, __shfl_xor(am, 16));
    am = fmaxf(am, __shfl_xor(am, 32));
    const uint32_t sb = fp4_scale_byte(am);
    const float is = fp4_inv_scale(sb);
#pragma unroll
    for (int db = 0; db < 8; ++db)
      *(uint16_t*)(orow + 2 * Hq * 128 + ((head * 128 + db * 16 + 4 * g) >> 1)) =
          (uint16_t)(fp4_code(st.o[db][0] * is) | (fp4_code(st.o[db][1] * is) << 4) | (fp4_code(st.o[db][2] * is) << 8) |
                     (fp4_code(st.o[db][3] * is) << 12));
    if (g == 0) row_scale[fp4_row_scale_offset(m, head, scale_groups)] = (unsigned char)sb;
  } else if (valid) {
    float inv = 1.f / lt;
    h16_t* orow = out + (size_t)(row0 + p0 + t) * 2 * Hq * 128 + head * 128 + 4 * g;  // row = [hi (Hq*128) | lo]
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      h16_t hi[4], lo[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) split_h16(st.o[db][i] * inv, hi[i], lo[i]);
      *(uint2*)(orow + db * 16) = make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
      *(uint2*)(orow + Hq * 128 + db * 16) = make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
    }
  }
}

// fp32 path: one wavefront per (row, query head); lane j takes tokens j, j+64, ...; page = [2][16][h] floats.
template <int H>
__global__ __launch_bounds__(64) void attn_f32_kernel(const float* __restrict__ q, const float* __restrict__ pool,
                                                      const int* __restrict__ block_table, int max_blocks, int n_blocks,
                                                      const int* __restrict__ row_pos, const int* __restrict__ row_seq,
                                                      float* __restrict__ out, int Hq, int Hkv) {
  const int m = blockIdx.y, head = blockIdx.x, lane = threadIdx.x;
  const int b = row_seq ? row_seq[m] : m;
  const int L = row_pos[m] + 1;
  const int kvh = head / (Hq / Hkv);
  const float* qr = q + ((size_t)m * Hq + head) * H;
  float qv[H];
#pragma unroll
  for (int i = 0; i < H; ++i) qv[i] = qr[i];
  const float scale = rsqrtf((float)H);
  float mx = -INFINITY, l = 0.f, o[H];
#pragma unroll
  for (int i = 0; i < H; ++i) o[i] = 0.f;
  const int* bt = block_table + (size_t)b * max_blocks;
  for (int tok = lane; tok < L; tok += 64) {
    const float* page = pool + ((size_t)kvh * n_blocks + bt[tok >> 4]) * (2 * 16 * H);
    const float* kr = page + (tok & 15) * H;
    const float* vr = page + 16 * H + (tok & 15) * H;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < H; ++i) s += qv[i] * kr[i];
    s *= scale;
    float mn = fmaxf(mx, s);
    float a = expf(mx - mn), pw = expf(s - mn);
    l = l * a + pw;
#pragma unroll
    for (int i = 0; i < H; ++i) o[i] = o[i] * a + pw * vr[i];
    mx = mn;
  }
  float M = wave_max(mx);
  float a = (mx == -INFINITY) ? 0.f : expf(mx - M);
  float den = wave_sum(l * a);
  float* orow = out + ((size_t)m * Hq + head) * H;
#pragma unroll
  for (int i = 0; i < H; ++i) {
    float v = wave_sum(o[i] * a);
    if (lane == 0) orow[i] = v / den;
  }
}

}  // namespace

static const float LOG2E = 1.4426950408889634f;

hipError_t launch_attn_decode_h16(hipStream_t s, const void* q, const void* kv_pool_layer, const int* block_table,
                                   int max_blocks, int n_blocks, const int* seq_len, void* out, int B, int Hq, int Hkv,
                                   void* row_scale, int scale_groups) {
  if (B <= 0) return hipSuccess;
  if (Hq % Hkv || Hq / Hkv > 16) return hipErrorInvalidValue;
  if (row_scale && scale_groups * 128 < B) return hipErrorInvalidValue;
  unsigned char* rs = (unsigned char*)row_scale;
  float scale_log2 = LOG2E / sqrtf((float)KV_HEAD_DIM);
  FusedArgs fa{};
  // (the form depends on the head counts only, never on the batch, so a sequence's result is the same bits in any batch)
  if (Hq / Hkv <= 8)
    attn_decode_kernel<false, 8, 8, false><<<dim3(Hkv, B), 512, 0, s>>>((const h16_t*)q, (char*)const_cast<void*>(kv_pool_layer),
                                                                        block_table, max_blocks, n_blocks, seq_len, (h16_t*)out,
                                                                        Hq, Hkv, scale_log2, fa, rs, scale_groups);
  else
    attn_decode_kernel<false, 4, 16, true><<<dim3(Hkv, B), 256, 0, s>>>((const h16_t*)q, (char*)const_cast<void*>(kv_pool_layer),
                                                                        block_table, max_blocks, n_blocks, seq_len, (h16_t*)out,
                                                                        Hq, Hkv, scale_log2, fa, rs, scale_groups);
  return hipGetLastError();
}

hipError_t launch_attn_decode_fused_h16(hipStream_t s, const float* qkv_part, int nsplit, size_t part_stride,
                                        const float* cos_t, const float* sin_t, void* kv_pool_layer,
                                        const int* block_table, int max_blocks, int n_blocks, const int* seq_len, void* out,
                                        int B, int Hq, int Hkv) {
  if (B <= 0) return hipSuccess;
  if (Hq % Hkv || Hq / Hkv > 16 || nsplit < 1 || nsplit > 8) return hipErrorInvalidValue;
  float scale_log2 = LOG2E / sqrtf((float)KV_HEAD_DIM);
  FusedArgs fa{qkv_part, nsplit, part_stride, (Hq + 2 * Hkv) * KV_HEAD_DIM, cos_t, sin_t};
  attn_decode_kernel<true, 4, 16, true><<<dim3(Hkv, B), 256, 0, s>>>(nullptr, (char*)kv_pool_layer, block_table, max_blocks, n_blocks,
                                                        seq_len, (h16_t*)out, Hq, Hkv, scale_log2, fa, nullptr, 0);
  return hipGetLastError();
}

hipError_t launch_attn_prefill_h16(hipStream_t s, const void* q, const void* kv_pool_layer, const int* block_table,
                                    int max_blocks, int n_blocks, const int* cu_seqlens, const int* seq_ids, void* out, int nseq,
                                    int max_len, int Hq, int Hkv, void* row_scale, int scale_groups) {
  if (nseq <= 0 || max_len <= 0) return hipSuccess;
  if (Hq % Hkv) return hipErrorInvalidValue;
  // (row_scale: the caller guarantees that 128 * scale_groups covers cu_seqlens[nseq], the number of rows)
  if (row_scale && scale_groups <= 0) return hipErrorInvalidValue;
  float scale_log2 = LOG2E / sqrtf((float)KV_HEAD_DIM);
  attn_prefill_kernel<<<dim3((max_len + 63) / 64, Hq, nseq), 256, 0, s>>>(
      (const h16_t*)q, (const char*)kv_pool_layer, block_table, max_blocks, n_blocks, cu_seqlens, seq_ids, (h16_t*)out, Hq, Hkv,
      scale_log2, (unsigned char*)row_scale, scale_groups);
  return hipGetLastError();
}

hipError_t launch_attn_f32(hipStream_t s, const float* q, const float* kv_pool_layer, const int* block_table,
                           int max_blocks, int n_blocks, const int* row_pos, const int* row_seq, float* out, int M, int Hq, int Hkv,
                           int h) {
  if (M <= 0) return hipSuccess;
  dim3 grid(Hq, M);
  if (h == 32)
    attn_f32_kernel<32><<<grid, 64, 0, s>>>(q, kv_pool_layer, block_table, max_blocks, n_blocks, row_pos, row_seq, out, Hq, Hkv);
  else if (h == 64)
    attn_f32_kernel<64><<<grid, 64, 0, s>>>(q, kv_pool_layer, block_table, max_blocks, n_blocks, row_pos, row_seq, out, Hq, Hkv);
  else if (h == 128)
    attn_f32_kernel<128><<<grid, 64, 0, s>>>(q, kv_pool_layer, block_table, max_blocks, n_blocks, row_pos, row_seq, out, Hq, Hkv);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}
