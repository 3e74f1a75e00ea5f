// Small memory-bound kernels of the rollout: token packing, embedding gather, RMSNorm (optionally fused
// with the reduction of split-K partial sums and the residual add), rotary embedding + KV-cache append,
// SwiGLU, and the per-step counter update.  All are plain vector-ALU kernels; none is a contraction.
#include "common.h"
#include "kernels.h"

__global__ void pack_tokens_kernel(const int* __restrict__ query_tokens, int Lmax, const int* __restrict__ tok_seq,
                                   const int* __restrict__ tok_pos, int T, int vocab, int* __restrict__ ids_out,
                                   int* __restrict__ err_flag) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= T) return;
  int id = query_tokens[(size_t)tok_seq[i] * Lmax + tok_pos[i]];
  if (id < 0 || id >= vocab) {
    *err_flag = 1;
    id = id < 0 ? 0 : vocab - 1;
  }
  ids_out[i] = id;
}

// Scoring pass: the fed sequence of row b is its query followed by its response; position p < qlen[b] reads the
// query, later positions the response.
__global__ void pack_tokens2_kernel(const int* __restrict__ query_tokens, int Lmax, const int* __restrict__ resp_tokens,
                                    int R, const int* __restrict__ qlen, const int* __restrict__ tok_seq,
                                    const int* __restrict__ tok_pos, int T, int vocab, int* __restrict__ ids_out,
                                    int* __restrict__ err_flag) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= T) return;
  int b = tok_seq[i], p = tok_pos[i], ql = qlen[b];
  int id = p < ql ? query_tokens[(size_t)b * Lmax + p] : resp_tokens[(size_t)b * R + (p - ql)];
  if (id < 0 || id >= vocab) {
    *err_flag = 1;
    id = id < 0 ? 0 : vocab - 1;
  }
  ids_out[i] = id;
  // The last response token is scored but never fed: the thread of the row's last fed position validates it too, so
  // that every token id of the call has been checked before the forward pass starts.
  if (p == ql + R - 2) {
    const int last = resp_tokens[(size_t)b * R + (R - 1)];
    if (last < 0 || last >= vocab) *err_flag = 1;
  }
}

hipError_t launch_pack_tokens2(hipStream_t s, const int* query_tokens, int Lmax, const int* resp_tokens, int R,
                               const int* qlen, const int* tok_seq, const int* tok_pos, int T, int vocab, int* ids_out,
                               int* err_flag) {
  if (T <= 0) return hipSuccess;
  pack_tokens2_kernel<<<(T + 255) / 256, 256, 0, s>>>(query_tokens, Lmax, resp_tokens, R, qlen, tok_seq, tok_pos, T, vocab,
                                                      ids_out, err_flag);
  return hipGetLastError();
}

hipError_t launch_pack_tokens(hipStream_t s, const int* query_tokens, int Lmax, const int* tok_seq, const int* tok_pos,
                              int T, int vocab, int* ids_out, int* err_flag) {
  if (T <= 0) return hipSuccess;
  pack_tokens_kernel<<<(T + 255) / 256, 256, 0, s>>>(query_tokens, Lmax, tok_seq, tok_pos, T, vocab, ids_out, err_flag);
  return hipGetLastError();
}

template <bool WBF16>
__global__ __launch_bounds__(256) void embed_kernel(const int* __restrict__ ids, const void* __restrict__ table,
                                                    float* __restrict__ x, int d, int vocab, int* __restrict__ err_flag) {
  int m = blockIdx.x;
  int id = ids[m];
  if (id < 0 || id >= vocab) {
    if (threadIdx.x == 0) *err_flag = 1;
    id = id < 0 ? 0 : vocab - 1;
  }
  float* xr = x + (size_t)m * d;
  if (WBF16) {
    const bf16_t* row = (const bf16_t*)table + (size_t)id * d;
    for (int i = threadIdx.x * 4; i < d; i += 1024) {
      uint2 v = *(const uint2*)(row + i);
      float4 o;
      o.x = __uint_as_float(v.x << 16);
      o.y = __uint_as_float(v.x & 0xffff0000u);
      o.z = __uint_as_float(v.y << 16);
      o.w = __uint_as_float(v.y & 0xffff0000u);
      *(float4*)(xr + i) = o;
    }
  } else {
    const float* row = (const float*)table + (size_t)id * d;
    for (int i = threadIdx.x * 4; i < d; i += 1024) *(float4*)(xr + i) = *(const float4*)(row + i);
  }
}

hipError_t launch_embed(hipStream_t s, const int* ids, const void* table, int w_bf16, float* x, int M, int d, int vocab,
                        int* err_flag) {
  if (M <= 0) return hipSuccess;
  if (w_bf16)
    embed_kernel<true><<<M, 256, 0, s>>>(ids, table, x, d, vocab, err_flag);
  else
    embed_kernel<false><<<M, 256, 0, s>>>(ids, table, x, d, vocab, err_flag);
  return hipGetLastError();
}

// One workgroup of NT threads per row, d <= 8 * 4 * NT, d % 4 == 0.  The sum of squares is taken in a fixed
// order, so the result does not change from run to run.  Partial sums are added in split order 0, 1, ...
// DUAL: 0 = one 16-bit (or fp32) value per element; 1 = fp16 pairs, row = [hi (d) | lo (d)]; 2 = fp16 high halves and
// 4-bit low halves, row = [hi (d) | lo4 (d / 2 bytes) | unused] with the same row pitch as form 1, one scale byte per
// 128 columns in row_scale (common.h, fp4_row_scale_offset; d % 128 == 0).
template <bool WBF16, bool A16, int NT, int DUAL>
__global__ __launch_bounds__(NT) void rmsnorm_kernel(float* __restrict__ x, const float* __restrict__ part, int nsplit,
                                                     size_t part_stride, const void* __restrict__ gain,
                                                     void* __restrict__ y, int d, float eps,
                                                     const int* __restrict__ rows, unsigned char* __restrict__ row_scale,
                                                     int scale_groups) {
  constexpr int IT = 8192 / (4 * NT);
  __shared__ float red[NT / 64];
  int m = blockIdx.x;
  int src = rows ? rows[m] : m;
  float* xr = x + (size_t)src * d;
  float4 v[IT];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    int i = (it * NT + threadIdx.x) * 4;
    if (i < d) {
      float4 a = *(const float4*)(xr + i);
      if (nsplit > 0) {
        const float* pp = part + (size_t)m * d + i;
        int sidx = 0;
        for (; sidx + 8 <= nsplit; sidx += 8) {  // the usual split counts (8, 16): eight independent loads in flight, added in order
          float4 pv[8];
#pragma unroll
          for (int s8 = 0; s8 < 8; ++s8) pv[s8] = *(const float4*)(pp + (size_t)(sidx + s8) * part_stride);
#pragma unroll
          for (int s8 = 0; s8 < 8; ++s8) { a.x += pv[s8].x; a.y += pv[s8].y; a.z += pv[s8].z; a.w += pv[s8].w; }
        }
        for (; sidx + 4 <= nsplit; sidx += 4) {  // four independent loads in flight, added in order
          float4 p0 = *(const float4*)(pp + (size_t)(sidx + 0) * part_stride);
          float4 p1 = *(const float4*)(pp + (size_t)(sidx + 1) * part_stride);
          float4 p2 = *(const float4*)(pp + (size_t)(sidx + 2) * part_stride);
          float4 p3 = *(const float4*)(pp + (size_t)(sidx + 3) * part_stride);
          a.x += p0.x; a.y += p0.y; a.z += p0.z; a.w += p0.w;
          a.x += p1.x; a.y += p1.y; a.z += p1.z; a.w += p1.w;
          a.x += p2.x; a.y += p2.y; a.z += p2.z; a.w += p2.w;
          a.x += p3.x; a.y += p3.y; a.z += p3.z; a.w += p3.w;
        }
        for (; sidx < nsplit; ++sidx) {
          float4 p = *(const float4*)(pp + (size_t)sidx * part_stride);
          a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
        }
        *(float4*)(xr + i) = a;
      }
      v[it] = a;
      ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
    }
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int i = 0; i < NT / 64; ++i) tot += red[i];
  float r = rsqrtf(tot / (float)d + eps);
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    int i = (it * NT + threadIdx.x) * 4;
    if (i < d) {
      float g0, g1, g2, g3;
      if (WBF16) {
        uint2 g = *(const uint2*)((const bf16_t*)gain + i);
        g0 = __uint_as_float(g.x << 16); g1 = __uint_as_float(g.x & 0xffff0000u);
        g2 = __uint_as_float(g.y << 16); g3 = __uint_as_float(g.y & 0xffff0000u);
      } else {
        float4 g = *(const float4*)((const float*)gain + i);
        g0 = g.x; g1 = g.y; g2 = g.z; g3 = g.w;
      }
      float4 a = v[it];
      float o0 = a.x * r * g0, o1 = a.y * r * g1, o2 = a.z * r * g2, o3 = a.w * r * g3;
      if (A16 && DUAL == 2) {
        const h16_t h0 = f32_to_h16(o0), h1 = f32_to_h16(o1), h2 = f32_to_h16(o2), h3 = f32_to_h16(o3);
        const float l0 = o0 - h16_to_f32(h0), l1 = o1 - h16_to_f32(h1), l2 = o2 - h16_to_f32(h2), l3 = o3 - h16_to_f32(h3);
        float am = fmaxf(fmaxf(fabsf(l0), fabsf(l1)), fmaxf(fabsf(l2), fabsf(l3)));
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) am = fmaxf(am, __shfl_xor(am, o));   // 32 threads = the 128 columns of one scale group
        const uint32_t sb = fp4_scale_byte(am);
        const float inv = fp4_inv_scale(sb);
        char* yr = (char*)y + (size_t)m * 4 * d;
        *(uint2*)(yr + 2 * i) = make_uint2((uint32_t)h0 | ((uint32_t)h1 << 16), (uint32_t)h2 | ((uint32_t)h3 << 16));
        *(uint16_t*)(yr + 2 * d + (i >> 1)) =
            (uint16_t)(fp4_code(l0 * inv) | (fp4_code(l1 * inv) << 4) | (fp4_code(l2 * inv) << 8) | (fp4_code(l3 * inv) << 12));
        if ((threadIdx.x & 31) == 0) row_scale[fp4_row_scale_offset(m, i >> 7, scale_groups)] = (unsigned char)sb;
      } else if (A16 && DUAL == 1) {  // row = [hi (d) | lo (d)]
        h16_t hi[4], lo[4];
        split_h16(o0, hi[0], lo[0]); split_h16(o1, hi[1], lo[1]);
        split_h16(o2, hi[2], lo[2]); split_h16(o3, hi[3], lo[3]);
        h16_t* yr = (h16_t*)y + (size_t)m * 2 * d + i;
        *(uint2*)yr = make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
        *(uint2*)(yr + d) = make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
      } else if (A16) {
        uint2 o;
        o.x = pack_h16x2(o0, o1);
        o.y = pack_h16x2(o2, o3);
        *(uint2*)((h16_t*)y + (size_t)m * d + i) = o;
      } else {
        *(float4*)((float*)y + (size_t)m * d + i) = make_float4(o0, o1, o2, o3);
      }
    }
  }
}

hipError_t launch_rmsnorm(hipStream_t s, float* x, const float* part, int nsplit, size_t part_stride, const void* gain,
                          int w_bf16, void* y, int act_bf16, int M, int d, float eps, const int* rows, int dual,
                          void* row_scale, int scale_groups) {
  if (M <= 0) return hipSuccess;
  if (d > 8192 || (d & 3)) return hipErrorInvalidValue;
  if (dual == 2 && (!row_scale || d % 128 || scale_groups * 128 < M || !(w_bf16 && act_bf16))) return hipErrorInvalidValue;
  if (!part) nsplit = 0;
  const bool wide = M <= 1024 && d >= 2048;  // few rows: spread each row over 1024 threads
  unsigned char* rs = (unsigned char*)row_scale;
  if (w_bf16 && act_bf16) {
    if (wide && dual == 2) rmsnorm_kernel<true, true, 1024, 2><<<M, 1024, 0, s>>>(x, part, nsplit, part_stride, gain, y, d, eps, rows, rs, scale_groups);
    else if (wide && dual) rmsnorm_kernel<true, true, 1024, 1><<<M, 1024, 0, s>>>(x, part, nsplit, part_stride, gain, y, d, eps, rows, rs, 0);
    else if (wide) rmsnorm_kernel<true, true, 1024, 0><<<M, 1024, 0, s>>>(x, part, nsplit, part_stride, gain, y, d, eps, rows, rs, 0);
    else if (dual == 2) rmsnorm_kernel<true, true, 256, 2><<<M, 256, 0, s>>>(x, part, nsplit, part_stride, gain, y, d, eps, rows, rs, scale_groups);
    else if (dual) rmsnorm_kernel<true, true, 256, 1><<<M, 256, 0, s>>>(x, part, nsplit, part_stride, gain, y, d, eps, rows, rs, 0);
    else rmsnorm_kernel<true, true, 256, 0><<<M, 256, 0, s>>>(x, part, nsplit, part_stride, gain, y, d, eps, rows, rs, 0);
  } else if (!w_bf16 && !act_bf16) {
    rmsnorm_kernel<false, false, 256, 0><<<M, 256, 0, s>>>(x, part, nsplit, part_stride, gain, y, d, eps, rows, rs, 0);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// One 64-thread workgroup per (token row, head of the fused q|k|v projection), so that every load of a launch is
// independent and in flight at once.  The rotation pairs dimension i with i + h/2 and uses the cos/sin tables built
// on the host in double precision (cos_t[pos * h/2 + i]).  16-bit path: h = 128, keys and values go to the
// MFMA-ordered page described in common.h.  fp32 path: page = [2][16][h] floats (keys, then values).
template <bool A16>
__global__ __launch_bounds__(64) void rope_append_kernel(const float* __restrict__ qkv, const float* __restrict__ part,
                                                         int nsplit, size_t part_stride,
                                                         const int* __restrict__ row_pos,
                                                         const int* __restrict__ row_seq,
                                                         const float* __restrict__ cos_t,
                                                         const float* __restrict__ sin_t, void* __restrict__ q_out,
                                                         void* __restrict__ pool, const int* __restrict__ block_table,
                                                         int max_blocks, int n_blocks, int Hq, int Hkv, int h) {
  const int m = blockIdx.y, head = blockIdx.x;
  const int pos = row_pos[m];
  const int b = row_seq ? row_seq[m] : m;
  const int half = h >> 1;
  const int width = (Hq + 2 * Hkv) * h;
  const float* row = qkv + (size_t)m * width + head * h;
  const float* prow = part + (size_t)m * width + head * h;
  const int blk = block_table[(size_t)b * max_blocks + (pos >> 4)];
  const int slot = pos & 15;
  if (head < Hq + Hkv) {
    for (int i = threadIdx.x; i < half; i += 64) {
      float a = row[i], bb = row[i + half];
      if (nsplit > 0) {   // (prefill passes complete sums: nothing to add, nothing to load)
        // up to 8 further partial sums with all loads in flight at once, added in split order
        float av[8], bv[8];
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) {
          const size_t so = (size_t)min(s8, max(nsplit - 1, 0)) * part_stride;
          av[s8] = prow[so + i];
          bv[s8] = prow[so + i + half];
        }
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8)
          if (s8 < nsplit) { a += av[s8]; bb += bv[s8]; }
        for (int sidx = 8; sidx < nsplit; ++sidx) {
          a += prow[sidx * part_stride + i];
          bb += prow[sidx * part_stride + i + half];
        }
      }
      float c = cos_t[(size_t)pos * half + i], sv = sin_t[(size_t)pos * half + i];
      float r0 = a * c - bb * sv, r1 = bb * c + a * sv;
      if (head < Hq) {
        if (A16) {  // [hi (h) | lo (h)] per head
          h16_t* qo = (h16_t*)q_out + ((size_t)m * Hq + head) * 2 * h;
          split_h16(r0, qo[i], qo[h + i]);
          split_h16(r1, qo[i + half], qo[h + i + half]);
        } else {
          float* qo = (float*)q_out + ((size_t)m * Hq + head) * h;
          qo[i] = r0;
          qo[i + half] = r1;
        }
      } else {
        const int kvh = head - Hq;
        if (A16) {
          char* page = (char*)pool + ((size_t)kvh * n_blocks + blk) * KV_PAGE_BYTES;
          *(h16_t*)(page + kpage_offset(slot, i)) = f32_to_h16(r0);
          *(h16_t*)(page + kpage_offset(slot, i + half)) = f32_to_h16(r1);
        } else {
          float* page = (float*)pool + ((size_t)kvh * n_blocks + blk) * (2 * 16 * h);
          page[slot * h + i] = r0;
          page[slot * h + i + half] = r1;
        }
      }
    }
  } else {
    const int kvh = head - Hq - Hkv;
    for (int dim = threadIdx.x; dim < h; dim += 64) {
      float v = row[dim];
      if (nsplit > 0) {
        float vv[8];
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) vv[s8] = prow[(size_t)min(s8, max(nsplit - 1, 0)) * part_stride + dim];
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8)
          if (s8 < nsplit) v += vv[s8];
        for (int sidx = 8; sidx < nsplit; ++sidx) v += prow[sidx * part_stride + dim];
      }
      if (A16) {
        char* page = (char*)pool + ((size_t)kvh * n_blocks + blk) * KV_PAGE_BYTES;
        *(h16_t*)(page + vpage_offset(slot, dim)) = f32_to_h16(v);
      } else {
        float* page = (float*)pool + ((size_t)kvh * n_blocks + blk) * (2 * 16 * h);
        page[16 * h + slot * h + dim] = v;
      }
    }
  }
}

hipError_t launch_rope_append(hipStream_t s, const float* qkv, const float* part, int nsplit, size_t part_stride,
                              const int* row_pos, const int* row_seq, const float* cos_t, const float* sin_t,
                              void* q_out, void* kv_pool_layer, const int* block_table, int max_blocks, int n_blocks,
                              int M, int Hq, int Hkv, int h, int act_bf16) {
  if (M <= 0) return hipSuccess;
  if (!part) { nsplit = 0; part = qkv; }
  dim3 grid(Hq + 2 * Hkv, M);
  if (act_bf16) {
    if (h != KV_HEAD_DIM) return hipErrorInvalidValue;
    rope_append_kernel<true><<<grid, 64, 0, s>>>(qkv, part, nsplit, part_stride, row_pos, row_seq, cos_t, sin_t, q_out,
                                                 kv_pool_layer, block_table, max_blocks, n_blocks, Hq, Hkv, h);
  } else {
    rope_append_kernel<false><<<grid, 64, 0, s>>>(qkv, part, nsplit, part_stride, row_pos, row_seq, cos_t, sin_t, q_out,
                                                  kv_pool_layer, block_table, max_blocks, n_blocks, Hq, Hkv, h);
  }
  return hipGetLastError();
}

template <bool A16>
__global__ __launch_bounds__(256) void swiglu_kernel(const float* __restrict__ gu, int nsplit, size_t part_stride,
                                                     void* __restrict__ h_out, int F) {
  int m = blockIdx.y;
  int f = blockIdx.x * 256 + threadIdx.x;
  if (f >= F) return;
  const float* row = gu + (size_t)m * 2 * F;
  float g = row[f], u = row[F + f];
  for (int sidx = 1; sidx < nsplit; ++sidx) {
    g += row[sidx * part_stride + f];
    u += row[sidx * part_stride + F + f];
  }
  float v = g / (1.f + __expf(-g)) * u;
  if (A16)
    ((h16_t*)h_out)[(size_t)m * F + f] = f32_to_h16(v);
  else
    ((float*)h_out)[(size_t)m * F + f] = v;
}

// Four features per thread, 16-bit output (F % 4 == 0): the decode path at 129..256 rows, where gate and up arrive
// as split-K planes.  Planes are added in order 0, 1, ..., like the scalar kernel.
__global__ __launch_bounds__(256) void swiglu4_kernel(const float* __restrict__ gu, int nsplit, size_t part_stride,
                                                      h16_t* __restrict__ h_out, int F) {
  const int m = blockIdx.y;
  const int f = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (f >= F) return;
  const float* row = gu + (size_t)m * 2 * F;
  float4 g = *(const float4*)(row + f), u = *(const float4*)(row + F + f);
  int sidx = 1;
  for (; sidx + 2 <= nsplit; sidx += 2) {
    const float4 g0 = *(const float4*)(row + (size_t)sidx * part_stride + f), u0 = *(const float4*)(row + (size_t)sidx * part_stride + F + f);
    const float4 g1 = *(const float4*)(row + (size_t)(sidx + 1) * part_stride + f), u1 = *(const float4*)(row + (size_t)(sidx + 1) * part_stride + F + f);
    g.x += g0.x; g.y += g0.y; g.z += g0.z; g.w += g0.w; u.x += u0.x; u.y += u0.y; u.z += u0.z; u.w += u0.w;
    g.x += g1.x; g.y += g1.y; g.z += g1.z; g.w += g1.w; u.x += u1.x; u.y += u1.y; u.z += u1.z; u.w += u1.w;
  }
  for (; sidx < nsplit; ++sidx) {
    const float4 g0 = *(const float4*)(row + (size_t)sidx * part_stride + f), u0 = *(const float4*)(row + (size_t)sidx * part_stride + F + f);
    g.x += g0.x; g.y += g0.y; g.z += g0.z; g.w += g0.w; u.x += u0.x; u.y += u0.y; u.z += u0.z; u.w += u0.w;
  }
  uint2 o;
  o.x = pack_h16x2(g.x / (1.f + __expf(-g.x)) * u.x, g.y / (1.f + __expf(-g.y)) * u.y);
  o.y = pack_h16x2(g.z / (1.f + __expf(-g.z)) * u.z, g.w / (1.f + __expf(-g.w)) * u.w);
  *(uint2*)(h_out + (size_t)m * F + f) = o;
}

hipError_t launch_swiglu(hipStream_t s, const float* gu, int nsplit, size_t part_stride, void* h_out, int act_bf16,
                         int M, int F) {
  if (M <= 0) return hipSuccess;
  if (nsplit < 1) nsplit = 1;
  if (act_bf16 && F % 4 == 0 && part_stride % 4 == 0) {
    swiglu4_kernel<<<dim3((F / 4 + 255) / 256, M), 256, 0, s>>>(gu, nsplit, part_stride, (h16_t*)h_out, F);
    return hipGetLastError();
  }
  dim3 grid((F + 255) / 256, M);
  if (act_bf16)
    swiglu_kernel<true><<<grid, 256, 0, s>>>(gu, nsplit, part_stride, h_out, F);
  else
    swiglu_kernel<false><<<grid, 256, 0, s>>>(gu, nsplit, part_stride, h_out, F);
  return hipGetLastError();
}

__global__ void advance_kernel(int* seq_len, int* step, int B) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < B) {
    seq_len[i] += 1;
    step[i] += 1;
  }
}

__global__ void fill_int_kernel(int* p, int n, int value) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = value;
}

hipError_t launch_fill_int(hipStream_t s, int* p, int n, int value) {
  if (n <= 0) return hipSuccess;
  fill_int_kernel<<<(n + 255) / 256, 256, 0, s>>>(p, n, value);
  return hipGetLastError();
}

hipError_t launch_advance(hipStream_t s, int* seq_len, int* step, int B) {
  advance_kernel<<<(B + 255) / 256, 256, 0, s>>>(seq_len, step, B);
  return hipGetLastError();
}

// Conversion of a bf16 weight matrix [rows, cols] to the fp16 working format in the tiled working layout of
// common.h (exact unless |w| < 2^-17, where fp16 subnormals keep an absolute accuracy of 2^-25; saturates beyond
// 65504).  One thread moves eight consecutive columns of one row.  With A != nullptr a low-rank update is folded in:
// dst[n, k] = fp16(src[n, k] + scale * sum_r B[row0 + n, r] A[r, k]) (LoRA adapters of the trainable Actor, Sec. V-A
// "Hyperparameters"; the sum runs over r ascending in fp32).  src and dst must not overlap (the layouts differ).
// SRC16: 0 = bf16 source, 1 = fp16 source (already in the working format, only re-tiled).
template <int SRC16>
__global__ void to_h16_tiled_kernel(const uint16_t* __restrict__ src, h16_t* __restrict__ dst, int rows, int cols,
                                    const bf16_t* __restrict__ A, const bf16_t* __restrict__ Bm, int rank, float scale,
                                    int row0) {
  const int cpr = cols >> 3;
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)rows * cpr) return;
  const int n = (int)(idx / cpr), k = (int)(idx % cpr) * 8;
  uint4 v = *(const uint4*)(src + (size_t)n * cols + k);
  uint4 o = v;
  if (SRC16 == 0) {
    float d[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (A != nullptr) {
      for (int r = 0; r < rank; ++r) {
        const float b = bf16_to_f32(Bm[(size_t)(row0 + n) * rank + r]);
        uint4 a = *(const uint4*)(A + (size_t)r * cols + k);
        const uint32_t aw[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          d[2 * j] = fmaf(b, __uint_as_float(aw[j] << 16), d[2 * j]);
          d[2 * j + 1] = fmaf(b, __uint_as_float(aw[j] & 0xffff0000u), d[2 * j + 1]);
        }
      }
    }
    const uint32_t vw[4] = {v.x, v.y, v.z, v.w};
    uint32_t ow[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      ow[j] = pack_h16x2(fmaf(scale, d[2 * j], __uint_as_float(vw[j] << 16)),
                         fmaf(scale, d[2 * j + 1], __uint_as_float(vw[j] & 0xffff0000u)));
    o = make_uint4(ow[0], ow[1], ow[2], ow[3]);
  }
  *(uint4*)(dst + wtile_offset(n, k, cols, rows)) = o;
}

// 4-bit copy of a tiled fp16 weight matrix for the low-half contraction of the large-tile GEMM: one workgroup per
// row; the row's largest magnitude fixes its scale byte, every group of four consecutive k becomes one 16-bit word of
// nibbles, and the words are laid out like a tiled matrix with cols / 4 columns (so cols % 512 == 0).
__global__ __launch_bounds__(256) void to_w4_tiled_kernel(const h16_t* __restrict__ src, uint16_t* __restrict__ dst,
                                                          unsigned char* __restrict__ row_scale, int rows, int cols) {
  __shared__ float red[4];
  const int n = blockIdx.x;
  float am = 0.f;
  for (int k = threadIdx.x * 4; k < cols; k += 1024) {
    const uint2 v = *(const uint2*)(src + wtile_offset(n, k, cols, rows));
    am = fmaxf(am, fmaxf(fmaxf(fabsf(h16_to_f32((h16_t)(v.x & 0xffff))), fabsf(h16_to_f32((h16_t)(v.x >> 16)))),
                         fmaxf(fabsf(h16_to_f32((h16_t)(v.y & 0xffff))), fabsf(h16_to_f32((h16_t)(v.y >> 16))))));
  }
  am = wave_max(am);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = am;
  __syncthreads();
  am = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  const uint32_t sb = fp4_scale_byte(am);
  const float inv = fp4_inv_scale(sb);
  for (int k = threadIdx.x * 4; k < cols; k += 1024) {
    const uint2 v = *(const uint2*)(src + wtile_offset(n, k, cols, rows));
    dst[wtile_offset(n, k >> 2, cols >> 2, rows)] =
        (uint16_t)(fp4_code(h16_to_f32((h16_t)(v.x & 0xffff)) * inv) | (fp4_code(h16_to_f32((h16_t)(v.x >> 16)) * inv) << 4) |
                   (fp4_code(h16_to_f32((h16_t)(v.y & 0xffff)) * inv) << 8) | (fp4_code(h16_to_f32((h16_t)(v.y >> 16)) * inv) << 12));
  }
  if (threadIdx.x == 0) row_scale[n] = (unsigned char)sb;
}

hipError_t launch_to_w4_tiled(hipStream_t s, const void* src_tiled_h16, void* dst, void* row_scale, int rows, int cols) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (rows % 16 || cols % 512 || !src_tiled_h16 || !dst || !row_scale) return hipErrorInvalidValue;
  to_w4_tiled_kernel<<<rows, 256, 0, s>>>((const h16_t*)src_tiled_h16, (uint16_t*)dst, (unsigned char*)row_scale, rows, cols);
  return hipGetLastError();
}

hipError_t launch_to_h16_tiled(hipStream_t s, const void* src, int src_is_h16, void* dst, int rows, int cols, const void* A,
                               const void* B, int rank, float scale, int row0) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (rows % 16 || cols % 128 || (A != nullptr && (rank < 1 || B == nullptr))) return hipErrorInvalidValue;
  size_t threads = (size_t)rows * (cols / 8);
  unsigned grid = (unsigned)((threads + 255) / 256);
  if (src_is_h16)
    to_h16_tiled_kernel<1><<<grid, 256, 0, s>>>((const uint16_t*)src, (h16_t*)dst, rows, cols, nullptr, nullptr, 0, 0.f, 0);
  else
    to_h16_tiled_kernel<0><<<grid, 256, 0, s>>>((const uint16_t*)src, (h16_t*)dst, rows, cols, (const bf16_t*)A,
                                               (const bf16_t*)B, rank, A ? scale : 0.f, row0);
  return hipGetLastError();
}
