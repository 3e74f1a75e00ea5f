// Shared device helpers for the gfx950 kernels: 16-bit conversions, MFMA wrappers,
// wavefront reductions, and the byte layout of one KV-cache page.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;  // raw bf16 bits (weights as the caller stores them)
typedef uint16_t h16_t;   // raw IEEE fp16 bits (activations, KV cache, working copies of the weights)
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
// fp32 -> fp16, round to nearest even, saturating at the largest finite fp16 instead of overflowing to infinity.
__device__ __forceinline__ h16_t f32_to_h16(float f) {
  _Float16 h = (_Float16)fminf(fmaxf(f, -65504.f), 65504.f);
  return __builtin_bit_cast(uint16_t, h);
}
// 16-byte load of data that is read exactly once and in whole cache lines per instruction (cached K/V pages in
// decode, the tiled weights of the decode GEMM): the nontemporal hint keeps it from displacing reusable lines in L2
// and measures 10-12 % faster than a plain load on MI355X for read-only streams (7.2 vs 6.4 TB/s at best).  It loses when
// one instruction takes only part of a line and another instruction the rest (the line is fetched twice).
typedef unsigned u32x4_native_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  u32x4_native_t v = __builtin_nontemporal_load((const u32x4_native_t*)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ uint32_t pack_h16x2(float lo, float hi) {
  return (uint32_t)f32_to_h16(lo) | ((uint32_t)f32_to_h16(hi) << 16);
}
__device__ __forceinline__ float h16_to_f32(h16_t v) { return (float)__builtin_bit_cast(_Float16, v); }
// Two-term fp16 representation v ~ hi + lo (22 significant bits).  The tensors whose rounding dominates the
// rollout's logit error (the input of the QKV and output projections, the rotated queries and the attention
// probabilities) are carried as such pairs and contracted with two MFMAs into the same accumulator.
__device__ __forceinline__ void split_h16(float v, h16_t& hi, h16_t& lo) {
  hi = f32_to_h16(v);
  lo = f32_to_h16(v - h16_to_f32(hi));
}

// All 16-bit MFMA operands are fp16 (11 significant bits): with bf16 activations the rounding error of a
// 32-layer rollout exceeds the parity tolerance several times over; the bf16 weights convert to fp16 exactly.
// D(16x16) += A(16x32) * B(32x16), fp16 in, fp32 out.  Lane l supplies row (l & 15) of A and column (l & 15) of
// B, eight consecutive k each, the k group chosen by l >> 4 in the same way for both operands.  Lane l receives
// D[4 (l >> 4) + i][l & 15], i = 0..3.
__device__ __forceinline__ f32x4_t mfma_16x16x32(uint4 a, uint4 b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}
// D(16x16) += A(16x16) * B(16x16): four consecutive k per lane, k group l >> 4.
__device__ __forceinline__ f32x4_t mfma_16x16x16(uint2 a, uint2 b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4_t, a), __builtin_bit_cast(f16x4_t, b), c, 0, 0, 0);
}
// D(32x32) += A(32x16) * B(16x32): lane l supplies row/column (l & 31), k group l >> 5 (8 k each).
// Lane l receives D[8 (i >> 2) + 4 (l >> 5) + (i & 3)][l & 31], i = 0..15.
__device__ __forceinline__ f32x16_t mfma_32x32x16(uint4 a, uint4 b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

// ---- 4-bit side format of the pair tensors' low halves (prefill GEMMs) ----------------------------------------
// The low half of an fp16 pair is 2^-11 of the value it corrects, so its product with the weights needs only a few
// good bits.  In the large-tile GEMM it is therefore contracted by the block-scaled 4-bit MFMA (32x32x64, four times
// the k extent of the fp16 MFMA per instruction at the same issue cost) against a 4-bit copy of the weights:
// elements are e2m1 (sign, then magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6), two per byte with the even k in the low
// nibble, and a group of elements (128 consecutive k of an activation row; a whole row of a weight matrix) shares a
// power-of-two scale stored as an E8M0 byte (scale = 2^(byte - 127)), chosen as the smallest that brings the group's
// largest magnitude to 6 or below.  A CPU simulation of the rounding (tests/test_precision_design_cpu.py) shows the
// logit error of the rollout unchanged within a few per cent of its rms against fp16 low halves.
__device__ __forceinline__ uint32_t fp4_scale_byte(float amax) {
  const uint32_t bits = __float_as_uint(amax);
  const int e = (int)(bits >> 23) - 2 + ((bits & 0x7fffffu) > 0x400000u ? 1 : 0);   // amax = m 2^x: 6 * 2^(x-2) covers m <= 1.5
  return (uint32_t)min(max(e, 1), 254);
}
__device__ __forceinline__ float fp4_inv_scale(uint32_t byte) { return __uint_as_float((254u - byte) << 23); }   // 2^(127 - byte)
// nearest e2m1 code of v (already divided by the scale, |v| <= 6)
__device__ __forceinline__ uint32_t fp4_code(float v) {
  const float a = fabsf(v);
  const uint32_t c = (uint32_t)(a > 0.25f) + (uint32_t)(a > 0.75f) + (uint32_t)(a > 1.25f) + (uint32_t)(a > 1.75f) +
                     (uint32_t)(a > 2.5f) + (uint32_t)(a > 3.5f) + (uint32_t)(a > 5.f);
  return c | (v < 0.f ? 8u : 0u);
}
// Scale bytes of the activation rows, as the large-tile GEMM fetches them: for k-group t (128 columns) the four bytes
// of rows r, r + 32, r + 64, r + 96 of a 128-row group lie in one 32-bit word, the 32 words of a group side by side.
// groups = number of 128-row groups the array was laid out for (twice the number of 256-row tiles).
__host__ __device__ __forceinline__ size_t fp4_row_scale_offset(int m, int t, int groups) {
  return (((size_t)t * groups + (m >> 7)) * 32 + (m & 31)) * 4 + ((m >> 5) & 3);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}

// ---- KV-cache page -------------------------------------------------------------------------
// One page holds 16 tokens of one KV head with head_dim 128 in fp16: 4096 B of keys followed by
// 4096 B of values, both pre-arranged as MFMA operands so that a wavefront reads a page with
// eight fully coalesced 16 B-per-lane loads and feeds the registers to the matrix cores as is.
//   keys:   16 B chunk (kk, lane) at kk*1024 + lane*16 holds K[token lane&15][dims 8*(4kk + (lane>>4)) .. +8]
//   values: 16 B chunk (j, lane) at 4096 + j*1024 + lane*16 holds, for tokens 4*(lane>>4) .. +4,
//           V[token][dim 32j + (lane&15)] in its first 8 B and V[token][dim 32j + 16 + (lane&15)] in the rest
// Working layout of a 16-bit weight matrix W [N, K] (N % 16 == 0, K % 128 == 0): tiles of 16 rows x 128 columns,
// 4 KB each; inside a tile the halves are ordered [k/32 % 4][row % 16][k/8 % 4][k % 8].  Tiles are grouped in slabs
// of 16 row-blocks (256 rows; the last slab of a matrix may hold fewer), slab after slab, and inside a slab they are
// ordered k-step major: [k/128][row-block in slab].  A wavefront of the weight-streaming GEMM takes one k-step of its
// 16 rows with four loads of 1 KB of consecutive bytes (whole cache lines, so the nontemporal hint pays), the eight
// wavefronts of a workgroup together read 32 KB of consecutive bytes per k-step (measured: a weight stream in which
// each wavefront walks a run of its own, 128 KB apart, reaches 4.1-5.5 TB/s on the decode shapes, this order 5.0-5.9),
// and the large-tile GEMM finds the 64 bytes of one (row, 32-column k-tile) together.  A slab is 256 whole rows, so
// a block of rows that starts at a multiple of 256 occupies the same bytes as in the row-major matrix, which is what
// the in-place conversion relies on.  Row-blocks in the slab of row-block rb, and offset in halves of element (n, k):
constexpr int WSLAB_RB = 16;
__host__ __device__ __forceinline__ int wslab_blocks(int rb, int N) {
  const int left = (N >> 4) - (rb & ~(WSLAB_RB - 1));
  return left < WSLAB_RB ? left : WSLAB_RB;
}
__host__ __device__ __forceinline__ size_t wtile_offset(int n, int k, int K, int N) {
  const int rb = n >> 4, s0 = rb & ~(WSLAB_RB - 1);
  const size_t tile = (size_t)s0 * (size_t)(K >> 7) + (size_t)(k >> 7) * (size_t)wslab_blocks(rb, N) + (size_t)(rb - s0);
  return tile * 2048 + (size_t)(((k >> 5) & 3) * 512 + (n & 15) * 32 + (k & 31));
}

constexpr int KV_PAGE_TOKENS = 16;
constexpr int KV_HEAD_DIM = 128;
constexpr int KV_PAGE_BYTES = 8192;
__host__ __device__ __forceinline__ int kpage_offset(int slot, int dim) {
  int c = dim >> 3, e = dim & 7;
  return (c >> 2) * 1024 + (((c & 3) << 4) + slot) * 16 + e * 2;
}
__host__ __device__ __forceinline__ int vpage_offset(int slot, int dim) {
  int j = dim >> 5, r = dim & 31;
  return 4096 + j * 1024 + (((slot >> 2) << 4) + (r & 15)) * 16 + (r >> 4) * 8 + (slot & 3) * 2;
}
