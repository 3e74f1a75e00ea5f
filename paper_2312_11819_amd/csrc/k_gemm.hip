// GEMMs of the rollout, out = A[M,K] * W[N,K]^T with both operands K-contiguous.
//   gemm_h16_dma_kernel : large-tile fp16 MFMA GEMM for prefill (M = thousands of tokens): 256x256x32 block tile,
//                         4 wavefronts of 128x128, LDS ring filled by LDS-DMA loads, 32x32x16 MFMA; pair inputs may
//                         carry their low halves in 4 bits, contracted by the block-scaled 32x32x64 MFMA.
//   gemm_skinny_kernel  : weight-streaming GEMM for decode (M = batch <= 128; up to 256 where the split-K form of the
//                         large-tile GEMM does not apply): W is the MFMA row operand read straight from HBM into
//                         registers exactly once, the activation slice is staged in LDS, split-K partial sums go
//                         to a workspace that the consumer kernel adds up in a fixed order.
//   gemm_skinny_xres_kernel : the same with the activation slice of a split resident in LDS (QKV at <= 64 rows).
//   gemm_f32_kernel     : plain-ALU fp32 GEMM for the small fp32 configuration.
#include <stdlib.h>

#include <algorithm>

#include "common.h"
#include "kernels.h"

namespace {

// ---------------------------------------------------------------------------------------------------
// Large-tile GEMM: 256x256 block tile, four wavefronts (one per SIMD) of 128x128, 32x32x16 MFMA with the 256
// accumulator registers of a wavefront in AGPRs, k-tiles of 32 that travel global memory -> LDS by LDS-DMA loads
// (no staging registers) through a ring of NS stages of 32 KB.
//   * A wavefront-wide DMA load writes lane i's 16 bytes to LDS base + 16 i, so one instruction fills sixteen
//     64-byte tile rows.  To keep the later 16-byte MFMA operand reads free of bank conflicts (64 banks: sixteen
//     lanes, i.e. sixteen consecutive rows, are served together and must cover 256 distinct bytes) the 16-byte chunk c
//     of row r is stored at slot c ^ ((r >> 2) & 3); the permutation is applied on the global side (each lane
//     fetches the chunk that belongs in its slot).
//   * The compiler would wait for every outstanding DMA load before any LDS read it knows about, which would
//     serialise the pipeline, so the operand reads are issued as inline ds_read_b128 and their completion is
//     awaited explicitly (s_waitcnt lgkmcnt); the barrier is the bare s_barrier for the same reason.
//   * One wavefront per SIMD has nobody to hide its issue slots behind: the sixteen operand reads and eight DMA
//     loads of a k-tile are interleaved by hand between pairs of MFMAs (scheduling barriers pin the order), and the
//     reads of the next half-tile are in flight while the current one multiplies.
//   * Rows of the W tile are permuted on the way in: MFMA column c of the 32-column blocks j = 2 jp and 2 jp + 1
//     holds output columns 2 c and 2 c + 1 of a 64-column group, so a lane owns two adjacent outputs and a store
//     instruction writes whole 128-byte (fp16) or 256-byte (fp32) row segments.
//   * Measured on MI355X: the k loop alone sustains about 1.0-1.1 PFLOP/s on random fp16 data (the MFMA pipe itself,
//     fed from registers, 1.6 PFLOP/s on such data and 2.3-2.5 on zeros: the clock follows the data).
constexpr int DMA_NS = 4;            // LDS stages
constexpr int DMA_STAGE = 512 * 64;  // bytes per stage: 256 A rows + 256 W rows of 32 halves

typedef unsigned __attribute__((ext_vector_type(4))) u32x4_t;  // native vector: can live in an asm "v" operand
template <int OFF>
__device__ __forceinline__ u32x4_t lds_read128(uint32_t addr) {
  u32x4_t v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
__device__ __forceinline__ f32x16_t mfma_32x32x16_v(u32x4_t a, u32x4_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}
__device__ __forceinline__ uint32_t lds_read32(uint32_t addr) {
  uint32_t v;
  asm volatile("ds_read_b32 %0, %1" : "=v"(v) : "v"(addr));
  return v;
}
// D(32x32) += A(32x64) * B(64x32) with 4-bit (e2m1) operands and one power-of-two scale per lane and operand: lane l
// supplies row/column (l & 31) and the 32 consecutive k of group l >> 5 as 16 bytes (even k in the low nibble); byte
// SELA of sa / SELB of sb is the E8M0 scale of the lane's 32 elements.  Same issue cost as the 32x32x16 fp16 MFMA
// (measured), four times its k extent; the accumulator layout is that of the fp16 MFMA.
typedef int __attribute__((ext_vector_type(4))) i32x4_t;
template <int SELA, int SELB>
__device__ __forceinline__ f32x16_t mfma_32x32x64_f4(u32x4_t a, u32x4_t b, f32x16_t c, uint32_t sa, uint32_t sb) {
  const i32x4_t ai = __builtin_bit_cast(i32x4_t, a), bi = __builtin_bit_cast(i32x4_t, b);
  return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(__builtin_shufflevector(ai, ai, 0, 1, 2, 3, -1, -1, -1, -1),
                                                         __builtin_shufflevector(bi, bi, 0, 1, 2, 3, -1, -1, -1, -1), c, 4, 4,
                                                         SELA, (int)sa, SELB, (int)sb);
}
#define LDS_WAIT8(N, f0, f1, f2, f3, f4, f5, f6, f7) \
  asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(f0), "+v"(f1), "+v"(f2), "+v"(f3), "+v"(f4), "+v"(f5), "+v"(f6), "+v"(f7))
#define LDS_WAIT9(N, f0, f1, f2, f3, f4, f5, f6, f7, f8) \
  asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(f0), "+v"(f1), "+v"(f2), "+v"(f3), "+v"(f4), "+v"(f5), "+v"(f6), "+v"(f7), "+v"(f8))

// LO4 form: what the low-half phase of the k loop needs besides A and W
struct Lo4Args {
  const void* w4;                  // 4-bit copy of W (launch_to_w4_tiled)
  const unsigned char* w_scale;    // its scale byte per row of W
  const unsigned char* a_scale;    // scale bytes of A's low halves, fp4_row_scale_offset order
  int groups;                      // 128-row groups that order was laid out for
};

// SPLIT: split-K form for a few hundred rows (large decode batches), where the output tiles alone cannot fill the
// chip: workgroup (tile, split) contracts k-tiles [kw0, kw1) of W only and stores its fp32 tile into plane `split` of
// `out` (plane_stride floats apart); the consumer kernel adds the planes in a fixed order.  With hi|lo inputs the
// split walks (k-tile, hi), (k-tile, lo), ... so that the W tile fetched for the hi half is still in L2 for the lo half.
// LO4: A rows are [hi (K) | 4-bit low halves (K / 2 bytes) | unused] at the pitch of the pair form.  The k loop runs
// the K / 32 fp16 k-tiles (SPLIT: those of its split, which begins at a multiple of four) and then the K / 128 stages
// of the low halves that cover the same columns, against the 4-bit copy of W: such a stage has the
// byte layout of an fp16 stage (64 bytes per row: here 128 columns), the same DMA loads, operand reads and schedule,
// and one 4-bit MFMA where the fp16 phase has one fp16 MFMA - a quarter of the pair form's second pass.  The scale
// bytes of the A rows travel with their stage: every wavefront brings the 128 words of its own rows into a small LDS
// ring by one more DMA load per stage (issued in the fp16 phase too, so that every stage counts the same number of
// memory operations) and reads its word back when the stage is consumed.
template <int EPI, bool SPLIT, bool LO4 = false>
__global__ __launch_bounds__(256) void gemm_h16_dma_kernel(const h16_t* __restrict__ A, const h16_t* __restrict__ W,
                                                            void* __restrict__ out, int M, int N, int K, int tilesM,
                                                            int tilesN, int a_dual, int nsplit, size_t plane_stride,
                                                            RopeEpi re, Lo4Args l4) {
  // a_dual: A rows are [hi (K) | lo (K)]; the k loop then runs over 2K columns of A against W's K columns twice.
  constexpr int NS = DMA_NS, DIST = NS - 1, LPT = 8;  // LPT: DMA loads per thread and k-tile
  constexpr int VMS = LPT + (LO4 ? 1 : 0);            // memory operations per wavefront and stage
  static_assert(!(LO4 && EPI == EPI_SWIGLU), "the 4-bit low-half phase exists for the plain, the split-K and the QKV forms");
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int pid = blockIdx.x;
  int split = 0;
  if (SPLIT) {
    split = pid % nsplit;
    pid /= nsplit;
  }
  const int total = tilesM * tilesN;
  if (!SPLIT && (total & 7) == 0) pid = (pid & 7) * (total >> 3) + (pid >> 3);  // consecutive tiles on one XCD (shared L2)
  const int band = 8 * tilesN;
  const int first_m = (pid / band) * 8;
  const int gsz = min(tilesM - first_m, 8);
  const int tm = first_m + (pid % band) % gsz;
  const int tn = (pid % band) / gsz;
  const int m0 = tm * 256;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  // global row of W behind row R (0..255) of the LDS tile: wavefront half wn, 32-column block j, MFMA column c
  auto wrow = [&](int R) -> int {
    const int wv = R >> 7, j = (R >> 5) & 3, c = R & 31;
    if (EPI == EPI_SWIGLU) return (j >> 1) * N + tn * 128 + wv * 64 + 2 * c + (j & 1);  // gate blocks 0,1; up blocks 2,3
    return tn * 256 + wv * 128 + 64 * (j >> 1) + 2 * c + (j & 1);
  };

  // DMA sources: wavefronts 0,1 bring the A rows (16 row groups of 16 each), 2,3 the W rows
  const bool loads_a = wave < 2;
  const char* gbase = loads_a ? (const char*)A : (const char*)W;
  uint32_t go[LPT];
#pragma unroll
  for (int it = 0; it < LPT; ++it) {
    const int row = 16 * ((wave & 1) * 8 + it) + (lane >> 2);
    const int grow = loads_a ? min(m0 + row, M - 1) : wrow(row);
    const uint32_t chunk = (uint32_t)((lane & 3) ^ ((row >> 2) & 3));
    // A is row-major; W is in the tiled working layout (16-row x 128-column tiles of 4 KB, a row's 64 bytes of one
    // k-tile together)
    go[it] = loads_a ? (uint32_t)grow * (uint32_t)(a_dual ? 2 * K : K) * 2u + chunk * 16u
                     : (uint32_t)(wtile_offset(grow, 0, K, EPI == EPI_SWIGLU ? 2 * N : N) * 2) + chunk * 16u;
  }
  const int nkw = K / 32;                 // k-tiles of W
  int kw0 = 0, kw1 = nkw;                 // this workgroup's k-tiles of W
  if (SPLIT) {
    int per = (nkw + nsplit - 1) / nsplit;
    if (LO4) per = (per + 3) & ~3;        // a low-half stage covers four k-tiles: splits begin at multiples of four
    kw0 = split * per;
    kw1 = min(nkw, kw0 + per);
  }
  const int nhi = LO4 ? kw1 - kw0 : 0;    // LO4: fp16 k-tiles [kw0, kw1), then the low-half stages [kw0 / 4, kw1 / 4)
  const int nlo = LO4 ? nhi / 4 : 0, lo0 = kw0 >> 2;
  const int nk = LO4 ? nhi + nlo : SPLIT ? (kw1 - kw0) * (a_dual ? 2 : 1) : (a_dual ? 2 * nkw : nkw);  // k-tiles of the product
  // 4-bit W: the tiled order of a matrix with K / 4 columns, so its slabs are a quarter as long (tile tn = slab tn)
  const size_t w4_adj = LO4 ? (size_t)tn * WSLAB_RB * (size_t)((K >> 7) - (K >> 9)) * 4096 : 0;
  typedef __attribute__((address_space(3))) void lds_void;
  typedef const __attribute__((address_space(1))) void g_void;
  char* dma_dst = smem + wave * 8192;
  // tile KT of this wavefront's operand (past the end: the last tile again, into a stage nobody reads any more)
  auto tile_src = [&](int kt) -> const char* {
    kt = min(kt, nk - 1);
    if (LO4) {
      if (kt >= nhi) {
        const int kl = lo0 + kt - nhi;
        if (loads_a) return gbase + (size_t)K * 2 + (size_t)kl * 64;
        return (const char*)l4.w4 + ((size_t)(kl >> 2) * (WSLAB_RB * 4096) + (size_t)(kl & 3) * 1024) - w4_adj;
      }
      const int kw = kw0 + kt;
      if (loads_a) return gbase + (size_t)kw * 64;
      return gbase + (size_t)(kw >> 2) * (WSLAB_RB * 4096) + (size_t)(kw & 3) * 1024;
    }
    if (SPLIT) {
      const int kw = kw0 + (a_dual ? kt >> 1 : kt);
      if (loads_a) return gbase + ((a_dual && (kt & 1)) ? (size_t)K * 2 : (size_t)0) + (size_t)kw * 64;
      return gbase + (size_t)(kw >> 2) * (WSLAB_RB * 4096) + (size_t)(kw & 3) * 1024;   // (every slab is full: rows % 256 == 0)
    }
    if (loads_a) return gbase + (size_t)kt * 64;
    const int kw = kt >= nkw ? kt - nkw : kt;
    return gbase + (size_t)(kw >> 2) * (WSLAB_RB * 4096) + (size_t)(kw & 3) * 1024;   // (every slab is full: rows % 256 == 0)
  };
#define DMA1(SRC, SOFF, IT) \
  __builtin_amdgcn_global_load_lds((g_void*)((SRC) + go[IT]), (lds_void*)(dma_dst + (SOFF) + (IT) * 1024), 16, 0, 0);
  // scale words of this wavefront's 128 A rows for stage KT (clamped into the low-half phase), one per lane (the upper
  // half of the wavefront repeats the lower), into this wavefront's 256 bytes of the ring slot of the stage at SOFF
  const char* sa_src = LO4 ? (const char*)l4.a_scale + ((size_t)((m0 >> 7) + wm) * 32 + (lane & 31)) * 4 : nullptr;
  const size_t sa_stride = (size_t)l4.groups * 128;
  char* sc_dst = smem + NS * DMA_STAGE + wave * 256;
#define DMAS(KT, SOFF)                                                                                             \
  if (LO4) {                                                                                                       \
    const int kl_ = lo0 + min(max((KT) - nhi, 0), nlo - 1);                                                        \
    __builtin_amdgcn_global_load_lds((g_void*)(sa_src + (size_t)kl_ * sa_stride), (lds_void*)(sc_dst + ((SOFF) >> 5)), 4, 0, 0); \
  }

  f32x16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // operand read addresses: row (lane & 31) of a 32-row block, chunk 2 ks + (lane >> 5), stored at slot chunk ^ ((row >> 2) & 3)
  const uint32_t lds0 = (uint32_t)(size_t)smem;
  const uint32_t sw = (uint32_t)((lane >> 2) & 3);
  uint32_t a_rd[2], b_rd[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const uint32_t slot = (uint32_t)(2 * ks + (lane >> 5)) ^ sw;
    a_rd[ks] = lds0 + (uint32_t)((wm * 128 + (lane & 31)) * 64) + slot * 16;
    b_rd[ks] = lds0 + (uint32_t)((256 + wn * 128 + (lane & 31)) * 64) + slot * 16;
  }
#pragma unroll
  for (int d = 0; d < DIST; ++d) {
    const char* src = tile_src(d);
#pragma unroll
    for (int it = 0; it < LPT; ++it) DMA1(src, d * DMA_STAGE, it)
    DMAS(d, d * DMA_STAGE)
  }
  // scale bytes of this lane's four W rows (32-column blocks j = 0..3), the same for every stage
  uint32_t scb = 0, sca = 0, scn = 0;   // scale words: W rows; A rows of the current and of the next stage
  const uint32_t sc_rd = (uint32_t)(size_t)smem + NS * DMA_STAGE + wave * 256 + lane * 4;
  if (LO4) {
#pragma unroll
    for (int j = 0; j < 4; ++j) scb |= (uint32_t)l4.w_scale[wrow(wn * 128 + j * 32 + (lane & 31))] << (8 * j);
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(scb)::"memory");   // (ordinary loads: keep them out of the DMA accounting below)
  }
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DIST - 1) * VMS) : "memory");
  __builtin_amdgcn_s_barrier();
  u32x4_t p0, p1, p2, p3, p4, p5, p6, p7, q0, q1, q2, q3, q4, q5, q6, q7;
  uint32_t so_cur = 0;                     // stage of k-tile kt
  uint32_t so_issue = DIST * DMA_STAGE;    // stage that k-tile kt + DIST goes to
  {
    const uint32_t ra = a_rd[0], rb = b_rd[0];
    p4 = lds_read128<0>(rb); p5 = lds_read128<2048>(rb); p6 = lds_read128<4096>(rb); p7 = lds_read128<6144>(rb);
    p0 = lds_read128<0>(ra); p1 = lds_read128<2048>(ra); p2 = lds_read128<4096>(ra); p3 = lds_read128<6144>(ra);
  }
#define SB0 __builtin_amdgcn_sched_barrier(0);
#define MFH(I, J, SA, SB) acc[I][J] = mfma_32x32x16_v(SA, SB, acc[I][J]);
#define MF4(I, J, SA, SB) acc[I][J] = mfma_32x32x64_f4<I, J>(SA, SB, acc[I][J], sca, scb);
  // One stage: its first half (chunks 0, 1 of every row: 16 columns of an fp16 k-tile, 64 of a low-half stage) from p
  // while the second half is read into q; then the barrier; then the second half from q while the first half of the
  // next stage (and its scale word) is read into p and the stage DIST ahead is requested.
#define KSTAGE(MF)                                                                                                  \
  {                                                                                                                 \
    {                                                                                                               \
      const uint32_t ra = a_rd[1] + so_cur, rb = b_rd[1] + so_cur;                                                  \
      LDS_WAIT9(0, p0, p1, p2, p3, p4, p5, p6, p7, scn);                                                            \
      sca = scn;                                                                                                    \
      SB0 MF(0, 0, p0, p4) MF(0, 1, p0, p5) SB0 q4 = lds_read128<0>(rb);                                            \
      SB0 MF(0, 2, p0, p6) MF(0, 3, p0, p7) SB0 q5 = lds_read128<2048>(rb);                                         \
      SB0 MF(1, 0, p1, p4) MF(1, 1, p1, p5) SB0 q6 = lds_read128<4096>(rb);                                         \
      SB0 MF(1, 2, p1, p6) MF(1, 3, p1, p7) SB0 q7 = lds_read128<6144>(rb);                                         \
      SB0 MF(2, 0, p2, p4) MF(2, 1, p2, p5) SB0 q0 = lds_read128<0>(ra);                                            \
      SB0 MF(2, 2, p2, p6) MF(2, 3, p2, p7) SB0 q1 = lds_read128<2048>(ra);                                         \
      SB0 MF(3, 0, p3, p4) MF(3, 1, p3, p5) SB0 q2 = lds_read128<4096>(ra);                                         \
      SB0 MF(3, 2, p3, p6) MF(3, 3, p3, p7) SB0 q3 = lds_read128<6144>(ra);                                         \
      SB0                                                                                                           \
    }                                                                                                               \
    /* stage kt + 1 has landed (this wavefront's share: the barrier covers the others'), and nobody reads the */    \
    /* stage of k-tile kt - 1 any more, which is where stage kt + DIST goes */                                      \
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DIST - 2) * VMS) : "memory");                                         \
    __builtin_amdgcn_s_barrier();                                                                                   \
    {                                                                                                               \
      const char* src = tile_src(kt + DIST);                                                                        \
      const uint32_t so_i = so_issue;                                                                               \
      so_cur = so_cur + DMA_STAGE == NS * DMA_STAGE ? 0 : so_cur + DMA_STAGE;                                       \
      so_issue = so_issue + DMA_STAGE == NS * DMA_STAGE ? 0 : so_issue + DMA_STAGE;                                 \
      const uint32_t ra = a_rd[0] + so_cur, rb = b_rd[0] + so_cur;                                                  \
      LDS_WAIT8(0, q0, q1, q2, q3, q4, q5, q6, q7);                                                                 \
      SB0 MF(0, 0, q0, q4) MF(0, 1, q0, q5) SB0 p4 = lds_read128<0>(rb);    DMA1(src, so_i, 0)                      \
      SB0 MF(0, 2, q0, q6) MF(0, 3, q0, q7) SB0 p5 = lds_read128<2048>(rb); DMA1(src, so_i, 1)                      \
      SB0 MF(1, 0, q1, q4) MF(1, 1, q1, q5) SB0 p6 = lds_read128<4096>(rb); DMA1(src, so_i, 2)                      \
      SB0 MF(1, 2, q1, q6) MF(1, 3, q1, q7) SB0 p7 = lds_read128<6144>(rb); DMA1(src, so_i, 3)                      \
      SB0 MF(2, 0, q2, q4) MF(2, 1, q2, q5) SB0 p0 = lds_read128<0>(ra);    DMA1(src, so_i, 4)                      \
      SB0 MF(2, 2, q2, q6) MF(2, 3, q2, q7) SB0 p1 = lds_read128<2048>(ra); DMA1(src, so_i, 5)                      \
      SB0 MF(3, 0, q3, q4) MF(3, 1, q3, q5) SB0 p2 = lds_read128<4096>(ra); DMA1(src, so_i, 6)                      \
      SB0 MF(3, 2, q3, q6) MF(3, 3, q3, q7) SB0 p3 = lds_read128<6144>(ra); DMA1(src, so_i, 7)                      \
      SB0 DMAS(kt + DIST, so_i)                                                                                     \
      if (LO4) scn = lds_read32(sc_rd + (so_cur >> 5));                                                             \
    }                                                                                                               \
  }
  {
    int kt = 0;
    const int nk_hi = LO4 ? nhi : nk;
    for (; kt < nk_hi; ++kt) KSTAGE(MFH)
    if (LO4)
      for (; kt < nk; ++kt) KSTAGE(MF4)
  }
#undef KSTAGE
#undef MFH
#undef MF4
#undef SB0
#undef DMA1
#undef DMAS
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // the trailing prefetches (never consumed) are done

  const int c2 = 2 * (lane & 31);
  if (EPI == EPI_QKV_ROPE) {
    // this wavefront's 128 columns are head hd of the fused q|k|v row; the lane holds dimensions c2, c2 + 1 (blocks 0, 1)
    // and 64 + c2, 64 + c2 + 1 (blocks 2, 3) of it: the pairs the rotation mixes
    const int hd = tn * 2 + wn;
    const bool is_q = hd < re.Hq, is_k = !is_q && hd < re.Hq + re.Hkv;
    const int kvh = is_k ? hd - re.Hq : hd - re.Hq - re.Hkv;
    if (!is_q && !is_k) {
      // Values: a lane holds four consecutive rows (e & 3) of each of its four dimensions, and the value layout keeps
      // the four tokens of an aligned group of slots next to each other: where the four rows are four consecutive
      // positions of one sequence starting at a multiple of four, they go out as one 8-byte store per dimension
      // instead of four 2-byte ones (a query of 512 tokens: always).
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int eg = 0; eg < 4; ++eg) {
          const int m = m0 + wm * 128 + i * 32 + 8 * eg + 4 * (lane >> 5);
          asm volatile("" ::: "memory");
          if (m >= M) continue;
          const int pos = re.row_pos[m];
          const int bseq = re.row_seq ? re.row_seq[m] : m;
          const int m3 = min(m + 3, M - 1);
          const bool together = m + 3 < M && (pos & 3) == 0 && re.row_pos[m3] == pos + 3 && re.row_seq != nullptr && re.row_seq[m3] == bseq;   // (no row_seq: every row is a sequence of its own)
          if (together) {
            const int blk = re.block_table[(size_t)bseq * re.max_blocks + (pos >> 4)];
            char* page = (char*)re.kv_pool_layer + ((size_t)kvh * re.n_blocks + blk) * KV_PAGE_BYTES;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int dim = c2 + (j & 1) + 64 * (j >> 1);   // blocks 0, 1: c2, c2 + 1; blocks 2, 3: 64 + c2, 65 + c2
              *(uint2*)(page + vpage_offset(pos & 15, dim)) =
                  make_uint2(pack_h16x2(acc[i][j][4 * eg], acc[i][j][4 * eg + 1]), pack_h16x2(acc[i][j][4 * eg + 2], acc[i][j][4 * eg + 3]));
            }
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              if (m + r >= M) continue;
              const int pr = re.row_pos[m + r], br = re.row_seq ? re.row_seq[m + r] : m + r;
              char* page = (char*)re.kv_pool_layer + ((size_t)kvh * re.n_blocks + re.block_table[(size_t)br * re.max_blocks + (pr >> 4)]) * KV_PAGE_BYTES;
#pragma unroll
              for (int j = 0; j < 4; ++j)
                *(h16_t*)(page + vpage_offset(pr & 15, c2 + (j & 1) + 64 * (j >> 1))) = f32_to_h16(acc[i][j][4 * eg + r]);
            }
          }
        }
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm * 128 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        asm volatile("" ::: "memory");   // one row at a time: hoisting the 64 rows' loads to the top would spill the accumulators
        if (m >= M) continue;
        const int pos = re.row_pos[m];
        float a0 = acc[i][0][e], a1 = acc[i][1][e], b0 = acc[i][2][e], b1 = acc[i][3][e];
        if (is_q || is_k) {
          const float2 cs = *(const float2*)(re.cos_t + (size_t)pos * 64 + c2), sn = *(const float2*)(re.sin_t + (size_t)pos * 64 + c2);
          const float r00 = a0 * cs.x - b0 * sn.x, r10 = b0 * cs.x + a0 * sn.x;
          const float r01 = a1 * cs.y - b1 * sn.y, r11 = b1 * cs.y + a1 * sn.y;
          a0 = r00; b0 = r10; a1 = r01; b1 = r11;
        }
        if (is_q) {
          h16_t* qo = (h16_t*)re.q_out + ((size_t)m * re.Hq + hd) * 256 + c2;   // [hi (128) | lo (128)]
          h16_t h[4], l[4];
          split_h16(a0, h[0], l[0]); split_h16(a1, h[1], l[1]); split_h16(b0, h[2], l[2]); split_h16(b1, h[3], l[3]);
          *(uint32_t*)(qo) = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
          *(uint32_t*)(qo + 64) = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
          *(uint32_t*)(qo + 128) = (uint32_t)l[0] | ((uint32_t)l[1] << 16);
          *(uint32_t*)(qo + 192) = (uint32_t)l[2] | ((uint32_t)l[3] << 16);
        } else {
          const int bseq = re.row_seq ? re.row_seq[m] : m;
          const int blk = re.block_table[(size_t)bseq * re.max_blocks + (pos >> 4)], slot = pos & 15;
          char* page = (char*)re.kv_pool_layer + ((size_t)kvh * re.n_blocks + blk) * KV_PAGE_BYTES;
          // two adjacent dimensions share a 16-byte chunk of the key layout
          *(uint32_t*)(page + kpage_offset(slot, c2)) = pack_h16x2(a0, a1);
          *(uint32_t*)(page + kpage_offset(slot, c2 + 64)) = pack_h16x2(b0, b1);
        }
      }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int m = m0 + wm * 128 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
      if (m >= M) continue;
      if (EPI == EPI_SWIGLU) {
        const int f = tn * 128 + wn * 64 + c2;
        const float g0 = acc[i][0][e], g1 = acc[i][1][e], u0 = acc[i][2][e], u1 = acc[i][3][e];
        const float v0 = g0 / (1.f + __expf(-g0)) * u0, v1 = g1 / (1.f + __expf(-g1)) * u1;
        *(uint32_t*)((h16_t*)out + (size_t)m * N + f) = pack_h16x2(v0, v1);
      } else {
#pragma unroll
        for (int jp = 0; jp < 2; ++jp) {
          const int n = tn * 256 + wn * 128 + 64 * jp + c2;
          const float v0 = acc[i][2 * jp][e], v1 = acc[i][2 * jp + 1][e];
          if (EPI == EPI_STORE_F32)
            *(float2*)((float*)out + (SPLIT ? (size_t)split * plane_stride : (size_t)0) + (size_t)m * N + n) = make_float2(v0, v1);
          if (EPI == EPI_RESID_F32) {
            float2* o = (float2*)((float*)out + (size_t)m * N + n);
            float2 r = *o;
            r.x += v0; r.y += v1;
            *o = r;
          }
          if (EPI == EPI_STORE_ACT) *(uint32_t*)((h16_t*)out + (size_t)m * N + n) = pack_h16x2(v0, v1);
        }
      }
    }
  }
}

template <int EPI>
hipError_t launch_large_dma(hipStream_t s, const void* A, const void* W, void* out, int M, int N, int K, int a_dual,
                            bool configure_only = false) {
  constexpr int SMEM = DMA_NS * DMA_STAGE;
  auto kern = gemm_h16_dma_kernel<EPI, false>;
  if (configure_only) return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
  int tilesM = (M + 255) / 256;
  int tilesN = (EPI == EPI_SWIGLU) ? N / 128 : N / 256;
  kern<<<tilesM * tilesN, 256, SMEM, s>>>((const h16_t*)A, (const h16_t*)W, out, M, N, K, tilesM, tilesN, a_dual, 1, 0, RopeEpi{}, Lo4Args{});
  return hipGetLastError();
}

hipError_t launch_large_dma_qkv_rope(hipStream_t s, const void* A, const void* W, int M, int N, int K, const RopeEpi* re,
                                     bool configure_only = false) {
  constexpr int SMEM = DMA_NS * DMA_STAGE;
  auto kern = gemm_h16_dma_kernel<EPI_QKV_ROPE, false>;
  if (configure_only) return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
  const int tilesM = (M + 255) / 256, tilesN = N / 256;
  kern<<<tilesM * tilesN, 256, SMEM, s>>>((const h16_t*)A, (const h16_t*)W, nullptr, M, N, K, tilesM, tilesN, 1, 1, 0, *re, Lo4Args{});
  return hipGetLastError();
}

// The form with 4-bit low halves (EPI_STORE_F32, EPI_RESID_F32 or EPI_QKV_ROPE)
template <int EPI>
hipError_t launch_large_dma_lo4(hipStream_t s, const void* A, const void* W, void* out, int M, int N, int K, const RopeEpi* re,
                                const Lo4Args* l4, bool configure_only = false) {
  constexpr int SMEM = DMA_NS * DMA_STAGE + DMA_NS * 1024;   // + the ring of scale words
  auto kern = gemm_h16_dma_kernel<EPI, false, true>;
  if (configure_only) return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
  const int tilesM = (M + 255) / 256, tilesN = N / 256;
  kern<<<tilesM * tilesN, 256, SMEM, s>>>((const h16_t*)A, (const h16_t*)W, out, M, N, K, tilesM, tilesN, 1, 1, 0,
                                          re ? *re : RopeEpi{}, *l4);
  return hipGetLastError();
}

// split-K form with 4-bit low halves
hipError_t launch_large_dma_split_lo4(hipStream_t s, const void* A, const void* W, float* part, int M, int N, int K, int nsplit,
                                      int plane_rows, const Lo4Args* l4, bool configure_only = false) {
  constexpr int SMEM = DMA_NS * DMA_STAGE + DMA_NS * 1024;
  auto kern = gemm_h16_dma_kernel<EPI_STORE_F32, true, true>;
  if (configure_only) return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
  const int tilesM = (M + 255) / 256, tilesN = N / 256;
  kern<<<tilesM * tilesN * nsplit, 256, SMEM, s>>>((const h16_t*)A, (const h16_t*)W, part, M, N, K, tilesM, tilesN, 1, nsplit,
                                                   (size_t)plane_rows * N, RopeEpi{}, *l4);
  return hipGetLastError();
}

// split-K form: fp32 partial planes part[split][plane_rows][N]
hipError_t launch_large_dma_split(hipStream_t s, const void* A, const void* W, float* part, int M, int N, int K, int a_dual,
                                  int nsplit, int plane_rows, bool configure_only = false) {
  constexpr int SMEM = DMA_NS * DMA_STAGE;
  auto kern = gemm_h16_dma_kernel<EPI_STORE_F32, true>;
  if (configure_only) return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
  const int tilesM = (M + 255) / 256, tilesN = N / 256;
  kern<<<tilesM * tilesN * nsplit, 256, SMEM, s>>>((const h16_t*)A, (const h16_t*)W, part, M, N, K, tilesM, tilesN, a_dual,
                                                   nsplit, (size_t)plane_rows * N, RopeEpi{}, Lo4Args{});
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
constexpr int SK = 128;                 // k extent of one staged activation slice
constexpr int SK_ROW = SK * 2 + 16;     // bytes per LDS row (padded)

// grid (Nw / (16 NW), nsplit), 64 NW threads; wavefront w owns W rows n0 + 16 w .. +16 and all M (<= 16 MB) columns
// (the fused gate/up form: 8 gate and 8 up rows per wavefront, grid ceil(F / 8 NW), last workgroup ragged).
// Loads run D - 1 k-steps ahead of the MFMAs through a register ring (weights and the activation slice alike:
// the memory counter retires in order, so both must share one prefetch distance); the activation slice then
// passes through a double-buffered LDS tile that the workgroup's wavefronts share.  D = 2 everywhere: on this
// memory system a deeper ring is slower, not faster - the bare weight stream of these grids measures 5.0-5.9 TB/s
// with three k-steps in flight per wavefront and 6.1-6.5 with one (QKV shape: 20.2 -> 16.4 us), and the whole
// kernels gain 1-2 us each.  What counts is that a workgroup's outstanding loads form one run of consecutive bytes.  What the time is made of,
// measured on MI355X on the 7B gate/up shape at 64 rows (37 us): the weight loads alone 29 us, the MFMAs +3, the
// LDS staging and its per-step barrier +1, the slice loads from L2 +2, the output stores +2.  Workgroups, not
// bytes, are the first-order term: the kernel is fastest with one workgroup per compute unit, all in flight from
// the first cycle (see the launchers for how the split count and the workgroup width are chosen for that).
template <int MB, int D, bool GLU, bool DUAL, int NW>
__global__ __launch_bounds__(64 * NW) void gemm_skinny_kernel(const h16_t* __restrict__ X, const h16_t* __restrict__ W,
                                                          float* __restrict__ part, int M, int Nw, int K,
                                                          int steps_per_split, int plane_rows) {
  static_assert(D == 2 || D == 4, "ring depth 2 or 4");
  // DUAL: X rows are [hi (K) | lo (K)] fp16 pairs; the LDS tile holds the hi rows followed by the lo rows and every
  // weight fragment is multiplied with both.
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int XR = DUAL ? 2 * MB : MB;   // 16-row blocks of the staged slice
  constexpr int XBYTES = 16 * XR * SK_ROW;
  constexpr int NT = 64 * NW;
  constexpr int XL = (256 * XR + NT - 1) / NT;   // 16-byte chunks of the slice each thread moves per k-step
  constexpr bool XEXACT = XL * NT == 256 * XR;   // otherwise the last round of chunks is taken by some threads only
  const int ldx = DUAL ? 2 * K : K;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, t = lane & 15, g = lane >> 4;
  // GLU: W = [gate rows | up rows] of F = Nw / 2 features each; the workgroup owns 8 NW features, each wavefront
  // 8 of them with the gate rows in MFMA rows 0..7 and the matching up rows in 8..15.  8 NW need not divide F: the
  // wavefronts of the last workgroup that fall beyond F go through the motions on rows 0.. and store nothing.
  const int n0 = GLU ? blockIdx.x * (8 * NW) : blockIdx.x * (16 * NW);
  const bool live = !GLU || n0 + 8 * w < (Nw >> 1);
  const int nb = live ? n0 + 8 * w : 0;
  const int nsteps_total = K / SK;
  const int s0 = blockIdx.y * steps_per_split;
  const int s1 = min(nsteps_total, s0 + steps_per_split);

  f32x4_t acc[MB];
#pragma unroll
  for (int i = 0; i < MB; ++i) acc[i] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

  const int wrow = GLU ? ((t < 8) ? nb + t : (Nw >> 1) + nb + (t - 8)) : n0 + 16 * w + t;
  // W is in the tiled working layout: consecutive k-steps of a row-block lie (row-blocks in its slab) tiles apart
  const h16_t* wp = W + wtile_offset(wrow, 8 * g, K, Nw);
  const size_t wstep = (size_t)wslab_blocks(wrow >> 4, Nw) * 2048;
  // Activation slice: 16 MB rows x 16 chunks of 16 B per k-step, MB chunks per thread.  Rows beyond M are read
  // from row M - 1 instead: they only feed output columns that are never stored.
  const h16_t* xp[XL];
  int xo[XL];
#pragma unroll
  for (int it = 0; it < XL; ++it) {
    int c = it * NT + tid;
    if (!XEXACT) c = min(c, 256 * XR - 1);            // (a thread without a chunk in the last round repeats the last chunk)
    const int r = c >> 4, kc = c & 15;                // r in [0, 16 XR): rows >= 16 MB are the lo parts
    int rr = DUAL ? r % (16 * MB) : r;
    xp[it] = X + (size_t)min(rr, M - 1) * ldx + ((DUAL && r >= 16 * MB) ? K : 0) + kc * 8;
    xo[it] = r * SK_ROW + kc * 16;
  }
  // Workgroups walk their k range from different starting points (wrapping around), so that they do not all
  // touch the same columns of W at the same time.
  const int nst = s1 - s0;
  // The starting point is a function of the rows, not of the workgroup shape, so that every output element is
  // accumulated in the same order whichever instantiation (4 or 8 wavefronts, any batch width) computes it.
  const unsigned grp = GLU ? (unsigned)n0 >> 6 : (unsigned)n0 >> 7;
  // (the pair-input variant walks k in order, like the resident-slice kernel that serves the same GEMMs at <= 64 rows)
  const int rot = (nst > 0 && !DUAL) ? (int)((grp * 5u + blockIdx.y * 3u) % (unsigned)nst) : 0;
  (void)NT;
  // Loads are issued without any branch around them (a step index past the end re-reads the last step, which
  // hits in cache): with straight-line code the compiler can keep D - 1 steps of loads in flight and wait only
  // for the oldest.
  auto step_off = [&](int i) -> size_t {   // the k-step behind ring index i
    int r = min(i, nst - 1) + rot;
    if (r >= nst) r -= nst;
    return (size_t)(s0 + r);
  };
  // Ring of D named slots (separate variables, so that they live in registers).  The weights are read once: the
  // nontemporal hint is worth 10 % on the gate/up and down projections.  In the pair-input variant it is worth 3-8 %
  // up to 32 rows (measured on the 13B and 70B shapes) but costs 3-5 % at 64 rows with their doubled activation slice
  // (7B output projection), so that variant uses it for the one- and two-block instantiations only.
  struct Slot { uint4 w[4]; uint4 x[XL]; };
  Slot r0, r1, r2, r3;
#define SKINNY_LOAD(S, I)                                                                                \
  {                                                                                                      \
    const size_t st_ = step_off(I);                                                                      \
    const h16_t* wq_ = wp + st_ * wstep;                                                                 \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk)                                                    \
        S.w[kk] = (DUAL && MB > 2) ? *(const uint4*)(wq_ + kk * 512) : load_stream16(wq_ + kk * 512);    \
    _Pragma("unroll") for (int it = 0; it < XL; ++it) S.x[it] = *(const uint4*)(xp[it] + st_ * SK);      \
  }
  // one k-step on slot S (LDS buffer PAR)
#define SKINNY_STEP(S, PAR)                                                                              \
  {                                                                                                      \
    char* buf = smem + (PAR) * XBYTES;                                                                   \
    _Pragma("unroll") for (int it = 0; it < XL; ++it)                                                    \
        if (XEXACT || it * NT + tid < 256 * XR) *(uint4*)(buf + xo[it]) = S.x[it];                       \
    __syncthreads();                                                                                     \
    uint4 xf[2][XR];                                                                                     \
    _Pragma("unroll") for (int mb = 0; mb < XR; ++mb)                                                    \
        xf[0][mb] = *(const uint4*)(buf + (mb * 16 + t) * SK_ROW + g * 16);                              \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) {                                                   \
      if (kk < 3) {                                                                                      \
        _Pragma("unroll") for (int mb = 0; mb < XR; ++mb)                                                \
            xf[(kk + 1) & 1][mb] = *(const uint4*)(buf + (mb * 16 + t) * SK_ROW + (kk + 1) * 64 + g * 16); \
      }                                                                                                  \
      _Pragma("unroll") for (int mb = 0; mb < XR; ++mb)                                                  \
          acc[mb % MB] = mfma_16x16x32(S.w[kk], xf[kk & 1][mb], acc[mb % MB]);                           \
    }                                                                                                    \
  }
  if (nst > 0) {
    int i = 0;
    if constexpr (D == 4) {
      SKINNY_LOAD(r0, 0)
      SKINNY_LOAD(r1, 1)
      SKINNY_LOAD(r2, 2)
      for (; i + 4 <= nst; i += 4) {
        SKINNY_LOAD(r3, i + 3)
        SKINNY_STEP(r0, 0)
        SKINNY_LOAD(r0, i + 4)
        SKINNY_STEP(r1, 1)
        SKINNY_LOAD(r1, i + 5)
        SKINNY_STEP(r2, 0)
        SKINNY_LOAD(r2, i + 6)
        SKINNY_STEP(r3, 1)
      }
      if (i < nst) {
        SKINNY_STEP(r0, 0)
        if (i + 1 < nst) {
          SKINNY_STEP(r1, 1)
          if (i + 2 < nst) SKINNY_STEP(r2, 0)
        }
      }
    } else {
      SKINNY_LOAD(r0, 0)
      for (; i + 2 <= nst; i += 2) {
        SKINNY_LOAD(r1, i + 1)
        SKINNY_STEP(r0, 0)
        SKINNY_LOAD(r0, i + 2)
        SKINNY_STEP(r1, 1)
      }
      if (i < nst) SKINNY_STEP(r0, 0)
      (void)r2; (void)r3;
    }
  }
#undef SKINNY_STEP
#undef SKINNY_LOAD
  if (GLU) {
    if (!live) return;
    // lane (t, g < 2) holds gate features 4g..4g+3 of column t, lane (t, g + 2) the matching up values
    h16_t* hout = (h16_t*)part;
    const int F = Nw >> 1;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      float up[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) up[i] = __shfl_xor(acc[mb][i], 32);
      int m = mb * 16 + t;
      if (g < 2 && m < M) {
        float hv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) hv[i] = acc[mb][i] / (1.f + __expf(-acc[mb][i])) * up[i];
        uint2 o;
        o.x = pack_h16x2(hv[0], hv[1]);
        o.y = pack_h16x2(hv[2], hv[3]);
        *(uint2*)(hout + (size_t)m * F + n0 + 8 * w + 4 * g) = o;
      }
    }
    return;
  }
  // split-K plane s holds plane_rows rows (>= M: the caller may compute a taller output in several row slabs)
  float* dst = part + (size_t)blockIdx.y * plane_rows * Nw;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    int m = mb * 16 + t;
    if (m < M) *(float4*)(dst + (size_t)m * Nw + n0 + 16 * w + 4 * g) = make_float4(acc[mb][0], acc[mb][1], acc[mb][2], acc[mb][3]);
  }
}

// ---------------------------------------------------------------------------------------------------
// Weight-streaming GEMM with the activation slice resident in LDS, for pair-input projections of up to 64 rows
// whose K is a multiple of 512 (QKV and output projection at d_model 4096 / 5120).  Grid (G, ns), ns = K / 512:
// workgroup (j, s) loads the slice X[:, 512 s .. 512 s + 512) (hi rows, then lo rows: 128 x 1 KB for 64 batch rows)
// into LDS once and then streams the k-range of the 128-row weight tiles j, j + G, j + 2 G, ... against it, writing
// one [M, 128] partial tile per weight tile into split plane s.  Compared with gemm_skinny_kernel the slice is
// fetched once per workgroup instead of once per weight tile (the counters showed those re-reads missing L2 under
// the weight stream and adding a quarter to the HBM traffic of these GEMMs), there is no barrier in the k loop, and
// the register ring of weight loads runs on across tile boundaries.  Accumulation order per output element is the
// same as in gemm_skinny_kernel<.., DUAL = true> (k ascending inside the split, hi then lo), so the two give
// identical bits.
constexpr int XRES_KS = 512;                  // k extent of a resident slice
constexpr int XRES_ROW = XRES_KS * 2 + 16;    // bytes per LDS row (padded: 16 lanes x 16 B cover all 64 banks)

template <int MB>
__global__ __launch_bounds__(512) void gemm_skinny_xres_kernel(const h16_t* __restrict__ X, const h16_t* __restrict__ W,
                                                               float* __restrict__ part, int M, int Nw, int K,
                                                               int plane_rows) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int XROWS = 32 * MB;              // hi rows of 16 MB batch rows, then their lo rows
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, t = lane & 15, g = lane >> 4;
  const int j = blockIdx.x, G = gridDim.x, s = blockIdx.y;
  const int T = Nw >> 7;                      // 128-row weight tiles
  const int ntiles = j < T ? (T - 1 - j) / G + 1 : 0;
  const int F = 4 * ntiles;                   // k-steps of this workgroup, tile after tile
  const int nsteps = K >> 7;

  // weight fragment of flattened step f: tile j + (f / 4) G, 16-row block w of it, k-step 4 s + f % 4
  const h16_t* wlane = W + (size_t)(t * 32 + g * 8);
  auto w_off = [&](int f) -> size_t {
    f = min(f, F - 1);
    return wtile_offset(((j + (f >> 2) * G) * 8 + w) * 16, (4 * s + (f & 3)) * 128, K, Nw);
  };
  // two slots, loads one k-step ahead (three ahead measured slower: 27.8 against 26.0 us on the 7B QKV shape; none at
  // all 27.2 us)
  struct Slot { uint4 w[4]; };
  Slot r0, r1;
#define XRES_LOAD(S, FI)                                                                              \
  {                                                                                                   \
    const h16_t* p_ = wlane + w_off(FI);                                                              \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) S.w[kk] = *(const uint4*)(p_ + kk * 512);        \
  }
  if (F > 0) XRES_LOAD(r0, 0)
  // stage the slice: XROWS rows of 64 chunks (16 bytes each); rows beyond M repeat row M - 1 (never stored)
  {
    constexpr int NCH = XROWS * 64, PER = NCH / 512;
    uint4 v[PER];
#pragma unroll
    for (int it = 0; it < PER; ++it) {
      const int c = it * 512 + tid, r = c >> 6, kc = c & 63;
      const int rb = r % (16 * MB);
      v[it] = *(const uint4*)(X + (size_t)min(rb, M - 1) * 2 * K + (r >= 16 * MB ? K : 0) + (size_t)s * XRES_KS + kc * 8);
    }
#pragma unroll
    for (int it = 0; it < PER; ++it) {
      const int c = it * 512 + tid, r = c >> 6, kc = c & 63;
      *(uint4*)(smem + r * XRES_ROW + kc * 16) = v[it];
    }
  }
  __syncthreads();

  f32x4_t acc[MB];
#pragma unroll
  for (int i = 0; i < MB; ++i) acc[i] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
  const char* xlane = smem + t * XRES_ROW + g * 16;
  // one k-step (ST = 0..3 inside the slice) on slot S
#define XRES_STEP(S, ST)                                                                              \
  {                                                                                                   \
    /* the slice never changes, so its fragments are loop invariant: keep the compiler from hoisting */ \
    /* all of them out of the tile loop into registers it does not have */                            \
    asm volatile("" ::: "memory");                                                                    \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) {                                                \
      uint4 xf[2 * MB];                                                                               \
      _Pragma("unroll") for (int mb = 0; mb < 2 * MB; ++mb)                                           \
          xf[mb] = *(const uint4*)(xlane + mb * 16 * XRES_ROW + (ST) * 256 + kk * 64);                \
      _Pragma("unroll") for (int mb = 0; mb < 2 * MB; ++mb)                                           \
          acc[mb % MB] = mfma_16x16x32(S.w[kk], xf[mb], acc[mb % MB]);                                \
    }                                                                                                 \
  }
  for (int ti = 0; ti < ntiles; ++ti) {
    const int f = 4 * ti;
    XRES_LOAD(r1, f + 1)
    XRES_STEP(r0, 0)
    XRES_LOAD(r0, f + 2)
    XRES_STEP(r1, 1)
    XRES_LOAD(r1, f + 3)
    XRES_STEP(r0, 2)
    XRES_LOAD(r0, f + 4)
    XRES_STEP(r1, 3)
    float* dst = part + (size_t)s * plane_rows * Nw + (size_t)(j + ti * G) * 128 + 16 * w + 4 * g;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int m = mb * 16 + t;
      if (m < M) *(float4*)(dst + (size_t)m * Nw) = make_float4(acc[mb][0], acc[mb][1], acc[mb][2], acc[mb][3]);
      acc[mb] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    }
  }
#undef XRES_STEP
#undef XRES_LOAD
}

int g_num_cu = 256;  // compute units of the device, set by gemm_configure

template <int MB>
hipError_t launch_skinny_xres(hipStream_t s, const void* A, const void* W, float* part, int M, int Nw, int K, int plane_rows,
                              bool configure_only = false) {
  constexpr int SMEM = 32 * MB * XRES_ROW;
  auto kern = gemm_skinny_xres_kernel<MB>;
  if (configure_only) return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
  const int ns = K / XRES_KS, T = Nw / 128;
  const int G = std::max(1, std::min(T, g_num_cu / ns));
  kern<<<dim3(G, ns), 512, SMEM, s>>>((const h16_t*)A, (const h16_t*)W, part, M, Nw, K, plane_rows);
  return hipGetLastError();
}

// the shapes the resident-slice kernel takes (and the split count it implies): at least one weight tile per workgroup.
// Even with a single tile (7B output projection: 32 tiles over 32 workgroups per split) it measures faster than
// gemm_skinny_kernel at 64 rows (11.9 against 13.7 us) and the same below: the slice arrives as one block up front
// instead of sharing the ring, and the k loop has no barrier.
inline bool skinny_xres_ok(int M, int Nw, int K, int nsplit) {
  if (!(M <= 64 && Nw % 128 == 0 && K % XRES_KS == 0 && K / XRES_KS == nsplit && nsplit <= 16)) return false;
  const int T = Nw / 128, G = std::max(1, std::min(T, g_num_cu / nsplit));
  return T >= G;
}

template <int MB, int NW>
hipError_t launch_skinny_nw(hipStream_t s, const void* A, const void* W, float* part, int M, int Nw, int K, int nsplit,
                            int a_dual, int plane_rows, bool configure_only) {
  constexpr int SMEM = 2 * 16 * MB * SK_ROW;
  constexpr int D = 2;   // loads one k-step ahead: measured faster than three ahead (see gemm_skinny_kernel)
  constexpr bool HAS_DUAL = MB <= 8;          // the doubled slice of the largest variant would not fit in LDS
  constexpr bool HAS_SINGLE = 4 * MB >= NW;   // at least one slice chunk per thread
  if (configure_only) {
    hipError_t e;
    if constexpr (HAS_SINGLE) {
      if ((e = hipFuncSetAttribute((const void*)gemm_skinny_kernel<MB, D, false, false, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM)) != hipSuccess) return e;
      if ((e = hipFuncSetAttribute((const void*)gemm_skinny_kernel<MB, D, true, false, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM)) != hipSuccess) return e;
    }
    if constexpr (HAS_DUAL)
      if ((e = hipFuncSetAttribute((const void*)gemm_skinny_kernel<MB, 2, false, true, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * SMEM)) != hipSuccess) return e;
    return hipSuccess;
  }
  const int rows_per_wg = 16 * NW;
  if (nsplit == 0) {  // fused SwiGLU: W = [2F, K], output fp16 [M, F], no split
    if (a_dual) return hipErrorInvalidValue;
    if constexpr (HAS_SINGLE)
      gemm_skinny_kernel<MB, D, true, false, NW><<<dim3(Nw / rows_per_wg, 1), 64 * NW, SMEM, s>>>((const h16_t*)A, (const h16_t*)W, part, M, Nw, K, K / SK, plane_rows);
    else
      return hipErrorInvalidValue;
    return hipGetLastError();
  }
  int steps = K / SK;
  int per = (steps + nsplit - 1) / nsplit;
  if (a_dual) {
    if constexpr (HAS_DUAL)
      gemm_skinny_kernel<MB, 2, false, true, NW><<<dim3(Nw / rows_per_wg, nsplit), 64 * NW, 2 * SMEM, s>>>((const h16_t*)A, (const h16_t*)W, part, M, Nw, K, per, plane_rows);
    else
      return hipErrorInvalidValue;
  } else {
    if constexpr (HAS_SINGLE)
      gemm_skinny_kernel<MB, D, false, false, NW><<<dim3(Nw / rows_per_wg, nsplit), 64 * NW, SMEM, s>>>((const h16_t*)A, (const h16_t*)W, part, M, Nw, K, per, plane_rows);
    else
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// Fused gate/up form (no split, so the grid cannot be tuned by the split count): NW wavefronts of 8 features each per
// workgroup, the last workgroup possibly ragged.
template <int MB, int NW>
hipError_t launch_skinny_glu(hipStream_t s, const void* A, const void* W, void* out, int M, int Nw, int K, bool configure_only) {
  constexpr int SMEM = 2 * 16 * MB * SK_ROW;
  constexpr int D = 2;   // loads one k-step ahead: measured faster than three ahead (see gemm_skinny_kernel)
  auto kern = gemm_skinny_kernel<MB, D, true, false, NW>;
  if (configure_only) return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
  const int F = Nw / 2;
  kern<<<dim3((F + 8 * NW - 1) / (8 * NW), 1), 64 * NW, SMEM, s>>>((const h16_t*)A, (const h16_t*)W, (float*)out, M, Nw, K, K / SK, M);
  return hipGetLastError();
}

// Workgroup width for the gate/up form: the one of 8, 7, 6 wavefronts that gives the most workgroups without
// exceeding the number of compute units (a function of F only, never of the batch).  Measured at 64 rows:
// 7B (F = 11008) 172 / 197 / 230 workgroups = 41.8 / 38.1 / 37.2 us and 276 workgroups (5 wavefronts) 56.6 us;
// 13B (F = 13824) 216 / 247 workgroups = 51.7 / 49.5 us, 288 workgroups 79.9 us; 70B (448 / 512 workgroups) no difference.
inline int skinny_glu_width(int F) {
  int best = 8, best_wgs = 0;
  for (int nw = 8; nw >= 6; --nw) {
    const int wgs = (F + 8 * nw - 1) / (8 * nw);
    if (wgs <= g_num_cu && wgs > best_wgs) { best = nw; best_wgs = wgs; }
  }
  return best;
}

template <int MB>
hipError_t launch_skinny(hipStream_t s, const void* A, const void* W, float* part, int M, int Nw, int K, int nsplit,
                         int a_dual, int plane_rows, bool configure_only = false) {
  if (configure_only) {
    hipError_t e = launch_skinny_nw<MB, 4>(s, A, W, part, M, Nw, K, nsplit, a_dual, plane_rows, true);
    if (e != hipSuccess) return e;
    if constexpr (MB <= 8) {
      if ((e = launch_skinny_glu<MB, 6>(s, A, W, part, M, Nw, K, true)) != hipSuccess) return e;
      if ((e = launch_skinny_glu<MB, 7>(s, A, W, part, M, Nw, K, true)) != hipSuccess) return e;
      if ((e = launch_skinny_glu<MB, 8>(s, A, W, part, M, Nw, K, true)) != hipSuccess) return e;
    }
    return launch_skinny_nw<MB, 8>(s, A, W, part, M, Nw, K, nsplit, a_dual, plane_rows, true);
  }
  if constexpr (MB <= 8) {
    if (nsplit == 0) {
      if (a_dual || Nw % 16) return hipErrorInvalidValue;
      switch (skinny_glu_width(Nw / 2)) {
        case 6: return launch_skinny_glu<MB, 6>(s, A, W, part, M, Nw, K, false);
        case 7: return launch_skinny_glu<MB, 7>(s, A, W, part, M, Nw, K, false);
        default: return launch_skinny_glu<MB, 8>(s, A, W, part, M, Nw, K, false);
      }
    }
  }
  // eight wavefronts (128 rows of W per workgroup) when the shape allows: half the activation-slice traffic
  const bool wide = Nw % 128 == 0 && (a_dual ? true : 4 * MB >= 8) && MB <= 8;
  return wide ? launch_skinny_nw<MB, 8>(s, A, W, part, M, Nw, K, nsplit, a_dual, plane_rows, false)
              : launch_skinny_nw<MB, 4>(s, A, W, part, M, Nw, K, nsplit, a_dual, plane_rows, false);
}

// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ W,
                                                       float* __restrict__ out, int M, int N, int K, int accumulate) {
  __shared__ float as[16][17], ws[16][17];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m = blockIdx.y * 16 + ty, n = blockIdx.x * 16 + tx;
  float acc = 0.f;
  for (int k0 = 0; k0 < K; k0 += 16) {
    int am = blockIdx.y * 16 + ty, wn = blockIdx.x * 16 + ty;
    as[ty][tx] = (am < M && k0 + tx < K) ? A[(size_t)am * K + k0 + tx] : 0.f;
    ws[ty][tx] = (wn < N && k0 + tx < K) ? W[(size_t)wn * K + k0 + tx] : 0.f;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) acc += as[ty][k] * ws[tx][k];
    __syncthreads();
  }
  if (m < M && n < N) {
    if (accumulate) out[(size_t)m * N + n] += acc;
    else out[(size_t)m * N + n] = acc;
  }
}

}  // namespace

hipError_t launch_gemm_h16(hipStream_t s, const void* A, const void* W, void* out, int M, int N, int K, int epi,
                           int a_dual) {
  if (M <= 0) return hipSuccess;
  if (K % 128) return hipErrorInvalidValue;   // W comes in 128-column tiles
  if (epi == EPI_SWIGLU ? (N % 128) : (N % 256)) return hipErrorInvalidValue;
  // the kernel addresses both operands with 32-bit byte offsets
  if ((size_t)M * (a_dual ? 2 : 1) * K * 2 >= ((size_t)1 << 32) || (size_t)N * (epi == EPI_SWIGLU ? 2 : 1) * K * 2 >= ((size_t)1 << 32))
    return hipErrorInvalidValue;
  switch (epi) {
    case EPI_STORE_F32: return launch_large_dma<EPI_STORE_F32>(s, A, W, out, M, N, K, a_dual);
    case EPI_RESID_F32: return launch_large_dma<EPI_RESID_F32>(s, A, W, out, M, N, K, a_dual);
    case EPI_SWIGLU: return launch_large_dma<EPI_SWIGLU>(s, A, W, out, M, N, K, a_dual);
    case EPI_STORE_ACT: return launch_large_dma<EPI_STORE_ACT>(s, A, W, out, M, N, K, a_dual);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_gemm_h16_lo4(hipStream_t s, const void* A, const void* W, const void* W4, const void* w_scale,
                               const void* a_scale, int scale_groups, void* out, int M, int N, int K, int epi, const RopeEpi* re) {
  if (M <= 0) return hipSuccess;
  if (epi == EPI_QKV_ROPE) {
    if (!re || re->Hq < 1 || re->Hkv < 1 || N != (re->Hq + 2 * re->Hkv) * KV_HEAD_DIM) return hipErrorInvalidValue;
  } else if (!out) {
    return hipErrorInvalidValue;
  }
  if (!A || !W || !W4 || !w_scale || !a_scale) return hipErrorInvalidValue;
  if (K % 512 || N % 256) return hipErrorInvalidValue;   // (the 4-bit copy of W is tiled as a matrix with K / 4 columns)
  if (scale_groups < 2 * ((M + 255) / 256)) return hipErrorInvalidValue;   // a scale word for every row of every 256-row tile
  if ((size_t)M * 2 * K * 2 >= ((size_t)1 << 32) || (size_t)N * K * 2 >= ((size_t)1 << 32)) return hipErrorInvalidValue;
  const Lo4Args l4{W4, (const unsigned char*)w_scale, (const unsigned char*)a_scale, scale_groups};
  switch (epi) {
    case EPI_STORE_F32: return launch_large_dma_lo4<EPI_STORE_F32>(s, A, W, out, M, N, K, nullptr, &l4);
    case EPI_RESID_F32: return launch_large_dma_lo4<EPI_RESID_F32>(s, A, W, out, M, N, K, nullptr, &l4);
    case EPI_QKV_ROPE: return launch_large_dma_lo4<EPI_QKV_ROPE>(s, A, W, nullptr, M, N, K, re, &l4);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_gemm_h16_qkv_rope(hipStream_t s, const void* A, const void* W, int M, int K, const RopeEpi& re) {
  if (M <= 0) return hipSuccess;
  const int N = (re.Hq + 2 * re.Hkv) * KV_HEAD_DIM;
  if (K % 128 || N % 256 || re.Hq < 1 || re.Hkv < 1) return hipErrorInvalidValue;   // (a 256-column tile = two whole heads)
  if ((size_t)M * 2 * K * 2 >= ((size_t)1 << 32) || (size_t)N * K * 2 >= ((size_t)1 << 32)) return hipErrorInvalidValue;
  return launch_large_dma_qkv_rope(s, A, W, M, N, K, &re);
}

int gemm_tiled_pick_split(int M, int N, int K, int max_splits, int lo4) {
  // as many splits as it takes to give every compute unit one workgroup, none of them empty
  const int tiles = ((M + 255) / 256) * (N / 256), nkw = K / 32;
  int want = std::max(1, std::min(g_num_cu / std::max(tiles, 1), max_splits));
  want = std::min(want, nkw);
  int per = (nkw + want - 1) / want;
  if (lo4) per = (per + 3) & ~3;   // (the 4-bit low-half stages cover four k-tiles each)
  return (nkw + per - 1) / per;
}

hipError_t launch_gemm_h16_splitk_lo4(hipStream_t s, const void* A, const void* W, const void* W4, const void* w_scale,
                                      const void* a_scale, int scale_groups, float* part, int M, int N, int K, int nsplit,
                                      int plane_rows) {
  if (M <= 0) return hipSuccess;
  if (plane_rows <= 0) plane_rows = M;
  if (!A || !W || !W4 || !w_scale || !a_scale || !part) return hipErrorInvalidValue;
  if (K % 512 || N % 256 || nsplit < 1 || plane_rows < M) return hipErrorInvalidValue;
  if (scale_groups < 2 * ((M + 255) / 256)) return hipErrorInvalidValue;
  const int nkw = K / 32, per = ((nkw + nsplit - 1) / nsplit + 3) & ~3;
  if ((nkw + per - 1) / per != nsplit) return hipErrorInvalidValue;   // a split would be empty
  if ((size_t)M * 2 * K * 2 >= ((size_t)1 << 32) || (size_t)N * K * 2 >= ((size_t)1 << 32)) return hipErrorInvalidValue;
  const Lo4Args l4{W4, (const unsigned char*)w_scale, (const unsigned char*)a_scale, scale_groups};
  return launch_large_dma_split_lo4(s, A, W, part, M, N, K, nsplit, plane_rows, &l4);
}

hipError_t launch_gemm_h16_splitk(hipStream_t s, const void* A, const void* W, float* part, int M, int N, int K, int a_dual,
                                  int nsplit, int plane_rows) {
  if (M <= 0) return hipSuccess;
  if (plane_rows <= 0) plane_rows = M;
  if (K % 128 || N % 256 || nsplit < 1 || plane_rows < M) return hipErrorInvalidValue;
  const int nkw = K / 32, per = (nkw + nsplit - 1) / nsplit;
  if ((nkw + per - 1) / per != nsplit) return hipErrorInvalidValue;   // a split would be empty
  if ((size_t)M * (a_dual ? 2 : 1) * K * 2 >= ((size_t)1 << 32) || (size_t)N * K * 2 >= ((size_t)1 << 32)) return hipErrorInvalidValue;
  return launch_large_dma_split(s, A, W, part, M, N, K, a_dual, nsplit, plane_rows);
}

// Raise the dynamic-LDS limit of every instantiation once per device (must not happen inside a stream capture).
hipError_t gemm_configure() {
  hipError_t e;
  if ((e = launch_large_dma<EPI_STORE_F32>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_large_dma<EPI_RESID_F32>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_large_dma<EPI_SWIGLU>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_large_dma<EPI_STORE_ACT>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_large_dma_split(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, 1, 0, true)) != hipSuccess) return e;
  if ((e = launch_large_dma_qkv_rope(nullptr, nullptr, nullptr, 0, 0, 0, nullptr, true)) != hipSuccess) return e;
  if ((e = launch_large_dma_lo4<EPI_STORE_F32>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, nullptr, nullptr, true)) != hipSuccess) return e;
  if ((e = launch_large_dma_lo4<EPI_RESID_F32>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, nullptr, nullptr, true)) != hipSuccess) return e;
  if ((e = launch_large_dma_lo4<EPI_QKV_ROPE>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, nullptr, nullptr, true)) != hipSuccess) return e;
  if ((e = launch_large_dma_split_lo4(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, 0, nullptr, true)) != hipSuccess) return e;
  {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
      g_num_cu = prop.multiProcessorCount;
  }
  if ((e = launch_skinny_xres<1>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny_xres<2>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny_xres<4>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny<1>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny<2>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny<4>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny<8>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny<16>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, 0, 0, true)) != hipSuccess) return e;
  return hipSuccess;
}

int gemm_skinny_pick_split(int M, int Nw, int K, int a_dual) {
  // The split is a function of the weight shape alone: the same for every batch size, so that an output element is
  // accumulated in the same order whether its row arrives in a whole batch or in a micro-batch.
  (void)M;
  const int tiles = Nw % 128 == 0 ? Nw / 128 : Nw / 64, steps = K / SK;
  // pair-input projections: the split of the resident-slice kernel (512 columns per split) where its workgroups
  // come out even, i.e. the tiles divide over the num_cu / splits workgroups of a split (7B QKV: 96 tiles over 32,
  // output projection 32 over 32).
  // Measured on the 13B and 70B shapes, where they do not, the ring kernel with fewer splits is 6-16 % faster.
  if (a_dual && Nw % 128 == 0 && K % XRES_KS == 0) {
    const int ns = K / XRES_KS;
    if (ns <= 10 && g_num_cu % ns == 0) {
      const int G = g_num_cu / ns;
      if (tiles >= G && tiles % G == 0) return ns;
    }
  }
  // Otherwise as many splits as give every compute unit at most one workgroup: measured over the 7B, 13B and 70B
  // shapes the fastest split is the one whose tiles x splits comes closest to the number of compute units from
  // below (13B down projection, 40 tiles: 6 splits 24 us, 8 splits 33 us; 70B down, 64 tiles: 4 splits 72 us, 8 splits
  // 80 us), because a second workgroup on some compute units makes those finish last.
  int want = std::max(1, std::min(8, g_num_cu / std::max(tiles, 1)));   // (the consumers take up to eight planes at full speed)
  if (want > steps) want = steps;
  if (want < 1) want = 1;
  const int per = (steps + want - 1) / want;
  return (steps + per - 1) / per;  // no empty split
}

hipError_t launch_gemm_skinny_h16(hipStream_t s, const void* A, const void* W, float* part, int M, int Nw, int K,
                                  int nsplit, int a_dual, int plane_rows) {
  if (M <= 0) return hipSuccess;
  if (plane_rows <= 0) plane_rows = M;
  if (K % SK || Nw % 64 || M > 256 || nsplit < 0 || plane_rows < M) return hipErrorInvalidValue;
  if (a_dual && skinny_xres_ok(M, Nw, K, nsplit)) {
    if (M <= 16) return launch_skinny_xres<1>(s, A, W, part, M, Nw, K, plane_rows);
    if (M <= 32) return launch_skinny_xres<2>(s, A, W, part, M, Nw, K, plane_rows);
    return launch_skinny_xres<4>(s, A, W, part, M, Nw, K, plane_rows);
  }
  if (M <= 16) return launch_skinny<1>(s, A, W, part, M, Nw, K, nsplit, a_dual, plane_rows);
  if (M <= 32) return launch_skinny<2>(s, A, W, part, M, Nw, K, nsplit, a_dual, plane_rows);
  if (M <= 64) return launch_skinny<4>(s, A, W, part, M, Nw, K, nsplit, a_dual, plane_rows);
  if (M <= 128) return launch_skinny<8>(s, A, W, part, M, Nw, K, nsplit, a_dual, plane_rows);
  return launch_skinny<16>(s, A, W, part, M, Nw, K, nsplit, a_dual, plane_rows);
}

hipError_t launch_gemm_f32(hipStream_t s, const float* A, const float* W, float* out, int M, int N, int K,
                           int accumulate) {
  if (M <= 0) return hipSuccess;
  dim3 grid((N + 15) / 16, (M + 15) / 16);
  gemm_f32_kernel<<<grid, 256, 0, s>>>(A, W, out, M, N, K, accumulate);
  return hipGetLastError();
}
