// GEMMs of the rollout, out = A[M,K] * W[N,K]^T with both operands K-contiguous.
//   gemm_h16_dma_kernel : large-tile fp16 MFMA GEMM for prefill (M = thousands of tokens): 256x256x64 block tile,
//                         8 wavefronts of 128x64, LDS double buffer filled by LDS-DMA loads, 32x32x16 MFMA.
//   gemm_skinny_kernel  : weight-streaming GEMM for decode (M = batch <= 256): W is the MFMA row operand read
//                         straight from HBM into registers exactly once, the activation slice is staged in LDS,
//                         split-K partial sums go to a workspace that the consumer kernel adds up in a fixed order.
//   gemm_f32_kernel     : plain-ALU fp32 GEMM for the small fp32 configuration.
#include <stdlib.h>

#include "common.h"
#include "kernels.h"

namespace {

// ---------------------------------------------------------------------------------------------------
// Large-tile GEMM: the operand tiles go from global memory straight into LDS (LDS-DMA loads, no staging
// registers), 256x256x64 block tile, two LDS stages of 64 KB, 8 wavefronts of 128x64, 32x32x16 MFMA.
//   * A wavefront-wide DMA load writes lane i's 16 bytes to LDS base + 16 i, so one instruction fills eight
//     128-byte tile rows.  To keep the later 16-byte MFMA operand reads free of bank conflicts (64 banks: sixteen
//     lanes, i.e. sixteen consecutive rows, are served per cycle and must cover 256 distinct bytes) the 16-byte
//     chunk c of row r is stored at slot c ^ ((r >> 1) & 7); the permutation is applied on the global side (each
//     lane fetches the chunk that belongs in its slot), so global reads stay whole 128-byte rows.
//   * The compiler would wait for every outstanding DMA load before any LDS read it knows about, which would
//     serialise the pipeline, so the operand reads are issued as inline ds_read_b128 and their completion is
//     awaited explicitly (s_waitcnt lgkmcnt), two k-steps of fragments in flight.
constexpr int DMA_STAGE = 65536;

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
#define LDS_WAIT6(N, f0, f1, f2, f3, f4, f5) \
  asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(f0), "+v"(f1), "+v"(f2), "+v"(f3), "+v"(f4), "+v"(f5))

template <int EPI>
__global__ __launch_bounds__(512) void gemm_h16_dma_kernel(const h16_t* __restrict__ A, const h16_t* __restrict__ W,
                                                            void* __restrict__ out, int M, int N, int K, int tilesM,
                                                            int tilesN, int a_dual) {
  // a_dual: A rows are [hi (K) | lo (K)]; the k loop then runs over 2K columns of A against W's K columns twice.
  constexpr int BM = 256, BN = 256, WN = 64;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int pid = blockIdx.x;
  const int total = tilesM * tilesN;
  if ((total & 7) == 0) pid = (pid & 7) * (total >> 3) + (pid >> 3);
  const int band = 8 * tilesN;
  const int first_m = (pid / band) * 8;
  const int gsz = min(tilesM - first_m, 8);
  const int tm = first_m + (pid % band) % gsz;
  const int tn = (pid % band) / gsz;
  const int m0 = tm * BM;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;

  auto wrow = [&](int r) -> int {
    if (EPI == EPI_SWIGLU) {
      int wv = r / WN, qd = r % WN;
      int half = qd / (WN / 2), j = qd % (WN / 2);
      return half * N + tn * (BN / 2) + wv * (WN / 2) + j;
    }
    return tn * BN + r;
  };

  // DMA sources: wavefronts 0-3 bring the A tile (32 row groups of 8), 4-7 the W tile
  const bool loads_a = wave < 4;
  const char* gbase = loads_a ? (const char*)A : (const char*)W;
  uint32_t go[8];
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    int row = 8 * ((wave & 3) * 8 + it) + (lane >> 3);
    int grow = loads_a ? min(m0 + row, M - 1) : wrow(row);
    go[it] = (uint32_t)grow * (uint32_t)(loads_a && a_dual ? 2 * K : K) * 2u + (uint32_t)(((lane & 7) ^ ((row >> 1) & 7)) * 16);
  }
  const int nkw = K / 64;                       // k-tiles of W
  const int nk = a_dual ? 2 * nkw : nkw;        // k-tiles of the product
  typedef __attribute__((address_space(3))) void lds_void;
  typedef const __attribute__((address_space(1))) void g_void;
  char* dma_dst = smem + wave * 8192;  // + stage * DMA_STAGE + it * 1024
#define DMA_ISSUE(KT, STAGE)                                                                              \
  {                                                                                                       \
    const char* src = gbase + (size_t)(loads_a ? (KT) : ((KT) >= nkw ? (KT) - nkw : (KT))) * 128;        \
    _Pragma("unroll") for (int it = 0; it < 8; ++it)                                                      \
        __builtin_amdgcn_global_load_lds((g_void*)(src + go[it]),                                         \
                                         (lds_void*)(dma_dst + (STAGE) * DMA_STAGE + it * 1024), 16, 0, 0); \
  }

  f32x16_t acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // operand read addresses: row (lane & 31) of a 32-row block, chunk 2 ks + (lane >> 5), stored at slot chunk ^ ((row >> 1) & 7)
  const uint32_t lds0 = (uint32_t)(size_t)smem;
  const uint32_t y = (uint32_t)((lane >> 5) ^ ((lane >> 1) & 7));
  uint32_t a_rd[4], b_rd[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    uint32_t slot = (uint32_t)(2 * ks) ^ y;
    a_rd[ks] = lds0 + (uint32_t)((wm * 128 + (lane & 31)) * 128) + slot * 16;
    b_rd[ks] = lds0 + (uint32_t)((BM + wn * 64 + (lane & 31)) * 128) + slot * 16;
  }

  DMA_ISSUE(0, 0)
  for (int kt = 0; kt < nk; ++kt) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (kt + 1 < nk) DMA_ISSUE(kt + 1, (kt + 1) & 1)
    const uint32_t so = (uint32_t)(kt & 1) * DMA_STAGE;
    u32x4_t p0, p1, p2, p3, p4, p5, q0, q1, q2, q3, q4, q5;
#define RD(S0, S1, S2, S3, S4, S5, KS)                                                      \
    S0 = lds_read128<0>(a_rd[KS] + so); S1 = lds_read128<4096>(a_rd[KS] + so);              \
    S2 = lds_read128<8192>(a_rd[KS] + so); S3 = lds_read128<12288>(a_rd[KS] + so);          \
    S4 = lds_read128<0>(b_rd[KS] + so); S5 = lds_read128<4096>(b_rd[KS] + so);
#define MM(S0, S1, S2, S3, S4, S5)                                                          \
    acc[0][0] = mfma_32x32x16_v(S0, S4, acc[0][0]); acc[0][1] = mfma_32x32x16_v(S0, S5, acc[0][1]); \
    acc[1][0] = mfma_32x32x16_v(S1, S4, acc[1][0]); acc[1][1] = mfma_32x32x16_v(S1, S5, acc[1][1]); \
    acc[2][0] = mfma_32x32x16_v(S2, S4, acc[2][0]); acc[2][1] = mfma_32x32x16_v(S2, S5, acc[2][1]); \
    acc[3][0] = mfma_32x32x16_v(S3, S4, acc[3][0]); acc[3][1] = mfma_32x32x16_v(S3, S5, acc[3][1]);
    RD(p0, p1, p2, p3, p4, p5, 0)
    RD(q0, q1, q2, q3, q4, q5, 1)
    LDS_WAIT6(6, p0, p1, p2, p3, p4, p5);
    MM(p0, p1, p2, p3, p4, p5)
    RD(p0, p1, p2, p3, p4, p5, 2)
    LDS_WAIT6(6, q0, q1, q2, q3, q4, q5);
    MM(q0, q1, q2, q3, q4, q5)
    RD(q0, q1, q2, q3, q4, q5, 3)
    LDS_WAIT6(6, p0, p1, p2, p3, p4, p5);
    MM(p0, p1, p2, p3, p4, p5)
    LDS_WAIT6(0, q0, q1, q2, q3, q4, q5);
    MM(q0, q1, q2, q3, q4, q5)
#undef RD
#undef MM
  }
#undef DMA_ISSUE

#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int m = m0 + wm * 128 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
      if (m >= M) continue;
      if (EPI == EPI_SWIGLU) {
        int f = tn * (BN / 2) + wn * (WN / 2) + (lane & 31);
        float gte = acc[i][0][e], up = acc[i][1][e];
        float v = gte / (1.f + __expf(-gte)) * up;
        ((h16_t*)out)[(size_t)m * N + f] = f32_to_h16(v);
      } else {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          int n = tn * BN + wn * WN + j * 32 + (lane & 31);
          float v = acc[i][j][e];
          if (EPI == EPI_STORE_F32) ((float*)out)[(size_t)m * N + n] = v;
          if (EPI == EPI_RESID_F32) ((float*)out)[(size_t)m * N + n] += v;
          if (EPI == EPI_STORE_ACT) ((h16_t*)out)[(size_t)m * N + n] = f32_to_h16(v);
        }
      }
    }
  }
}

template <int EPI>
hipError_t launch_large_dma(hipStream_t s, const void* A, const void* W, void* out, int M, int N, int K, int a_dual,
                            bool configure_only = false) {
  constexpr int SMEM = 2 * DMA_STAGE;
  auto kern = gemm_h16_dma_kernel<EPI>;
  if (configure_only) return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
  int tilesM = (M + 255) / 256;
  int tilesN = (EPI == EPI_SWIGLU) ? N / 128 : N / 256;
  kern<<<tilesM * tilesN, 512, SMEM, s>>>((const h16_t*)A, (const h16_t*)W, out, M, N, K, tilesM, tilesN, a_dual);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
constexpr int SK = 128;                 // k extent of one staged activation slice
constexpr int SK_ROW = SK * 2 + 16;     // bytes per LDS row (padded)

// grid (Nw / (16 NW), nsplit), 64 NW threads; wavefront w owns W rows n0 + 16 w .. +16 and all M (<= 16 MB) columns.
// Measured on MI355X the kernel's time follows (weight bytes + activation-slice bytes requested from L2) / ~6.5 TB/s,
// so the slice re-reads matter as much as the weights: eight wavefronts per workgroup (128 rows of W) halve them.
// Loads run D - 1 k-steps ahead of the MFMAs through a register ring (weights and the activation slice alike:
// the memory counter retires in order, so both must share one prefetch distance); the activation slice then
// passes through a double-buffered LDS tile that the four wavefronts share.
template <int MB, int D, bool GLU, bool DUAL, int NW>
__global__ __launch_bounds__(64 * NW) void gemm_skinny_kernel(const h16_t* __restrict__ X, const h16_t* __restrict__ W,
                                                          float* __restrict__ part, int M, int Nw, int K,
                                                          int steps_per_split) {
  static_assert(D == 2 || D == 4, "ring depth 2 or 4");
  // DUAL: X rows are [hi (K) | lo (K)] fp16 pairs; the LDS tile holds the hi rows followed by the lo rows and every
  // weight fragment is multiplied with both.
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int XR = DUAL ? 2 * MB : MB;   // 16-row blocks of the staged slice
  constexpr int XBYTES = 16 * XR * SK_ROW;
  constexpr int NT = 64 * NW;
  constexpr int XL = 256 * XR / NT;        // 16-byte chunks of the slice each thread moves per k-step
  static_assert(XL * NT == 256 * XR, "slice chunks must divide evenly over the threads");
  const int ldx = DUAL ? 2 * K : K;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, t = lane & 15, g = lane >> 4;
  // GLU: W = [gate rows | up rows] of F = Nw / 2 features each; the workgroup owns 32 features, each wavefront
  // 8 of them with the gate rows in MFMA rows 0..7 and the matching up rows in 8..15.
  const int n0 = GLU ? blockIdx.x * (8 * NW) : blockIdx.x * (16 * NW);
  const int nsteps_total = K / SK;
  const int s0 = blockIdx.y * steps_per_split;
  const int s1 = min(nsteps_total, s0 + steps_per_split);

  f32x4_t acc[MB];
#pragma unroll
  for (int i = 0; i < MB; ++i) acc[i] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

  const int wrow = GLU ? ((t < 8) ? n0 + 8 * w + t : (Nw >> 1) + n0 + 8 * w + (t - 8)) : n0 + 16 * w + t;
  const h16_t* wp = W + (size_t)wrow * K + 8 * g;
  // Activation slice: 16 MB rows x 16 chunks of 16 B per k-step, MB chunks per thread.  Rows beyond M are read
  // from row M - 1 instead: they only feed output columns that are never stored.
  const h16_t* xp[XL];
  int xo[XL];
#pragma unroll
  for (int it = 0; it < XL; ++it) {
    int c = it * NT + tid, r = c >> 4, kc = c & 15;   // r in [0, 16 XR): rows >= 16 MB are the lo parts
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
  const int rot = nst > 0 ? (int)((grp * 5u + blockIdx.y * 3u) % (unsigned)nst) : 0;
  (void)NT;
  // Loads are issued without any branch around them (a step index past the end re-reads the last step, which
  // hits in cache): with straight-line code the compiler can keep D - 1 steps of loads in flight and wait only
  // for the oldest.
  auto step_off = [&](int i) -> size_t {
    int r = min(i, nst - 1) + rot;
    if (r >= nst) r -= nst;
    return (size_t)(s0 + r) * SK;
  };
  // Ring of D named slots (separate variables, so that they live in registers).
  struct Slot { uint4 w[4]; uint4 x[XL]; };
  Slot r0, r1, r2, r3;
#define SKINNY_LOAD(S, I)                                                                                \
  {                                                                                                      \
    const size_t ko = step_off(I);                                                                       \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) S.w[kk] = *(const uint4*)(wp + ko + kk * 32);       \
    _Pragma("unroll") for (int it = 0; it < XL; ++it) S.x[it] = *(const uint4*)(xp[it] + ko);            \
  }
  // one k-step on slot S (LDS buffer PAR)
#define SKINNY_STEP(S, PAR)                                                                              \
  {                                                                                                      \
    char* buf = smem + (PAR) * XBYTES;                                                                   \
    _Pragma("unroll") for (int it = 0; it < XL; ++it) *(uint4*)(buf + xo[it]) = S.x[it];                 \
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
  float* dst = part + (size_t)blockIdx.y * M * Nw;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    int m = mb * 16 + t;
    if (m < M) *(float4*)(dst + (size_t)m * Nw + n0 + 16 * w + 4 * g) = make_float4(acc[mb][0], acc[mb][1], acc[mb][2], acc[mb][3]);
  }
}

inline bool skinny_force_narrow() {
  static const bool v = getenv("RLHF_SKINNY_NARROW") && atoi(getenv("RLHF_SKINNY_NARROW"));
  return v;
}

template <int MB, int NW>
hipError_t launch_skinny_nw(hipStream_t s, const void* A, const void* W, float* part, int M, int Nw, int K, int nsplit,
                            int a_dual, bool configure_only) {
  constexpr int SMEM = 2 * 16 * MB * SK_ROW;
  constexpr int D = MB <= 4 ? 4 : 2;
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
      gemm_skinny_kernel<MB, D, true, false, NW><<<dim3(Nw / rows_per_wg, 1), 64 * NW, SMEM, s>>>((const h16_t*)A, (const h16_t*)W, part, M, Nw, K, K / SK);
    else
      return hipErrorInvalidValue;
    return hipGetLastError();
  }
  int steps = K / SK;
  int per = (steps + nsplit - 1) / nsplit;
  if (a_dual) {
    if constexpr (HAS_DUAL)
      gemm_skinny_kernel<MB, 2, false, true, NW><<<dim3(Nw / rows_per_wg, nsplit), 64 * NW, 2 * SMEM, s>>>((const h16_t*)A, (const h16_t*)W, part, M, Nw, K, per);
    else
      return hipErrorInvalidValue;
  } else {
    if constexpr (HAS_SINGLE)
      gemm_skinny_kernel<MB, D, false, false, NW><<<dim3(Nw / rows_per_wg, nsplit), 64 * NW, SMEM, s>>>((const h16_t*)A, (const h16_t*)W, part, M, Nw, K, per);
    else
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int MB>
hipError_t launch_skinny(hipStream_t s, const void* A, const void* W, float* part, int M, int Nw, int K, int nsplit,
                         int a_dual, bool configure_only = false) {
  if (configure_only) {
    hipError_t e = launch_skinny_nw<MB, 4>(s, A, W, part, M, Nw, K, nsplit, a_dual, true);
    if (e != hipSuccess) return e;
    return launch_skinny_nw<MB, 8>(s, A, W, part, M, Nw, K, nsplit, a_dual, true);
  }
  // eight wavefronts (128 rows of W per workgroup) when the shape allows: half the activation-slice traffic
  const bool wide = Nw % 128 == 0 && (a_dual ? true : 4 * MB >= 8) && MB <= 8 && !skinny_force_narrow();
  return wide ? launch_skinny_nw<MB, 8>(s, A, W, part, M, Nw, K, nsplit, a_dual, false)
              : launch_skinny_nw<MB, 4>(s, A, W, part, M, Nw, K, nsplit, a_dual, false);
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
  if (K % 64) return hipErrorInvalidValue;
  if (epi == EPI_SWIGLU ? (N % 128) : (N % 256)) return hipErrorInvalidValue;
  switch (epi) {
    case EPI_STORE_F32: return launch_large_dma<EPI_STORE_F32>(s, A, W, out, M, N, K, a_dual);
    case EPI_RESID_F32: return launch_large_dma<EPI_RESID_F32>(s, A, W, out, M, N, K, a_dual);
    case EPI_SWIGLU: return launch_large_dma<EPI_SWIGLU>(s, A, W, out, M, N, K, a_dual);
    case EPI_STORE_ACT: return launch_large_dma<EPI_STORE_ACT>(s, A, W, out, M, N, K, a_dual);
  }
  return hipErrorInvalidValue;
}

// Raise the dynamic-LDS limit of every instantiation once per device (must not happen inside a stream capture).
hipError_t gemm_configure() {
  hipError_t e;
  if ((e = launch_large_dma<EPI_STORE_F32>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_large_dma<EPI_RESID_F32>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_large_dma<EPI_SWIGLU>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_large_dma<EPI_STORE_ACT>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny<1>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny<2>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny<4>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny<8>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny<16>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, 0, true)) != hipSuccess) return e;
  return hipSuccess;
}

int gemm_skinny_pick_split(int M, int Nw, int K) {
  (void)M;
  int tiles = (Nw % 128 == 0 && !skinny_force_narrow()) ? Nw / 128 : Nw / 64, steps = K / SK;
  int want = (768 + tiles - 1) / tiles;
  if (want > 8) want = 8;
  if (want > steps) want = steps;
  if (want < 1) want = 1;
  int per = (steps + want - 1) / want;
  return (steps + per - 1) / per;  // no empty split
}

hipError_t launch_gemm_skinny_h16(hipStream_t s, const void* A, const void* W, float* part, int M, int Nw, int K,
                                  int nsplit, int a_dual) {
  if (M <= 0) return hipSuccess;
  if (K % SK || Nw % 64 || M > 256 || nsplit < 0) return hipErrorInvalidValue;
  if (M <= 16) return launch_skinny<1>(s, A, W, part, M, Nw, K, nsplit, a_dual);
  if (M <= 32) return launch_skinny<2>(s, A, W, part, M, Nw, K, nsplit, a_dual);
  if (M <= 64) return launch_skinny<4>(s, A, W, part, M, Nw, K, nsplit, a_dual);
  if (M <= 128) return launch_skinny<8>(s, A, W, part, M, Nw, K, nsplit, a_dual);
  return launch_skinny<16>(s, A, W, part, M, Nw, K, nsplit, a_dual);
}

hipError_t launch_gemm_f32(hipStream_t s, const float* A, const float* W, float* out, int M, int N, int K,
                           int accumulate) {
  if (M <= 0) return hipSuccess;
  dim3 grid((N + 15) / 16, (M + 15) / 16);
  gemm_f32_kernel<<<grid, 256, 0, s>>>(A, W, out, M, N, K, accumulate);
  return hipGetLastError();
}
