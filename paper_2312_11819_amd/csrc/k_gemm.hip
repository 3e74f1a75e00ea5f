// GEMMs of the rollout, out = A[M,K] * W[N,K]^T with both operands K-contiguous.
//   gemm_bf16_kernel    : large-tile bf16 MFMA GEMM for prefill (M = thousands of tokens): 256x256x64 block tile,
//                         8 wavefronts of 128x64, LDS double buffer fed through registers, 32x32x16 MFMA.
//   gemm_skinny_kernel  : weight-streaming GEMM for decode (M = batch <= 256): W is the MFMA row operand read
//                         straight from HBM into registers exactly once, the activation slice is staged in LDS,
//                         split-K partial sums go to a workspace that the consumer kernel adds up in a fixed order.
//   gemm_f32_kernel     : plain-ALU fp32 GEMM for the small fp32 configuration.
#include <stdlib.h>

#include "common.h"
#include "kernels.h"

namespace {

constexpr int BK = 64;            // k extent of one LDS tile
constexpr int LDS_ROW = BK * 2 + 16;  // bytes per tile row; the 16 B pad spreads 16 B reads over all banks

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_bf16_kernel(const bf16_t* __restrict__ A,
                                                                               const bf16_t* __restrict__ W,
                                                                               void* __restrict__ out, int M, int N,
                                                                               int K, int tilesM, int tilesN) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr int WAVES_N = BN / WN;
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int A_IT = BM * 8 / NT, B_IT = BN * 8 / NT;
  constexpr int TILE_BYTES = (BM + BN) * LDS_ROW;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  // workgroup -> tile: consecutive ids on one XCD (ids are dealt round-robin to 8 XCDs) walk a band of 8 row
  // tiles column by column, so the W tile and the 8 A tiles in flight stay in that XCD's L2.
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
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  // global row of W for LDS B-tile row r
  auto wrow = [&](int r) -> int {
    if (EPI == EPI_SWIGLU) {
      int wv = r / WN, qd = r % WN;
      int half = qd / (WN / 2), j = qd % (WN / 2);
      return half * N + tn * (BN / 2) + wv * (WN / 2) + j;  // N = F here
    }
    return tn * BN + r;
  };

  const bf16_t* a_ptr[A_IT];
  const bf16_t* b_ptr[B_IT];
  int a_off[A_IT], b_off[B_IT];
#pragma unroll
  for (int it = 0; it < A_IT; ++it) {
    int c = it * NT + tid, r = c >> 3, kc = c & 7;
    int gr = min(m0 + r, M - 1);
    a_ptr[it] = A + (size_t)gr * K + kc * 8;
    a_off[it] = r * LDS_ROW + kc * 16;
  }
#pragma unroll
  for (int it = 0; it < B_IT; ++it) {
    int c = it * NT + tid, r = c >> 3, kc = c & 7;
    b_ptr[it] = W + (size_t)wrow(r) * K + kc * 8;
    b_off[it] = BM * LDS_ROW + r * LDS_ROW + kc * 16;
  }

  f32x16_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  uint4 ra[A_IT], rb[B_IT];
  const int nk = K / BK;
#pragma unroll
  for (int it = 0; it < A_IT; ++it) ra[it] = *(const uint4*)(a_ptr[it]);
#pragma unroll
  for (int it = 0; it < B_IT; ++it) rb[it] = *(const uint4*)(b_ptr[it]);
#pragma unroll
  for (int it = 0; it < A_IT; ++it) *(uint4*)(smem + a_off[it]) = ra[it];
#pragma unroll
  for (int it = 0; it < B_IT; ++it) *(uint4*)(smem + b_off[it]) = rb[it];
  __syncthreads();

  const int a_frag = (wm * WM + (lane & 31)) * LDS_ROW + (lane >> 5) * 16;
  const int b_frag = BM * LDS_ROW + (wn * WN + (lane & 31)) * LDS_ROW + (lane >> 5) * 16;

  for (int kt = 0; kt < nk; ++kt) {
    const char* cur = smem + (kt & 1) * TILE_BYTES;
    char* nxt = smem + ((kt + 1) & 1) * TILE_BYTES;
    if (kt + 1 < nk) {
#pragma unroll
      for (int it = 0; it < A_IT; ++it) ra[it] = *(const uint4*)(a_ptr[it] + (size_t)(kt + 1) * BK);
#pragma unroll
      for (int it = 0; it < B_IT; ++it) rb[it] = *(const uint4*)(b_ptr[it] + (size_t)(kt + 1) * BK);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      uint4 af[MI], bfr[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i) af[i] = *(const uint4*)(cur + a_frag + i * 32 * LDS_ROW + ks * 32);
#pragma unroll
      for (int j = 0; j < NI; ++j) bfr[j] = *(const uint4*)(cur + b_frag + j * 32 * LDS_ROW + ks * 32);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = mfma_32x32x16(af[i], bfr[j], acc[i][j]);
    }
    if (kt + 1 < nk) {
#pragma unroll
      for (int it = 0; it < A_IT; ++it) *(uint4*)(nxt + a_off[it]) = ra[it];
#pragma unroll
      for (int it = 0; it < B_IT; ++it) *(uint4*)(nxt + b_off[it]) = rb[it];
    }
    __syncthreads();
  }

  // epilogue: lane holds column (lane & 31) and rows 8 (e >> 2) + 4 (lane >> 5) + (e & 3) of each 32x32 tile
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      int m = m0 + wm * WM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
      if (m >= M) continue;
      if (EPI == EPI_SWIGLU) {
#pragma unroll
        for (int j = 0; j < NI / 2; ++j) {
          int f = tn * (BN / 2) + wn * (WN / 2) + j * 32 + (lane & 31);
          float gte = acc[i][j][e], up = acc[i][j + NI / 2][e];
          float v = gte / (1.f + __expf(-gte)) * up;
          ((bf16_t*)out)[(size_t)m * N + f] = f32_to_bf16(v);
        }
      } else {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
          int n = tn * BN + wn * WN + j * 32 + (lane & 31);
          float v = acc[i][j][e];
          if (EPI == EPI_STORE_F32) ((float*)out)[(size_t)m * N + n] = v;
          if (EPI == EPI_RESID_F32) ((float*)out)[(size_t)m * N + n] += v;
          if (EPI == EPI_STORE_ACT) ((bf16_t*)out)[(size_t)m * N + n] = f32_to_bf16(v);
        }
      }
    }
  }
}

template <int EPI>
hipError_t launch_large(hipStream_t s, const void* A, const void* W, void* out, int M, int N, int K, bool configure_only = false) {
  constexpr int BM = 256, BN = 256, WM = 128, WN = 64;
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  constexpr int SMEM = 2 * (BM + BN) * LDS_ROW;
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN, EPI>;
  if (configure_only) return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
  int tilesM = (M + BM - 1) / BM;
  int tilesN = (EPI == EPI_SWIGLU) ? N / (BN / 2) : N / BN;
  kern<<<tilesM * tilesN, NT, SMEM, s>>>((const bf16_t*)A, (const bf16_t*)W, out, M, N, K, tilesM, tilesN);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
constexpr int SK = 128;                 // k extent of one staged activation slice
constexpr int SK_ROW = SK * 2 + 16;     // bytes per LDS row (padded)

// grid (Nw / 64, nsplit), 256 threads; wavefront w owns W rows n0 + 16 w .. +16 and all M (<= 16 MB) columns.
// Loads run D - 1 k-steps ahead of the MFMAs through a register ring (weights and the activation slice alike:
// the memory counter retires in order, so both must share one prefetch distance); the activation slice then
// passes through a double-buffered LDS tile that the four wavefronts share.
template <int MB, int D, bool GLU = false>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(const bf16_t* __restrict__ X, const bf16_t* __restrict__ W,
                                                          float* __restrict__ part, int M, int Nw, int K,
                                                          int steps_per_split) {
  static_assert(D == 2 || D == 4, "ring depth 2 or 4");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int XBYTES = 16 * MB * SK_ROW;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, t = lane & 15, g = lane >> 4;
  // GLU: W = [gate rows | up rows] of F = Nw / 2 features each; the workgroup owns 32 features, each wavefront
  // 8 of them with the gate rows in MFMA rows 0..7 and the matching up rows in 8..15.
  const int n0 = GLU ? blockIdx.x * 32 : blockIdx.x * 64;
  const int nsteps_total = K / SK;
  const int s0 = blockIdx.y * steps_per_split;
  const int s1 = min(nsteps_total, s0 + steps_per_split);

  f32x4_t acc[MB];
#pragma unroll
  for (int i = 0; i < MB; ++i) acc[i] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

  const int wrow = GLU ? ((t < 8) ? n0 + 8 * w + t : (Nw >> 1) + n0 + 8 * w + (t - 8)) : n0 + 16 * w + t;
  const bf16_t* wp = W + (size_t)wrow * K + 8 * g;
  // Activation slice: 16 MB rows x 16 chunks of 16 B per k-step, MB chunks per thread.  Rows beyond M are read
  // from row M - 1 instead: they only feed output columns that are never stored.
  const bf16_t* xp[MB];
  int xo[MB];
#pragma unroll
  for (int it = 0; it < MB; ++it) {
    int c = it * 256 + tid, r = c >> 4, kc = c & 15;
    xp[it] = X + (size_t)min(r, M - 1) * K + kc * 8;
    xo[it] = r * SK_ROW + kc * 16;
  }
  // Workgroups walk their k range from different starting points (wrapping around), so that they do not all
  // touch the same columns of W at the same time.
  const int nst = s1 - s0;
  const int rot = nst > 0 ? (int)((blockIdx.x * 5u + blockIdx.y * 3u) % (unsigned)nst) : 0;
  // Loads are issued without any branch around them (a step index past the end re-reads the last step, which
  // hits in cache): with straight-line code the compiler can keep D - 1 steps of loads in flight and wait only
  // for the oldest.
  auto step_off = [&](int i) -> size_t {
    int r = min(i, nst - 1) + rot;
    if (r >= nst) r -= nst;
    return (size_t)(s0 + r) * SK;
  };
  // Ring of D named slots (separate variables, so that they live in registers).
  struct Slot { uint4 w[4]; uint4 x[MB]; };
  Slot r0, r1, r2, r3;
#define SKINNY_LOAD(S, I)                                                                                \
  {                                                                                                      \
    const size_t ko = step_off(I);                                                                       \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) S.w[kk] = *(const uint4*)(wp + ko + kk * 32);       \
    _Pragma("unroll") for (int it = 0; it < MB; ++it) S.x[it] = *(const uint4*)(xp[it] + ko);            \
  }
  // one k-step on slot S (LDS buffer PAR)
#define SKINNY_STEP(S, PAR)                                                                              \
  {                                                                                                      \
    char* buf = smem + (PAR) * XBYTES;                                                                   \
    _Pragma("unroll") for (int it = 0; it < MB; ++it) *(uint4*)(buf + xo[it]) = S.x[it];                 \
    __syncthreads();                                                                                     \
    uint4 xf[2][MB];                                                                                     \
    _Pragma("unroll") for (int mb = 0; mb < MB; ++mb)                                                    \
        xf[0][mb] = *(const uint4*)(buf + (mb * 16 + t) * SK_ROW + g * 16);                              \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) {                                                   \
      if (kk < 3) {                                                                                      \
        _Pragma("unroll") for (int mb = 0; mb < MB; ++mb)                                                \
            xf[(kk + 1) & 1][mb] = *(const uint4*)(buf + (mb * 16 + t) * SK_ROW + (kk + 1) * 64 + g * 16); \
      }                                                                                                  \
      _Pragma("unroll") for (int mb = 0; mb < MB; ++mb)                                                  \
          acc[mb] = mfma_16x16x32(S.w[kk], xf[kk & 1][mb], acc[mb]);                                     \
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
    bf16_t* hout = (bf16_t*)part;
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
        o.x = pack_bf16x2(hv[0], hv[1]);
        o.y = pack_bf16x2(hv[2], hv[3]);
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

template <int MB>
hipError_t launch_skinny(hipStream_t s, const void* A, const void* W, float* part, int M, int Nw, int K, int nsplit,
                         bool configure_only = false) {
  constexpr int SMEM = 2 * 16 * MB * SK_ROW;
  constexpr int D = MB <= 4 ? 4 : 2;
  auto kern = gemm_skinny_kernel<MB, D>;
  if (configure_only) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void*)gemm_skinny_kernel<MB, D, true>, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
  }
  if (nsplit == 0) {  // fused SwiGLU: W = [2F, K], output bf16 [M, F], no split
    gemm_skinny_kernel<MB, D, true><<<dim3(Nw / 64, 1), 256, SMEM, s>>>((const bf16_t*)A, (const bf16_t*)W, part, M, Nw, K, K / SK);
    return hipGetLastError();
  }
  int steps = K / SK;
  int per = (steps + nsplit - 1) / nsplit;
  kern<<<dim3(Nw / 64, nsplit), 256, SMEM, s>>>((const bf16_t*)A, (const bf16_t*)W, part, M, Nw, K, per);
  return hipGetLastError();
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

hipError_t launch_gemm_bf16(hipStream_t s, const void* A, const void* W, void* out, int M, int N, int K, int epi) {
  if (M <= 0) return hipSuccess;
  if (K % BK) return hipErrorInvalidValue;
  if (epi == EPI_SWIGLU ? (N % 128) : (N % 256)) return hipErrorInvalidValue;
  switch (epi) {
    case EPI_STORE_F32: return launch_large<EPI_STORE_F32>(s, A, W, out, M, N, K);
    case EPI_RESID_F32: return launch_large<EPI_RESID_F32>(s, A, W, out, M, N, K);
    case EPI_SWIGLU: return launch_large<EPI_SWIGLU>(s, A, W, out, M, N, K);
    case EPI_STORE_ACT: return launch_large<EPI_STORE_ACT>(s, A, W, out, M, N, K);
  }
  return hipErrorInvalidValue;
}

// Raise the dynamic-LDS limit of every instantiation once per device (must not happen inside a stream capture).
hipError_t gemm_configure() {
  hipError_t e;
  if ((e = launch_large<EPI_STORE_F32>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_large<EPI_RESID_F32>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_large<EPI_SWIGLU>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_large<EPI_STORE_ACT>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, true)) != hipSuccess) return e;
  if ((e = launch_skinny<1>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, true)) != hipSuccess) return e;
  if ((e = launch_skinny<2>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, true)) != hipSuccess) return e;
  if ((e = launch_skinny<4>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, true)) != hipSuccess) return e;
  if ((e = launch_skinny<8>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, true)) != hipSuccess) return e;
  if ((e = launch_skinny<16>(nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 1, true)) != hipSuccess) return e;
  return hipSuccess;
}

int gemm_skinny_pick_split(int M, int Nw, int K) {
  (void)M;
  int tiles = Nw / 64, steps = K / SK;
  int want = (512 + tiles - 1) / tiles;
  if (want > 8) want = 8;
  if (want > steps) want = steps;
  if (want < 1) want = 1;
  int per = (steps + want - 1) / want;
  return (steps + per - 1) / per;  // no empty split
}

hipError_t launch_gemm_skinny_bf16(hipStream_t s, const void* A, const void* W, float* part, int M, int Nw, int K,
                                   int nsplit) {
  if (M <= 0) return hipSuccess;
  if (K % SK || Nw % 64 || M > 256 || nsplit < 0) return hipErrorInvalidValue;
  if (M <= 16) return launch_skinny<1>(s, A, W, part, M, Nw, K, nsplit);
  if (M <= 32) return launch_skinny<2>(s, A, W, part, M, Nw, K, nsplit);
  if (M <= 64) return launch_skinny<4>(s, A, W, part, M, Nw, K, nsplit);
  if (M <= 128) return launch_skinny<8>(s, A, W, part, M, Nw, K, nsplit);
  return launch_skinny<16>(s, A, W, part, M, Nw, K, nsplit);
}

hipError_t launch_gemm_f32(hipStream_t s, const float* A, const float* W, float* out, int M, int N, int K,
                           int accumulate) {
  if (M <= 0) return hipSuccess;
  dim3 grid((N + 15) / 16, (M + 15) / 16);
  gemm_f32_kernel<<<grid, 256, 0, s>>>(A, W, out, M, N, K, accumulate);
  return hipGetLastError();
}
