// GEMMs of the rollout, out = A[M,K] * W[N,K]^T with both operands K-contiguous.
//   gemm_bf16_kernel    : large-tile bf16 MFMA GEMM for prefill (M = thousands of tokens): 256x256x64 block tile,
//                         8 wavefronts of 128x64, LDS double buffer fed through registers, 32x32x16 MFMA.
//   gemm_skinny_kernel  : weight-streaming GEMM for decode (M = batch <= 256): W is the MFMA row operand read
//                         straight from HBM into registers exactly once, the activation slice is staged in LDS,
//                         split-K partial sums go to a workspace that the consumer kernel adds up in a fixed order.
//   gemm_f32_kernel     : plain-ALU fp32 GEMM for the small fp32 configuration.
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
template <int MB>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(const bf16_t* __restrict__ X, const bf16_t* __restrict__ W,
                                                          float* __restrict__ part, int M, int Nw, int K,
                                                          int steps_per_split) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int XBYTES = 16 * MB * SK_ROW;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, t = lane & 15, g = lane >> 4;
  const int n0 = blockIdx.x * 64;
  const int nsteps_total = K / SK;
  const int s0 = blockIdx.y * steps_per_split;
  const int s1 = min(nsteps_total, s0 + steps_per_split);

  f32x4_t acc[MB];
#pragma unroll
  for (int i = 0; i < MB; ++i) acc[i] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

  const bf16_t* wp = W + (size_t)(n0 + 16 * w + t) * K + 8 * g;
  // activation slice: 16 MB rows x 16 chunks of 16 B; thread handles MB chunks
  const bf16_t* xp[MB];
  int xo[MB];
  bool xv[MB];
#pragma unroll
  for (int it = 0; it < MB; ++it) {
    int c = it * 256 + tid, r = c >> 4, kc = c & 15;
    xv[it] = r < M;
    xp[it] = X + (size_t)(xv[it] ? r : 0) * K + kc * 8;
    xo[it] = r * SK_ROW + kc * 16;
  }
  uint4 wa[4], wb[4], xr[MB];
  if (s0 < s1) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) wa[kk] = *(const uint4*)(wp + (size_t)s0 * SK + kk * 32);
#pragma unroll
    for (int it = 0; it < MB; ++it)
      xr[it] = xv[it] ? *(const uint4*)(xp[it] + (size_t)s0 * SK) : make_uint4(0, 0, 0, 0);
  }
  for (int st = s0; st < s1; ++st) {
    char* buf = smem + ((st - s0) & 1) * XBYTES;
#pragma unroll
    for (int it = 0; it < MB; ++it) *(uint4*)(buf + xo[it]) = xr[it];
    __syncthreads();
    if (st + 1 < s1) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) wb[kk] = *(const uint4*)(wp + (size_t)(st + 1) * SK + kk * 32);
#pragma unroll
      for (int it = 0; it < MB; ++it)
        xr[it] = xv[it] ? *(const uint4*)(xp[it] + (size_t)(st + 1) * SK) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        uint4 xf = *(const uint4*)(buf + (mb * 16 + t) * SK_ROW + kk * 64 + g * 16);
        acc[mb] = mfma_16x16x32(wa[kk], xf, acc[mb]);
      }
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) wa[kk] = wb[kk];
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
  auto kern = gemm_skinny_kernel<MB>;
  if (configure_only) return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
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
  if (K % SK || Nw % 64 || M > 256 || nsplit < 1) return hipErrorInvalidValue;
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
