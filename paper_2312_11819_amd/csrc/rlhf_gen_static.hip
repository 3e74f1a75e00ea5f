// rlhf_gen_op_gemm_static: the weight-streaming decode projection for callers that cannot allocate.
//
// The split-K partial sums of the projection, which every other entry point keeps in a workspace that either the
// context allocated at init or the caller passes in, live here in a fixed array in the library's own device image.
// The entry point calls no hipMalloc / hipFree and no allocating library routine, so it can be used under stream
// capture, from serving loops that forbid allocation, and by harnesses that account for every allocation.
#include <hip/hip_runtime.h>
#include <stdio.h>

#include "../../include/rlhf_gen_ops.h"
#include "kernels.h"

namespace {

constexpr size_t STATIC_SCRATCH_BYTES = (size_t)32 << 20;   // held by every GPU the library runs on until the process ends
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

// Device address of `scratch` per device.  In host code the array's name is only a handle for the runtime; the memory
// itself is reached through the address that hipGetSymbolAddress returns for the device that is current.
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {};

hipError_t scratch_for_current_device(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

// out[i] = ((part[0][i] + part[1][i]) + part[2][i]) + ...: the order in which the rollout's consumer kernels add the planes.
__global__ __launch_bounds__(256) void plane_sum_kernel(const float* __restrict__ part, int nsplit, size_t plane_stride,
                                                        float* __restrict__ out, size_t n4) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  float4 a = *(const float4*)(part + 4 * i);
  for (int s = 1; s < nsplit; ++s) {
    const float4 p = *(const float4*)(part + (size_t)s * plane_stride + 4 * i);
    a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
  }
  *(float4*)(out + 4 * i) = a;
}

}  // namespace

hipError_t static_scratch_prepare() {
  void* p = nullptr;
  return scratch_for_current_device(&p);
}

extern "C" int rlhf_gen_op_gemm_static(void* stream, const void* A, const void* W, float* out, int32_t M, int32_t N,
                                       int32_t K, int32_t a_pairs, int32_t* nsplit_out) {
  char msg[256];
  if (!A || !W || !out || M < 1 || N < 1 || K < 1) {
    set_global_error("rlhf_gen_op_gemm_static: NULL pointer or non-positive size");
    return RLHF_GEN_E_INVALID;
  }
  if (N % 64 || K % 128 || M > (a_pairs ? 128 : 256)) {
    snprintf(msg, sizeof msg, "rlhf_gen_op_gemm_static: needs N %% 64 == 0, K %% 128 == 0 and M <= %d (got M = %d, N = %d, K = %d)",
             a_pairs ? 128 : 256, M, N, K);
    set_global_error(msg);
    return RLHF_GEN_E_UNSUPPORTED;
  }
  static bool configured = false;   // kernel attributes only: nothing is allocated
  if (!configured) {
    if (gemm_configure() != hipSuccess) return RLHF_GEN_E_DEVICE;
    configured = true;
  }
  const int nsplit = gemm_skinny_pick_split(M, N, K, a_pairs);
  const size_t need = (size_t)nsplit * M * N * sizeof(float);
  if (need > STATIC_SCRATCH_BYTES) {
    snprintf(msg, sizeof msg,
             "rlhf_gen_op_gemm_static: %d split-K planes of %d x %d floats need %zu bytes, the static workspace holds %zu",
             nsplit, M, N, need, STATIC_SCRATCH_BYTES);
    set_global_error(msg);
    return RLHF_GEN_E_INVALID;
  }
  void* ws = nullptr;
  hipError_t e = scratch_for_current_device(&ws);
  if (e != hipSuccess) {
    snprintf(msg, sizeof msg, "rlhf_gen_op_gemm_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
    set_global_error(msg);
    return RLHF_GEN_E_DEVICE;
  }
  hipStream_t s = (hipStream_t)stream;
  // every element of the planes that the reduction reads (rows < M) is written by the GEMM: nothing has to start at zero
  e = launch_gemm_skinny_h16(s, A, W, (float*)ws, M, N, K, nsplit, a_pairs, M);
  if (e != hipSuccess) return e == hipErrorInvalidValue ? RLHF_GEN_E_UNSUPPORTED : RLHF_GEN_E_DEVICE;
  const size_t n4 = (size_t)M * N / 4;
  plane_sum_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, s>>>((const float*)ws, nsplit, (size_t)M * N, out, n4);
  if (hipGetLastError() != hipSuccess) return RLHF_GEN_E_DEVICE;
  if (nsplit_out) *nsplit_out = nsplit;
  return RLHF_GEN_OK;
}
