// Hardware probes: what this card sustains for the two resources the rollout is bound by, measured with nothing else
// in the way, so that the benchmark can quote its kernels against achievable rates as well as datasheet peaks.
//   stream_read_kernel : read-only stream over a buffer, 16 bytes per lane, eight loads in flight per lane
//   mfma_loop_kernel   : v_mfma_f32_32x32x16_f16 on register-resident operands (no memory traffic in the loop)
#include "common.h"
#include "kernels.h"

namespace {

template <bool NT>
__global__ __launch_bounds__(256) void stream_read_kernel(const char* __restrict__ buf, size_t nchunks,
                                                          unsigned* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6), nw = (size_t)gridDim.x * 4;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (size_t c = wave; c < nchunks; c += nw) {   // one chunk = 8 KB = eight wavefront-wide 1 KB loads
    const char* p = buf + c * 8192 + lane * 16;
    uint4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = NT ? load_stream16(p + i * 1024) : *(const uint4*)(p + i * 1024);
#pragma unroll
    for (int i = 0; i < 8; ++i) { acc.x ^= v[i].x; acc.y ^= v[i].y; acc.z ^= v[i].z; acc.w ^= v[i].w; }
  }
  // keep the loads alive without writing anything in the common case
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345677u) out[threadIdx.x] = acc.x;
}

__global__ __launch_bounds__(256) void mfma_loop_kernel(const uint4* __restrict__ operands, int iters,
                                                        float* __restrict__ out) {
  // four A and two B fragments per wavefront, eight independent 32x32 accumulators
  uint4 a[4], b[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = operands[(threadIdx.x * 4 + i) & 1023];
#pragma unroll
  for (int i = 0; i < 2; ++i) b[i] = operands[(threadIdx.x * 2 + i + 512) & 1023];
  f32x16_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i * 2 + j] = mfma_32x32x16(a[i], b[j], acc[i * 2 + j]);
  }
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) r += acc[i][e];
  if (r == 1234.567f) out[threadIdx.x] = r;
}

}  // namespace

hipError_t launch_probe_stream_read(hipStream_t s, const void* buf, size_t bytes, int nontemporal, void* scratch) {
  if (bytes < 8192) return hipErrorInvalidValue;
  const size_t nchunks = bytes / 8192;
  // one workgroup per compute unit, each walking the buffer with a stride of the whole grid: the launch shape that
  // measured fastest (7.2 TB/s over 4 GiB; 7.1 with eight times as many workgroups)
  static int num_cu = 0;
  if (num_cu == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    num_cu = (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
                 ? prop.multiProcessorCount : 256;
  }
  const unsigned grid = (unsigned)std::min<size_t>((size_t)num_cu, (nchunks + 3) / 4);
  if (nontemporal)
    stream_read_kernel<true><<<grid, 256, 0, s>>>((const char*)buf, nchunks, (unsigned*)scratch);
  else
    stream_read_kernel<false><<<grid, 256, 0, s>>>((const char*)buf, nchunks, (unsigned*)scratch);
  return hipGetLastError();
}

hipError_t launch_probe_mfma_loop(hipStream_t s, const void* operands, int workgroups, int iters, void* scratch) {
  if (workgroups < 1 || iters < 1) return hipErrorInvalidValue;
  mfma_loop_kernel<<<workgroups, 256, 0, s>>>((const uint4*)operands, iters, (float*)scratch);
  return hipGetLastError();
}
