// Measurement kernels with no part in the sampler: the ceilings that the sampler's
// kernels are held against are measured on the same device, in the same run.
#include "common.hpp"

#include <algorithm>

using namespace augur;

namespace {

// dst[i] = src[i], 16 bytes a thread and trip: the plain streaming copy whose rate stands for
// the bandwidth of the memory system that a kernel can reach, and whose known size scales the
// profiler's byte counters.
__global__ __launch_bounds__(256) void stream_copy_kernel(const float4* __restrict__ src,
                                                           float4* __restrict__ dst, int64_t n16) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
       i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

}  // namespace

namespace augur {
__global__ void sweep_counter_add_kernel(uint32_t* counter, uint32_t add) {
  if (blockIdx.x == 0 && threadIdx.x == 0) *counter += add;
}
__global__ void sweep_counter_set_kernel(uint32_t* counter, uint32_t value) {
  if (blockIdx.x == 0 && threadIdx.x == 0) *counter = value;
}
}  // namespace augur

extern "C" {

int augur_probe_stream_copy(const void* src, void* dst, int64_t bytes, int32_t reps, void* stream,
                            double* ms_per_copy) {
  AUGUR_REQUIRE(src != nullptr && dst != nullptr && ms_per_copy != nullptr, "NULL argument");
  AUGUR_REQUIRE(bytes > 0 && bytes % 16 == 0 && reps > 0, "bytes must be a positive multiple of 16 and reps positive");
  AUGUR_REQUIRE(((uintptr_t)src & 15) == 0 && ((uintptr_t)dst & 15) == 0, "src and dst must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int64_t n16 = bytes / 16;
  const unsigned blocks = (unsigned)std::min<int64_t>((n16 + 255) / 256, 256 * 32);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  AUGUR_HIP_TRY(hipEventCreate(&e0));
  hipError_t err = hipEventCreate(&e1);
  if (err == hipSuccess) {
    hipLaunchKernelGGL(stream_copy_kernel, dim3(blocks), dim3(256), 0, s, (const float4*)src, (float4*)dst, n16);  // warm-up
    err = hipEventRecord(e0, s);
  }
  for (int r = 0; r < reps && err == hipSuccess; ++r) {
    hipLaunchKernelGGL(stream_copy_kernel, dim3(blocks), dim3(256), 0, s, (const float4*)src, (float4*)dst, n16);
    err = hipGetLastError();
  }
  if (err == hipSuccess) err = hipEventRecord(e1, s);
  if (err == hipSuccess) err = hipEventSynchronize(e1);
  float ms = 0.f;
  if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  AUGUR_HIP_TRY(err);
  *ms_per_copy = (double)ms / reps;
  return AUGUR_OK;
}

}  // extern "C"
