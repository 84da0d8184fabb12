// gnnagg_copy_probe: a plain streaming copy, used to measure the HBM copy rate
// next to the aggregation kernels and to calibrate the profiler's byte counters
// against a kernel whose traffic is known (bytes read = bytes written = n).
#include "common.hpp"

namespace gnnagg {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kBlock) void copy_probe_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                            int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace
}  // namespace gnnagg

using namespace gnnagg;

extern "C" int gnnagg_copy_probe(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src) return GNNAGG_ENULL;
  if (bytes % 16 || ((uintptr_t)dst % 16) || ((uintptr_t)src % 16)) return GNNAGG_EINVAL;
  if (bytes == 0) return GNNAGG_OK;
  const int64_t n16 = (int64_t)(bytes / 16);
  int64_t blocks = ceil_div(n16, kBlock);
  if (blocks > 256 * 32) blocks = 256 * 32;  // 32 workgroups per compute unit, grid-stride beyond
  hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, (hipStream_t)stream,
                     (const u32x4*)src, (u32x4*)dst, n16);
  GNNAGG_HIP_TRY(hipGetLastError());
  return GNNAGG_OK;
}
