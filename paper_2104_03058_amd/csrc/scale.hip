// gnnagg_gcn_factors, gnnagg_scale_rows: GCN's aggregation weights in factored form (the GCN operator
// of Section III).  1/sqrt(d_i d_j) is a product of one factor per destination and one per source; with
// the sources' factors multiplied into the feature rows once, the aggregation is a plain sum that is
// scaled per destination at its store (GNNAGG_SUM_SCALED), and the per-edge weights are never read.
#include <hip/hip_runtime.h>

#include "common.hpp"
#include "device_utils.hpp"

namespace gnnagg {
namespace {

__global__ __launch_bounds__(kBlock) void gcn_factors_kernel(int64_t N, const int64_t* __restrict__ rowptr,
                                                             float* __restrict__ s) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= N) return;
  const int64_t d = rowptr[i + 1] - rowptr[i];
  s[i] = d > 0 ? (float)(1.0 / sqrt((double)d)) : 0.0f;
}

struct ScaleArgs {
  const void* X;
  const float* scale;
  float* out;
  int64_t N, F, x_pitch, out_pitch;
  int32_t lanes_log2;  // 2^lanes_log2 lanes share a row; a wavefront covers 64 >> lanes_log2 rows
};

// Lanes take four columns a step (rows may start at any element: the vector types promise element
// alignment only), then one column each over the last F % 4.
template <typename T>
__global__ __launch_bounds__(kBlock) void scale_rows_kernel(const ScaleArgs a) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  const int L = a.lanes_log2;
  const int64_t r = (wave << (6 - L)) + (lane >> L);
  if (r >= a.N) return;
  const float s = a.scale[r];
  // no restrict: X and out may be the same matrix (each element is read, then written, by one lane)
  const T* x = static_cast<const T*>(a.X) + r * a.x_pitch;
  float* o = a.out + r * a.out_pitch;
  const int64_t sub = lane & ((1 << L) - 1);
  const int64_t F4 = a.F & ~(int64_t)3;
  for (int64_t c = sub * 4; c < F4; c += (int64_t)4 << L) {
    float v[4];
    unpack(load_raw<T, 4>(x + c), v);
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] *= s;
    store_row<4>(o + c, v);
  }
  for (int64_t c = F4 + sub; c < a.F; c += (int64_t)1 << L) {
    float v[1];
    unpack(load_raw<T, 1>(x + c), v);
    o[c] = v[0] * s;
  }
}

template <typename T>
int launch_scale(const ScaleArgs& a, hipStream_t stream) {
  const int64_t rows_per_block = (int64_t)kWavesPerBlock << (6 - a.lanes_log2);
  const int64_t blocks = ceil_div(a.N, rows_per_block);
  if (blocks > 0x7fffffffll) return GNNAGG_EUNSUPPORTED;
  hipLaunchKernelGGL((scale_rows_kernel<T>), dim3((unsigned)blocks), dim3(kBlock), 0, stream, a);
  return hipGetLastError() == hipSuccess ? GNNAGG_OK : GNNAGG_EDEVICE;
}

}  // namespace
}  // namespace gnnagg

using namespace gnnagg;

extern "C" int gnnagg_gcn_factors(int64_t N, const int64_t* rowptr, float* s, void* stream) {
  if (N < 0) return GNNAGG_EINVAL;
  if (N == 0) return GNNAGG_OK;
  if (!rowptr || !s) return GNNAGG_ENULL;
  if (((uintptr_t)rowptr % 8) || ((uintptr_t)s % 4)) return GNNAGG_EINVAL;
  const int64_t blocks = ceil_div(N, (int64_t)kBlock);
  if (blocks > 0x7fffffffll) return GNNAGG_EUNSUPPORTED;
  hipLaunchKernelGGL(gcn_factors_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, static_cast<hipStream_t>(stream), N,
                     rowptr, s);
  return hipGetLastError() == hipSuccess ? GNNAGG_OK : GNNAGG_EDEVICE;
}

extern "C" int gnnagg_scale_rows(int64_t N, int32_t F, const void* X, int x_dtype, int64_t x_pitch, const float* scale,
                                 float* out, int64_t out_pitch, void* stream) {
  if (N < 0 || F <= 0) return GNNAGG_EINVAL;
  if (x_dtype != GNNAGG_F32 && x_dtype != GNNAGG_BF16) return GNNAGG_EINVAL;
  if (x_pitch == 0) x_pitch = F;
  if (out_pitch == 0) out_pitch = F;
  if (x_pitch < F || out_pitch < F || x_pitch > (1ll << 40) || out_pitch > (1ll << 40)) return GNNAGG_EINVAL;
  if (N == 0) return GNNAGG_OK;
  if (!X || !scale || !out) return GNNAGG_ENULL;
  const size_t xs = (x_dtype == GNNAGG_F32) ? 4 : 2;
  if (((uintptr_t)X % xs) || ((uintptr_t)out % 4) || ((uintptr_t)scale % 4)) return GNNAGG_EINVAL;
  // in place only when every element is read and written by the same lane at the same address
  if (X == (const void*)out && (x_dtype != GNNAGG_F32 || x_pitch != out_pitch)) return GNNAGG_EINVAL;
  ScaleArgs a;
  a.X = X;
  a.scale = scale;
  a.out = out;
  a.N = N;
  a.F = F;
  a.x_pitch = x_pitch;
  a.out_pitch = out_pitch;
  const int64_t steps = ceil_div((int64_t)F, 4);  // lane-steps a row takes
  int L = 0;
  while (L < 6 && ((int64_t)1 << L) < steps) ++L;
  a.lanes_log2 = L;
  return (x_dtype == GNNAGG_F32) ? launch_scale<float>(a, static_cast<hipStream_t>(stream))
                                 : launch_scale<bf16_t>(a, static_cast<hipStream_t>(stream));
}
