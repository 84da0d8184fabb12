// gnnagg_combine: the Combination phase (Section I: the per-vertex MLP update; Algorithm 1, Update)
// as one dense layer  out = act(X W + b).
//
// Why it is here: the paper runs Combination ahead of Aggregation so that Aggregation works at the
// hidden width (Section III); Aggregation is linear for sum / weighted sum / mean, so
// aggregate(X) W = aggregate(X W), and on the dense benchmark graph aggregating 32 columns instead of
// 602 is 20x less gather traffic.
//
// The layer is a tall-skinny GEMM (N x F times F x H, H <= a few hundred) and the one dense contraction
// of the path, so it runs on the matrix cores: v_mfma_f64_16x16x4_f64.  fp64 because the products of
// fp32 inputs are exact there and the sum is rounded once, like every other reduction of this library;
// at H = 32 the fp64 MFMA time (2 N F H flop at 78.6 TFLOP/s) is about the time HBM needs to deliver X
// once, so nothing is lost against fp32 MFMA.  A 256-thread workgroup computes 128 rows x up to 128
// columns: X and W tiles go through LDS (X transposed, so that the 16 lanes of an MFMA operand row read
// consecutive words), each wave owns 32 rows.
#include "common.hpp"
#include "device_utils.hpp"

namespace gnnagg {
namespace {

constexpr int kRowsPerBlock = 128;  // 4 waves x 32 rows
constexpr int kKTile = 32;          // k extent staged per step
constexpr int kMaxColTiles = 8;     // 8 x 16 = 128 output columns per pass
constexpr int kALd = kRowsPerBlock + 4;  // row pitch of the transposed X tile (words)

typedef double f64x4 __attribute__((ext_vector_type(4)));

struct CombineArgs {
  const void* X;
  const float* W;
  const float* bias;
  float* out;
  int64_t N;
  int32_t F, H;
  int32_t col0;       // first output column of this pass
  int32_t col_tiles;  // 16-column tiles in this pass (<= kMaxColTiles)
  int32_t relu;
};

__device__ inline float elem_as_float(const float* p) { return *p; }
__device__ inline float elem_as_float(const bf16_t* p) { return __uint_as_float((uint32_t)p->bits << 16); }

template <typename T, int CT>
__global__ __launch_bounds__(kBlock) void combine_kernel(const CombineArgs a) {
  __shared__ float As[kKTile * kALd];       // As[k][row]
  __shared__ float Bs[kKTile * CT * 16];    // Bs[k][col]
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
  const int64_t row0 = (int64_t)blockIdx.x * kRowsPerBlock;
  const T* __restrict__ X = static_cast<const T*>(a.X);
  constexpr int BN = CT * 16;

  f64x4 acc[2][CT];
#pragma unroll
  for (int r = 0; r < 2; ++r)
#pragma unroll
    for (int c = 0; c < CT; ++c) acc[r][c] = (f64x4){0.0, 0.0, 0.0, 0.0};

  for (int k0 = 0; k0 < a.F; k0 += kKTile) {
    // ---- stage the X tile, transposed: thread t reads 4 consecutive k of one row, 4 times
#pragma unroll
    for (int it = 0; it < (kRowsPerBlock * kKTile) / (kBlock * 4); ++it) {
      const int q = it * kBlock + tid;       // quad index: 8 quads per row
      const int r = q >> 3, kq = (q & 7) * 4;
      const int64_t row = row0 + r;
      float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      if (row < a.N) {
        const T* p = X + row * a.F + k0 + kq;
        if (k0 + kq + 4 <= a.F) {
          unpack(load_raw<T, 4>(p), v);  // one element-aligned vector load
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (k0 + kq + i < a.F) v[i] = elem_as_float(p + i);
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) As[(kq + i) * kALd + r] = v[i];
    }
    // ---- stage the W tile: Bs[k][j] = W[k0 + k][col0 + j], zero outside
    for (int q = tid; q < kKTile * BN; q += kBlock) {
      const int k = q / BN, j = q - k * BN;
      const int kk = k0 + k, col = a.col0 + j;
      Bs[q] = (kk < a.F && col < a.H) ? a.W[(int64_t)kk * a.H + col] : 0.0f;
    }
    __syncthreads();
    // ---- 8 MFMA steps of 4 k each; operand layout of v_mfma_f64_16x16x4_f64:
    //      A: lane l holds A[i = l % 16][k = l / 16], B: lane l holds B[k = l / 16][j = l % 16]
#pragma unroll
    for (int ks = 0; ks < kKTile; ks += 4) {
      const int k = ks + (lane >> 4);
      double av[2], bv[CT];
#pragma unroll
      for (int r = 0; r < 2; ++r) av[r] = (double)As[k * kALd + wv * 32 + r * 16 + (lane & 15)];
#pragma unroll
      for (int c = 0; c < CT; ++c) bv[c] = (double)Bs[k * BN + c * 16 + (lane & 15)];
#pragma unroll
      for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[r][c] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[r], bv[c], acc[r][c], 0, 0, 0);
    }
    __syncthreads();
  }
  // ---- epilogue; result layout: lane l holds D[i = 4 * v + l / 16][j = l % 16], v = 0..3
#pragma unroll
  for (int r = 0; r < 2; ++r) {
#pragma unroll
    for (int c = 0; c < CT; ++c) {
      const int col = a.col0 + c * 16 + (lane & 15);
      if (col >= a.H) continue;
      const double b = a.bias ? (double)a.bias[col] : 0.0;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int64_t row = row0 + wv * 32 + r * 16 + 4 * v + (lane >> 4);
        if (row >= a.N) continue;
        float y = (float)(acc[r][c][v] + b);
        if (a.relu) y = y > 0.0f ? y : 0.0f;
        a.out[row * a.H + col] = y;
      }
    }
  }
}

template <typename T>
int launch_combine(const CombineArgs& a, hipStream_t stream) {
  const dim3 grid((unsigned)ceil_div(a.N, kRowsPerBlock));
  switch (a.col_tiles) {
    case 1: hipLaunchKernelGGL((combine_kernel<T, 1>), grid, dim3(kBlock), 0, stream, a); break;
    case 2: hipLaunchKernelGGL((combine_kernel<T, 2>), grid, dim3(kBlock), 0, stream, a); break;
    case 3: case 4: hipLaunchKernelGGL((combine_kernel<T, 4>), grid, dim3(kBlock), 0, stream, a); break;
    default: hipLaunchKernelGGL((combine_kernel<T, 8>), grid, dim3(kBlock), 0, stream, a); break;
  }
  return hipGetLastError() == hipSuccess ? GNNAGG_OK : GNNAGG_EDEVICE;
}

}  // namespace
}  // namespace gnnagg

using namespace gnnagg;

extern "C" int gnnagg_combine(int64_t N, const void* X, int x_dtype, int32_t F, const float* W, const float* bias,
                              int32_t H, int relu, float* out, void* stream_) {
  if (N < 0 || F <= 0 || H <= 0 || (relu != 0 && relu != 1)) return GNNAGG_EINVAL;
  if (x_dtype != GNNAGG_F32 && x_dtype != GNNAGG_BF16) return GNNAGG_EINVAL;
  if (N == 0) return GNNAGG_OK;
  if (!X || !W || !out) return GNNAGG_ENULL;
  const size_t xs = (x_dtype == GNNAGG_F32) ? 4 : 2;
  if (((uintptr_t)X % xs) || ((uintptr_t)W % 4) || ((uintptr_t)out % 4) || (bias && ((uintptr_t)bias % 4)))
    return GNNAGG_EINVAL;
  if (X == (const void*)out) return GNNAGG_EINVAL;
  if (ceil_div(N, kRowsPerBlock) > 0x7fffffffll) return GNNAGG_EUNSUPPORTED;
  hipStream_t stream = (hipStream_t)stream_;
  // output columns in passes of at most 128: X is re-read once per pass
  for (int32_t col0 = 0; col0 < H; col0 += kMaxColTiles * 16) {
    CombineArgs a;
    a.X = X;
    a.W = W;
    a.bias = bias;
    a.out = out;
    a.N = N;
    a.F = F;
    a.H = H;
    a.col0 = col0;
    const int32_t cols = (H - col0 < kMaxColTiles * 16) ? H - col0 : kMaxColTiles * 16;
    a.col_tiles = (int32_t)ceil_div(cols, 16);
    a.relu = relu;
    int rc = (x_dtype == GNNAGG_F32) ? launch_combine<float>(a, stream) : launch_combine<bf16_t>(a, stream);
    if (rc != GNNAGG_OK) return rc;
  }
  return GNNAGG_OK;
}
