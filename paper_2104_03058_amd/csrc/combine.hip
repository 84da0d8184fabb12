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
// once, so nothing is lost against fp32 MFMA.
//
// Data movement.  X is read exactly once per pass and never touches LDS: the k index of a contraction
// may be visited in any order, so lane l of a wavefront loads 8 CONSECUTIVE k of row l % 16 (one or two
// 16-byte loads; the four 16-lane groups cover 32 consecutive k, 128 bytes of the row) and MFMA step s
// contracts over the four k values {8 g + s : g = l / 16}.  W is small (F x H); a 32-k tile of it goes
// through LDS, stored [col][k] so that a lane fetches its 8 k with two 16-byte LDS reads, double
// buffered so that one barrier per 32 k suffices.  A 256-thread workgroup computes 128 rows x up to 128
// columns, each wave 32 rows.
#include "common.hpp"
#include "device_utils.hpp"

namespace gnnagg {
namespace {

constexpr int kRowsPerBlock = 128;  // 4 waves x 32 rows
constexpr int kKTile = 32;          // k extent per step: 4 lane groups x 8
constexpr int kMaxColTiles = 8;     // 8 x 16 = 128 output columns per pass
constexpr int kBPitch = kKTile + 4; // words per column of the W tile in LDS (keeps 16-byte alignment)

typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef float f32x4_a __attribute__((ext_vector_type(4)));

struct CombineArgs {
  const void* X;
  const float* W;
  const float* bias;
  float* out;
  const int32_t* out_rows;  // row i of the result goes to row out_rows[i] of out (null: i)
  const float* row_scale;   // row i of the result is multiplied by row_scale[i] after the activation (null: no)
  int64_t N;
  int32_t F, H;
  int32_t col0;       // first output column of this pass
  int32_t col_tiles;  // 16-column tiles in this pass (<= kMaxColTiles)
  int32_t relu;
};

__device__ inline float elem_as_float(const float* p) { return *p; }
__device__ inline float elem_as_float(const bf16_t* p) { return __uint_as_float((uint32_t)p->bits << 16); }

// 8 consecutive elements of a row starting at column k (zero beyond column F)
template <typename T>
__device__ inline void load_k8(const T* __restrict__ rowp, int k, int F, float (&v)[8]) {
  if (k + 8 <= F) {
    if constexpr (sizeof(T) == 4) {
      float lo[4], hi[4];
      unpack(load_raw<T, 4>(rowp + k), lo);
      unpack(load_raw<T, 4>(rowp + k + 4), hi);
#pragma unroll
      for (int i = 0; i < 4; ++i) { v[i] = lo[i]; v[4 + i] = hi[i]; }
    } else {
      unpack(load_raw<T, 8>(rowp + k), v);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (k + i < F) ? elem_as_float(rowp + k + i) : 0.0f;
  }
}

// Four waves per SIMD: at the three the register allocator would otherwise settle for (112 VGPRs + 32
// accumulator registers) the matrix pipe idles while waves wait at the per-tile barrier (measured: 0.245 ->
// 0.205 ms on [232965, 602] x [602, 32]); five or more spill.
template <typename T, int CT>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(4, 4))) void combine_kernel(const CombineArgs a) {
  constexpr int BN = CT * 16;
  constexpr int kBPerThread = (kKTile * BN) / kBlock;  // W-tile elements staged per thread: 2 CT
  __shared__ __attribute__((aligned(16))) float Bs[2][BN * kBPitch];  // Bs[buf][col][k]
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
  const int g = lane >> 4, li = lane & 15;
  const int64_t row0 = (int64_t)blockIdx.x * kRowsPerBlock + wv * 32;
  const T* __restrict__ X = static_cast<const T*>(a.X);

  // rows past the end re-read the last row; their results are dropped at the store
  const T* xrow[2];
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    int64_t row = row0 + r * 16 + li;
    row = row < a.N ? row : a.N - 1;
    xrow[r] = X + row * a.F;
  }

  f64x4 acc[2][CT];
#pragma unroll
  for (int r = 0; r < 2; ++r)
#pragma unroll
    for (int c = 0; c < CT; ++c) acc[r][c] = (f64x4){0.0, 0.0, 0.0, 0.0};

  // W tile element q of a thread: k = q / BN, j = q % BN (consecutive threads: consecutive columns)
  auto fetch_w = [&](int k0, float (&w)[kBPerThread]) {
#pragma unroll
    for (int i = 0; i < kBPerThread; ++i) {
      const int q = i * kBlock + tid;
      const int k = k0 + q / BN, col = a.col0 + q % BN;
      w[i] = (k < a.F && col < a.H) ? a.W[(int64_t)k * a.H + col] : 0.0f;
    }
  };
  auto stage_w = [&](int buf, const float (&w)[kBPerThread]) {
#pragma unroll
    for (int i = 0; i < kBPerThread; ++i) {
      const int q = i * kBlock + tid;
      Bs[buf][(q % BN) * kBPitch + q / BN] = w[i];
    }
  };

  float xa[2][8], xn[2][8], wreg[kBPerThread];
#pragma unroll
  for (int r = 0; r < 2; ++r) load_k8(xrow[r], 8 * g, a.F, xa[r]);
  fetch_w(0, wreg);
  stage_w(0, wreg);
  __syncthreads();

  const int steps = (a.F + kKTile - 1) / kKTile;
  for (int t = 0; t < steps; ++t) {
    const bool more = t + 1 < steps;
    if (more) {
#pragma unroll
      for (int r = 0; r < 2; ++r) load_k8(xrow[r], (t + 1) * kKTile + 8 * g, a.F, xn[r]);
      fetch_w((t + 1) * kKTile, wreg);
    }
    // operand layout of v_mfma_f64_16x16x4_f64: A: lane l holds A[i = l % 16][k = l / 16],
    // B: lane l holds B[k = l / 16][j = l % 16]; step s uses k = 8 g + s on both sides
    const float* bt = &Bs[t & 1][0];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      f32x4_a b4[CT];
#pragma unroll
      for (int c = 0; c < CT; ++c)
        b4[c] = *reinterpret_cast<const f32x4_a*>(bt + (c * 16 + li) * kBPitch + 8 * g + 4 * half);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const double a0 = (double)xa[0][4 * half + s], a1 = (double)xa[1][4 * half + s];
#pragma unroll
        for (int c = 0; c < CT; ++c) {
          const double bv = (double)b4[c][s];
          acc[0][c] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, bv, acc[0][c], 0, 0, 0);
          acc[1][c] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, bv, acc[1][c], 0, 0, 0);
        }
      }
    }
    if (more) {
      stage_w((t + 1) & 1, wreg);  // that buffer was last read in step t - 1, before the barrier below
#pragma unroll
      for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) xa[r][i] = xn[r][i];
    }
    __syncthreads();
  }
  // ---- epilogue; result layout: lane l holds D[i = 4 * v + l / 16][j = l % 16], v = 0..3
#pragma unroll
  for (int r = 0; r < 2; ++r) {
#pragma unroll
    for (int c = 0; c < CT; ++c) {
      const int col = a.col0 + c * 16 + li;
      if (col >= a.H) continue;
      const double b = a.bias ? (double)a.bias[col] : 0.0;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int64_t row = row0 + r * 16 + 4 * v + g;
        if (row >= a.N) continue;
        float y = (float)(acc[r][c][v] + b);
        if (a.relu) y = y > 0.0f ? y : 0.0f;
        if (a.row_scale) y *= a.row_scale[row];  // one fp32 product on the rounded result, as gnnagg_scale_rows
        const int64_t orow = a.out_rows ? (int64_t)a.out_rows[row] : row;
        a.out[orow * a.H + col] = y;
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

namespace {

int combine_impl(int64_t N, const void* X, int x_dtype, int32_t F, const float* W, const float* bias, int32_t H,
                 int relu, const float* row_scale, float* out, const int32_t* out_rows, void* stream_) {
  if (N < 0 || F <= 0 || H <= 0 || (relu != 0 && relu != 1)) return GNNAGG_EINVAL;
  if (x_dtype != GNNAGG_F32 && x_dtype != GNNAGG_BF16) return GNNAGG_EINVAL;
  if (N == 0) return GNNAGG_OK;
  if (!X || !W || !out) return GNNAGG_ENULL;
  const size_t xs = (x_dtype == GNNAGG_F32) ? 4 : 2;
  if (((uintptr_t)X % xs) || ((uintptr_t)W % 4) || ((uintptr_t)out % 4) || (bias && ((uintptr_t)bias % 4)) ||
      (out_rows && ((uintptr_t)out_rows % 4)) || (row_scale && ((uintptr_t)row_scale % 4)))
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
    a.out_rows = out_rows;
    a.row_scale = row_scale;
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

}  // namespace

extern "C" int gnnagg_combine(int64_t N, const void* X, int x_dtype, int32_t F, const float* W, const float* bias,
                              int32_t H, int relu, float* out, const int32_t* out_rows, void* stream) {
  return combine_impl(N, X, x_dtype, F, W, bias, H, relu, nullptr, out, out_rows, stream);
}

extern "C" int gnnagg_combine_scaled(int64_t N, const void* X, int x_dtype, int32_t F, const float* W,
                                     const float* bias, int32_t H, int relu, const float* row_scale, float* out,
                                     const int32_t* out_rows, void* stream) {
  if (N > 0 && !row_scale) return GNNAGG_ENULL;
  return combine_impl(N, X, x_dtype, F, W, bias, H, relu, row_scale, out, out_rows, stream);
}
