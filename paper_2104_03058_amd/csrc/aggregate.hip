// gnnagg_aggregate: sum / weighted sum / mean / max over CSR neighbour lists,
// one feature slice at a time (paper Algorithm 1: Message, Aggregate, Concat).
//
// Work decomposition for wave64 hardware
//   - A feature slice is at most 64 lanes x VEC columns (VEC columns = 16 bytes
//     of input per lane), so the lanes that share a neighbour read one
//     contiguous piece of its row: the gathers coalesce.
//   - 2^g lanes span the slice; a row gets 2^L lanes (L >= g), i.e. 2^(L-g)
//     neighbour slots that walk the row's edge list interleaved and are merged
//     with cross-lane shuffles at the end.  L comes from the row's degree class:
//     short rows share a wave (several rows per wave), long rows get a wave,
//     hub rows get the whole workgroup and meet in LDS.
//   - Slices are enumerated chunk-major over the grid, so chunks run in the
//     chunk-outer / vertex-inner order of Algorithm 1 and each slice is written
//     straight into its columns of `out` (the Concat step costs nothing).
//   - Sums accumulate in fp64 (full rate on this chip) and are rounded to fp32
//     once, so the result does not depend on the degree or on how the row was
//     split; max works on order-preserving integer keys and is exact.
#include <atomic>
#include <mutex>

#include "common.hpp"
#include "schedule.hpp"
#include "device_utils.hpp"
#include "gather.hpp"

namespace gnnagg {
namespace {

enum { OPK_SUM = 0, OPK_WSUM = 1, OPK_MAX = 2 };

// Wide slices hand the edge indices round with swizzles.  The alternative through LDS tiles
// (gather_wide_staged) is kept for comparison, behind a definition at build time: it measured level to
// 4 % slower on the benchmark shapes.
#ifndef GNNAGG_STAGE_INDICES
#define GNNAGG_STAGE_INDICES 0
#endif
constexpr bool kStageIndices = GNNAGG_STAGE_INDICES != 0;

struct AggArgs {
  const int64_t* rowptr;
  const int32_t* colidx;
  const float* edge_w;
  const float* row_scale;  // [N]: the finished sum of row r is multiplied by row_scale[r] (null: by 1)
  const void* X;
  void* out;
  int32_t out_bf16;  // 1: out holds bf16 (the fp32 result rounded to nearest even), 0: fp32
  const int32_t* order;
  int64_t F;
  int64_t x_pitch, out_pitch;  // elements between consecutive rows of X / out (>= F)
  int64_t N;
  SliceLaunch sl;
  int32_t mean;
  uint32_t lds_per_workgroup;  // host only: LDS each workgroup should occupy (0 = no cap)
  double* ws;                  // partial results of split rows: [slot][F] (null: no row is split)
  // One source block of a blocked call (all null: the whole edge list of every row).  The call walks
  // edges [e_begin[r], e_end[r]) of row r only; `pin` (N rows of p_pitch doubles) holds the state the
  // earlier blocks left (sums as doubles, max as its integer key in a double), `pout` receives this
  // block's instead of a finished row.  The degree that finishes a row (mean, empty-row rule of max)
  // stays rowptr's.
  const int64_t* e_begin;
  const int64_t* e_end;
  const double* pin;
  double* pout;
  int64_t p_pitch;  // doubles between the rows of pin / pout (rows start on 128-byte lines)
  // Update step at the store (Algorithm 1: Update follows Aggregate): y = act(a + bias), or with W2
  // (kernels built with FUSE only) y = act(a W2 + bias) on the aggregated row a while it is still on chip
  const float* bias;  // [F], or [H2] with W2; null: none
  const float* W2;    // [F, H2] row-major; null: no fused dense layer
  int32_t H2;
  int32_t relu;
  SegTable segs;
};

// act(a + b) for the store: one fp32 addition (correctly rounded), then the activation
__device__ inline float update_bias_act(float a, const float* __restrict__ bias, int64_t col, int relu) {
  float y = bias ? a + bias[col] : a;
  return (relu && !(y > 0.0f)) ? 0.0f : y;
}

// float bits <-> integer key whose signed order is the float order with
// -0 below +0 (the map is its own inverse)
__device__ inline int32_t order_key(float f) {
  const int32_t b = __float_as_int(f);
  return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ inline float key_value(int32_t k) { return __int_as_float(k ^ ((k >> 31) & 0x7fffffff)); }

// Per-lane reduction state for VEC columns.  Sums accumulate in fp64: on this
// hardware the fp64 vector pipe runs at the same rate as unpacked fp32, the
// product of two fp32 values is exact in fp64, and a sum of 2^32 fp32 terms
// keeps ~20 guard bits, so the value rounded to fp32 at the end does not
// depend on the degree of the row or on how the row was split over lanes.
template <int OPK, int VEC>
struct State {
  double acc[VEC];
  __device__ inline void init() {
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = 0.0;
  }
  // MASKED: an entry that does not exist contributes an exact zero, whatever was read for it
  template <bool MASKED>
  __device__ inline void add(const float (&v)[VEC], float w, bool ok) {
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
      const double x = (double)((MASKED && !ok) ? 0.0f : v[k]);  // masked as a float: one select, not two
      if (OPK == OPK_WSUM) acc[k] = __builtin_fma((double)w, x, acc[k]);
      else acc[k] += x;
    }
  }
  __device__ inline void merge(const State& o) {
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] += o.acc[k];
  }
  __device__ inline State shuffled_xor(int stride) const {
    State o;
#pragma unroll
    for (int k = 0; k < VEC; ++k) o.acc[k] = __shfl_xor(acc[k], stride, kWave);
    return o;
  }
  __device__ inline void park(double* slot) const {
#pragma unroll
    for (int k = 0; k < VEC; ++k) slot[k] = acc[k];
  }
  __device__ inline void unpark(const double* slot) {
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = slot[k];
  }
  // the row's value: the mean divides by the degree, every other sum takes the row's factor (exact for 1)
  __device__ inline float result(int k, int64_t deg, bool mean, double scale) const {
    return (float)((mean && deg > 0) ? acc[k] / (double)deg : acc[k] * scale);
  }
  // partial result of one piece of a split row, one double per column
  __device__ inline void dump(double* p) const {
#pragma unroll
    for (int k = 0; k < VEC; ++k) p[k] = acc[k];
  }
  // a state that another pass left joins this one: earlier edges first, as in the row's own order.  The
  // states in transit are streamed (read once, written once): non-temporal, so that they do not push the
  // gathered rows out of L2.
  __device__ inline void fold_earlier(const double* p) {
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = __builtin_nontemporal_load(p + k) + acc[k];
  }
  __device__ inline void hand_on(double* p) const {
#pragma unroll
    for (int k = 0; k < VEC; ++k) __builtin_nontemporal_store(acc[k], p + k);
  }
};

// max: integer keys, exact and independent of the order of the operands
template <int VEC>
struct State<OPK_MAX, VEC> {
  int32_t key[VEC];
  __device__ inline void init() {
#pragma unroll
    for (int k = 0; k < VEC; ++k) key[k] = (int32_t)0x80000000;
  }
  template <bool MASKED>
  __device__ inline void add(const float (&v)[VEC], float, bool ok) {
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
      const int32_t b = (MASKED && !ok) ? (int32_t)0x80000000 : order_key(v[k]);
      key[k] = key[k] > b ? key[k] : b;
    }
  }
  __device__ inline void merge(const State& o) {
#pragma unroll
    for (int k = 0; k < VEC; ++k) key[k] = key[k] > o.key[k] ? key[k] : o.key[k];
  }
  __device__ inline State shuffled_xor(int stride) const {
    State o;
#pragma unroll
    for (int k = 0; k < VEC; ++k) o.key[k] = __shfl_xor(key[k], stride, kWave);
    return o;
  }
  __device__ inline void park(double* slot) const {
    int32_t* p = reinterpret_cast<int32_t*>(slot);
#pragma unroll
    for (int k = 0; k < VEC; ++k) p[k] = key[k];
  }
  __device__ inline void unpark(const double* slot) {
    const int32_t* p = reinterpret_cast<const int32_t*>(slot);
#pragma unroll
    for (int k = 0; k < VEC; ++k) key[k] = p[k];
  }
  __device__ inline float result(int k, int64_t deg, bool, double) const {
    return deg > 0 ? key_value(key[k]) : 0.0f;
  }
  __device__ inline void dump(double* p) const {  // an int32 key is exact in a double
#pragma unroll
    for (int k = 0; k < VEC; ++k) p[k] = (double)key[k];
  }
  __device__ inline void fold_earlier(const double* p) {
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
      const int32_t b = (int32_t)__builtin_nontemporal_load(p + k);
      key[k] = key[k] > b ? key[k] : b;
    }
  }
  __device__ inline void hand_on(double* p) const {
#pragma unroll
    for (int k = 0; k < VEC; ++k) __builtin_nontemporal_store((double)key[k], p + k);
  }
};

// Accumulator policy of the walk in gather.hpp: one 16-byte piece of the source row per edge.
// BITMASK: a missing entry is zeroed in the bits it was loaded as (sums only; the slices of 1 to 32 lanes,
// where every batch is masked), instead of by selects on the widened values (wave-wide slices, where only
// a row's last batch is masked and the selects are scalar-driven).
template <typename T, int OPK, int VEC, bool BITMASK>
struct AggAcc {
  static constexpr bool kWeighted = (OPK == OPK_WSUM);
  State<OPK, VEC> st;
  const char* __restrict__ xb;  // X plus this lane's column offset, in bytes
  int64_t rowbytes;
  typename Raw<T, VEC>::type raw[kUnroll];
  __device__ inline void fetch(int u, int32_t j) {
    // j is a vertex id (below 2^31) and the row pitch in bytes is below 2^32: one 32 x 32 -> 64 bit multiply-add
    raw[u] = load_raw<T, VEC>(reinterpret_cast<const T*>(xb + (uint64_t)(uint32_t)j * (uint64_t)(uint32_t)rowbytes));
  }
  __device__ inline void fetch_uniform(int u, int64_t j) {
    raw[u] = load_raw<T, VEC>(reinterpret_cast<const T*>(xb + j * rowbytes));
  }
  template <bool MASKED>
  __device__ inline void use(int u, float w, bool ok) {
    float v[VEC];
    if constexpr (MASKED && BITMASK && OPK != OPK_MAX) {
      // sums: a missing entry is zeroed in the bits it was loaded as, then takes the unmasked path
      unpack(and_bits(raw[u], keep_bits(ok)), v);
      st.template add<false>(v, w, true);
    } else {
      unpack(raw[u], v);
      st.template add<MASKED>(v, w, ok);
    }
  }
};

template <typename T, int OPK, int VEC, int MODE, bool FUSE>
__global__ __launch_bounds__(kBlock) void aggregate_kernel(const AggArgs a) {
  __shared__ double lds[(kWavesPerBlock - 1) * kWave * VEC];
  // FUSE: the aggregated rows of this workgroup (fp32, at most 256 lanes x VEC columns) and their row ids
  __shared__ float tile[FUSE ? kBlock * VEC : 1];
  __shared__ int32_t tile_row[FUSE ? kBlock : 1];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;

  const LaneRole role = lane_role(a.sl, a.segs, blockIdx.x, tid);
  const int g = role.g, col = role.col;
  const bool hub = role.hub, row_ok = role.row_ok, col_ok = role.col_ok;
  int64_t r = 0, e0 = 0, e1 = 0;
  if (row_ok) {
    r = a.order ? (int64_t)a.order[role.ridx] : role.ridx;
    e0 = (a.e_begin ? a.e_begin : a.rowptr)[r];
    e1 = (a.e_begin ? a.e_end : a.rowptr + 1)[r];
  }
  int64_t deg = e1 - e0;
  if (role.split_log2 > 0) {  // this workgroup walks one piece of the row
    e0 += (int64_t)role.piece << kSplitLenLog2;
    if (e0 > e1) e0 = e1;
    if (e1 - e0 > ((int64_t)1 << kSplitLenLog2)) e1 = e0 + ((int64_t)1 << kSplitLenLog2);
  }
  AggAcc<T, OPK, VEC, MODE != MODE_WAVE> acc;
  acc.st.init();
  // A later source block: the lane that will write the row starts from the state the earlier blocks left
  // (the other lanes of the row from nothing), so the read is in flight while the row is gathered and the
  // earlier edges still come first in the sum.  Pieces of split rows meet that state in the merge kernel.
  if (a.pin && role.writer && role.split_log2 == 0) acc.st.fold_earlier(a.pin + r * a.p_pitch + col);
  acc.xb = static_cast<const char*>(a.X) + (int64_t)col * (int64_t)sizeof(T);
  acc.rowbytes = a.x_pitch * (int64_t)sizeof(T);
  const int64_t nnz = (MODE == MODE_NARROW) ? a.rowptr[a.N] : 0;
  if constexpr (MODE == MODE_WIDE && kStageIndices) {
    __shared__ __attribute__((aligned(16))) int32_t stage[kWavesPerBlock * 2 * kWave];
    gather_row<MODE>(acc, a.colidx, a.edge_w, e0, e1, role.ng, g, role.L, col_ok, lane, nnz, stage + wv * 2 * kWave);
  } else {
    gather_row<MODE>(acc, a.colidx, a.edge_w, e0, e1, role.ng, g, role.L, col_ok, lane, nnz);
  }
  State<OPK, VEC>& st = acc.st;

  // ---- merge the neighbour slots of a row -------------------------------------
  const int lanes_in_wave = hub ? kWave : (1 << role.L);
  for (int stride = 1 << g; stride < lanes_in_wave; stride <<= 1) st.merge(st.shuffled_xor(stride));
  if (hub) {
    // lanes [0, 2^g) of each wave now hold that wave's partial for their columns (if 2^g < 64);
    // waves 1..3 park theirs in LDS, wave 0 folds them in wave order
    if (wv > 0) st.park(lds + ((wv - 1) * kWave + lane) * VEC);
    __syncthreads();
    if (wv == 0) {
      for (int ww = 1; ww < kWavesPerBlock; ++ww) {
        State<OPK, VEC> o;
        o.unpark(lds + ((ww - 1) * kWave + lane) * VEC);
        st.merge(o);
      }
    }
  }

  // ---- write the slice of the output row ----------------------------------------
  if (role.writer && role.split_log2 > 0) {
    st.dump(a.ws + (int64_t)role.ws_slot * a.F + col);
  } else if (role.writer && a.pout) {
    // a source block that is not the last: hand the state on instead of finishing the row
    st.hand_on(a.pout + r * a.p_pitch + col);
  } else if (role.writer) {
    if (a.e_begin) deg = a.rowptr[r + 1] - a.rowptr[r];  // source blocks: the row's whole degree finishes it
    const double scale = a.row_scale ? (double)a.row_scale[r] : 1.0;
    float res[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) res[k] = st.result(k, deg, a.mean != 0, scale);
    if constexpr (FUSE) {
      // one slice, one chunk, columns [0, F): park the row for the dense layer below
      const int lrow = hub ? 0 : (wv << (6 - role.L)) + (lane >> role.L);
#pragma unroll
      for (int k = 0; k < VEC; ++k) tile[lrow * (int)a.F + col + k] = res[k];
    } else {
      if (a.bias || a.relu) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) res[k] = update_bias_act(res[k], a.bias, col + k, a.relu);
      }
      if (a.out_bf16) store_row_bf16<VEC>(static_cast<uint16_t*>(a.out) + r * a.out_pitch + col, res);
      else store_row<VEC>(static_cast<float*>(a.out) + r * a.out_pitch + col, res);
    }
  }
  if constexpr (FUSE) {
    // y[h] = act(sum_f a[f] W2[f, h] + bias[h]) for the rows parked above: fp64 FMAs in column order,
    // one rounding; thread t takes (row t / H2, column t % H2), so W2 and out are read and written in runs
    if (role.split_log2 > 0) return;  // pieces of a split row: the merge kernel finishes the row
    const int rows_here = hub ? 1 : (kWavesPerBlock << (6 - role.L));
    if (role.ng == 0 && col == 0 && col_ok) {
      const int lrow = hub ? 0 : (wv << (6 - role.L)) + (lane >> role.L);
      tile_row[lrow] = row_ok ? (int32_t)r : -1;
    }
    __syncthreads();
    const int F = (int)a.F, H2 = a.H2;
    for (int t = tid; t < rows_here * H2; t += kBlock) {
      const int lrow = t / H2, h = t - lrow * H2;
      const int64_t rr = tile_row[lrow];
      if (rr < 0) continue;
      double y = 0.0;
      for (int f = 0; f < F; ++f) y = __builtin_fma((double)tile[lrow * F + f], (double)a.W2[f * H2 + h], y);
      if (a.bias) y += (double)a.bias[h];  // like gnnagg_combine: bias joins the fp64 sum, one rounding
      const float res = update_bias_act((float)y, nullptr, h, a.relu);
      if (a.out_bf16) static_cast<uint16_t*>(a.out)[rr * a.out_pitch + h] = (uint16_t)bf16_bits(res);
      else static_cast<float*>(a.out)[rr * a.out_pitch + h] = res;
    }
  }
}

// Folds the pieces of the split rows, in piece order, into `out`: one thread per (split row, column).
struct MergeArgs {
  const int64_t* rowptr;
  const int32_t* order;
  void* out;
  const double* ws;
  int64_t F, out_pitch;
  int64_t rows;  // split rows in all runs together
  int32_t out_bf16, mean, nrun;
  const float* row_scale;  // as in AggArgs
  const float* bias;       // the Update step, as in AggArgs
  const float* W2;
  int32_t H2, relu;
  const double* pin;  // source blocks, as in AggArgs (rowptr is the whole graph's: it gives the degree)
  double* pout;
  int64_t p_pitch;
  Seg run[kMaxSplitSeg];
};

template <int OPK>
__global__ __launch_bounds__(kBlock) void split_merge_kernel(const MergeArgs a) {
  const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (t >= a.rows * a.F) return;
  int64_t i = t / a.F;  // which split row, counted over the runs
  const int64_t col = t - i * a.F;
  int k = 0;
  while (k + 1 < a.nrun && i >= (int64_t)a.run[k].row_end - a.run[k].row_begin) {
    i -= (int64_t)a.run[k].row_end - a.run[k].row_begin;
    ++k;
  }
  const Seg run = a.run[k];
  const int64_t r = a.order[run.row_begin + i];
  const int64_t deg = a.rowptr[r + 1] - a.rowptr[r];
  const int64_t pieces = (int64_t)1 << run.split_log2;
  const double* p = a.ws + ((int64_t)run.ws_begin + i * pieces) * a.F + col;
  State<OPK, 1> st;
  st.init();
  for (int64_t q = 0; q < pieces; ++q) {
    State<OPK, 1> o;
    if constexpr (OPK == OPK_MAX) o.key[0] = (int32_t)p[q * a.F];
    else o.acc[0] = p[q * a.F];
    st.merge(o);
  }
  if (a.pin) st.fold_earlier(a.pin + r * a.p_pitch + col);
  if (a.pout) {
    st.hand_on(a.pout + r * a.p_pitch + col);
    return;
  }
  const double scale = a.row_scale ? (double)a.row_scale[r] : 1.0;
  const float res = update_bias_act(st.result(0, deg, a.mean != 0, scale), a.bias, col, a.relu);
  if (a.out_bf16) static_cast<uint16_t*>(a.out)[r * a.out_pitch + col] = (uint16_t)bf16_bits(res);
  else static_cast<float*>(a.out)[r * a.out_pitch + col] = res;
}

// The same for a call with a fused dense layer: one thread per (split row, output column h) folds the
// pieces of every input column in piece order, rounds the aggregate to fp32 and contracts it with W2.
template <int OPK>
__global__ __launch_bounds__(kBlock) void split_merge_fused_kernel(const MergeArgs a) {
  const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (t >= a.rows * a.H2) return;
  int64_t i = t / a.H2;
  const int64_t h = t - i * a.H2;
  int k = 0;
  while (k + 1 < a.nrun && i >= (int64_t)a.run[k].row_end - a.run[k].row_begin) {
    i -= (int64_t)a.run[k].row_end - a.run[k].row_begin;
    ++k;
  }
  const Seg run = a.run[k];
  const int64_t r = a.order[run.row_begin + i];
  const int64_t deg = a.rowptr[r + 1] - a.rowptr[r];
  const int64_t pieces = (int64_t)1 << run.split_log2;
  const double* p = a.ws + ((int64_t)run.ws_begin + i * pieces) * a.F;
  const double scale = a.row_scale ? (double)a.row_scale[r] : 1.0;
  double y = 0.0;
  for (int64_t f = 0; f < a.F; ++f) {
    State<OPK, 1> st;
    st.init();
    for (int64_t q = 0; q < pieces; ++q) {
      State<OPK, 1> o;
      if constexpr (OPK == OPK_MAX) o.key[0] = (int32_t)p[q * a.F + f];
      else o.acc[0] = p[q * a.F + f];
      st.merge(o);
    }
    y = __builtin_fma((double)st.result(0, deg, a.mean != 0, scale), (double)a.W2[f * a.H2 + h], y);
  }
  if (a.bias) y += (double)a.bias[h];
  const float res = update_bias_act((float)y, nullptr, h, a.relu);
  if (a.out_bf16) static_cast<uint16_t*>(a.out)[r * a.out_pitch + h] = (uint16_t)bf16_bits(res);
  else static_cast<float*>(a.out)[r * a.out_pitch + h] = res;
}

template <typename T, int OPK, int VEC, int MODE, bool FUSE>
int launch_fused_or_not(const AggArgs& a, uint64_t grid, hipStream_t stream) {
  // Unused dynamic LDS is how the number of resident workgroups per compute unit is capped (see
  // resident_workgroup_cap): a workgroup that claims 1/k of the LDS leaves room for k of them.
  const size_t static_lds = sizeof(double) * (kWavesPerBlock - 1) * kWave * VEC;
  const size_t dyn_lds = a.lds_per_workgroup > static_lds ? a.lds_per_workgroup - static_lds : 0;
  hipLaunchKernelGGL((aggregate_kernel<T, OPK, VEC, MODE, FUSE>), dim3((unsigned)grid), dim3(kBlock), dyn_lds, stream,
                     a);
  return hipGetLastError() == hipSuccess ? GNNAGG_OK : GNNAGG_EDEVICE;
}

// A fused dense layer needs the whole aggregated row in one workgroup: rows of at most 64 columns, i.e.
// slices of at most 16 lanes - never the wave-wide kernel.
template <typename T, int OPK, int VEC, int MODE>
int launch_one(const AggArgs& a, uint64_t grid, hipStream_t stream) {
  if constexpr (MODE != MODE_WAVE) {
    if (a.W2) return launch_fused_or_not<T, OPK, VEC, MODE, true>(a, grid, stream);
  } else {
    if (a.W2) return GNNAGG_EUNSUPPORTED;
  }
  return launch_fused_or_not<T, OPK, VEC, MODE, false>(a, grid, stream);
}

// Slices wider than four lanes only occur with the widest per-lane vector (16 bytes of input), so the
// wave and wide kernels exist for that vector width only; narrow slices come in every width.
template <typename T, int OPK>
int launch_vec(const AggArgs& a, uint64_t grid, hipStream_t stream) {
  constexpr int kMaxVec = 16 / (int)sizeof(T);
  if (a.sl.g_log2 >= 3) {
    if (a.sl.vec != kMaxVec) return GNNAGG_EINVAL;
    return a.sl.g_log2 == 6 ? launch_one<T, OPK, kMaxVec, MODE_WAVE>(a, grid, stream)
                            : launch_one<T, OPK, kMaxVec, MODE_WIDE>(a, grid, stream);
  }
  switch (a.sl.vec) {
    case 1: return launch_one<T, OPK, 1, MODE_NARROW>(a, grid, stream);
    case 2: return launch_one<T, OPK, 2, MODE_NARROW>(a, grid, stream);
    case 4: return launch_one<T, OPK, 4, MODE_NARROW>(a, grid, stream);
    case 8:
      if constexpr (sizeof(T) == 2) return launch_one<T, OPK, 8, MODE_NARROW>(a, grid, stream);
      return GNNAGG_EINVAL;
    default: return GNNAGG_EINVAL;
  }
}

template <typename T>
int launch_op(int opk, const AggArgs& a, uint64_t grid, hipStream_t stream) {
  switch (opk) {
    case OPK_SUM: return launch_vec<T, OPK_SUM>(a, grid, stream);
    case OPK_WSUM: return launch_vec<T, OPK_WSUM>(a, grid, stream);
    default: return launch_vec<T, OPK_MAX>(a, grid, stream);
  }
}

}  // namespace
}  // namespace gnnagg

using namespace gnnagg;

// Scratch of gnnagg_aggregate_noalloc: the partial results of split rows, for callers that cannot hand
// over a workspace of their own.  One copy per GPU, at an address of its own on each; host code reaches
// it only through the pointer hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) unsigned char scratch[GNNAGG_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_of_device[kMaxDevices];  // device address of `scratch` per GPU, looked up on first use

int scratch_for_current_device(void** p) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GNNAGG_EDEVICE;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_of_device[dev]) {
    void* q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return GNNAGG_EDEVICE;
    scratch_of_device[dev] = q;
  }
  *p = scratch_of_device[dev];
  return GNNAGG_OK;
}

// Measurement override of the resident-workgroup cap (gnnagg_set_workgroup_cap): -1 = the library's rule.
std::atomic<int> forced_workgroup_cap{-1};

// One source block of a blocked call (all null: a plain call).  pin and pout must not be the same array:
// lanes that re-read a slice's last columns store the same element twice.
struct Block {
  const int64_t* e_begin = nullptr;
  const int64_t* e_end = nullptr;
  const double* pin = nullptr;
  double* pout = nullptr;
  int64_t p_pitch = 0;
};

// The Update step of a call (all null / zero: none).
struct Update {
  const float* bias = nullptr;
  const float* W2 = nullptr;
  int32_t H2 = 0;
  int32_t relu = 0;
};

// Argument checks shared by the aggregation entry points; GNNAGG_OK with *nothing = true means
// there is nothing to do.
int check_aggregate_args(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx, const float* edge_w,
                         const void* X, int x_dtype, void* out, int out_dtype, int32_t F, int32_t f_chunk,
                         const int32_t* row_order, const int64_t* class_off, bool* nothing) {
  *nothing = false;
  if (op < GNNAGG_SUM || op > GNNAGG_SUM_SCALED) return GNNAGG_EINVAL;
  if (N < 0 || F <= 0 || f_chunk < GNNAGG_F_CHUNK_AUTO) return GNNAGG_EINVAL;
  if (x_dtype != GNNAGG_F32 && x_dtype != GNNAGG_BF16) return GNNAGG_EINVAL;
  if (out_dtype != GNNAGG_F32 && out_dtype != GNNAGG_BF16) return GNNAGG_EINVAL;
  if (N >= (1ll << 31)) return GNNAGG_EUNSUPPORTED;
  if ((row_order == nullptr) != (class_off == nullptr)) return GNNAGG_EINVAL;
  if (N == 0) {
    *nothing = true;
    return GNNAGG_OK;
  }
  if (!rowptr || !X || !out) return GNNAGG_ENULL;
  if ((op == GNNAGG_WSUM || op == GNNAGG_SUM_SCALED) && !edge_w) return GNNAGG_ENULL;
  // colidx may only be NULL for a graph without edges, which the host cannot see; require it
  if (!colidx) return GNNAGG_ENULL;
  const size_t xs = (x_dtype == GNNAGG_F32) ? 4 : 2;
  if (((uintptr_t)X % xs) || ((uintptr_t)out % (out_dtype == GNNAGG_F32 ? 4 : 2)) || ((uintptr_t)rowptr % 8) ||
      ((uintptr_t)colidx % 4) || (edge_w && ((uintptr_t)edge_w % 4)))
    return GNNAGG_EINVAL;
  if (X == out) return GNNAGG_EINVAL;
  return GNNAGG_OK;
}

// Pitches and plan of the calls that take them; the workspace size a plan asks for (0: no row is split).
int check_pitches_and_plan(int64_t N, int32_t F, int32_t out_cols, int64_t* x_pitch, int64_t* out_pitch,
                           const int32_t* row_order, const int64_t* class_off, size_t* need) {
  if (N < 0 || F <= 0 || out_cols <= 0) return GNNAGG_EINVAL;
  if (*x_pitch == 0) *x_pitch = F;
  if (*out_pitch == 0) *out_pitch = out_cols;
  if (*x_pitch < F || *out_pitch < out_cols || *x_pitch > (1ll << 40) || *out_pitch > (1ll << 40))
    return GNNAGG_EINVAL;
  if ((row_order == nullptr) != (class_off == nullptr)) return GNNAGG_EINVAL;
  if (N >= (1ll << 31)) return GNNAGG_EUNSUPPORTED;
  SegTable probe;
  int rc = build_segments(class_off, N, 6, true, &probe);  // the split runs do not depend on the slice width
  if (rc != GNNAGG_OK) return rc;
  *need = (size_t)probe.ws_slots * (size_t)F * sizeof(double);
  return GNNAGG_OK;
}

// ws == nullptr: no row is split.  Otherwise ws holds segs.ws_slots * F doubles.  Everything a call
// needs on the host lives on the stack: nothing is allocated, on the host or on the device.
int aggregate_impl(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx, const float* edge_w,
                   const void* X, int x_dtype, int64_t x_pitch, void* out, int out_dtype, int64_t out_pitch,
                   int32_t F, int32_t f_chunk, const int32_t* row_order, const int64_t* class_off, double* ws,
                   const Update& up, hipStream_t stream, const Block& blk = Block()) {
  const size_t xs = (x_dtype == GNNAGG_F32) ? 4 : 2;
  if ((uint64_t)x_pitch * xs >= (1ull << 32)) return GNNAGG_EUNSUPPORTED;  // row addresses: 32 x 32 -> 64 bit
  const bool rows_on_lines = ((uintptr_t)X % 128) == 0 && ((uint64_t)x_pitch * xs) % 128 == 0;
  if (up.W2 && blk.e_begin) return GNNAGG_EUNSUPPORTED;
  if (up.W2) f_chunk = 0;  // the dense layer contracts whole rows
  if (f_chunk == GNNAGG_F_CHUNK_AUTO) f_chunk = auto_f_chunk(N, F, (int)xs, rows_on_lines, class_off);
  LaunchList launches;
  const bool capped = resident_workgroup_cap(class_off, N, 6, kWave, true) > 0;  // dense graph: caps in play
  plan_columns(F, f_chunk, (int)(16 / xs), 0, rows_on_lines ? (int)(128 / xs) : 0, capped, &launches);
  if (launches.overflow || launches.empty()) return GNNAGG_EUNSUPPORTED;
  if (up.W2 && (launches.size() != 1 || launches[0].n_sub != 1 || launches[0].n_chunks != 1 ||
                launches[0].g_log2 > 4))
    return GNNAGG_EUNSUPPORTED;  // cannot happen for F <= 64
  const int opk = (op == GNNAGG_WSUM) ? OPK_WSUM : (op == GNNAGG_MAX ? OPK_MAX : OPK_SUM);
  // a sum with factors per destination: the edge_w argument holds N factors, and no edge has a weight
  const float* row_scale = nullptr;
  if (op == GNNAGG_SUM_SCALED) {
    row_scale = edge_w;
    edge_w = nullptr;
  }

  // build and validate every launch before the first one is enqueued
  AggArgs args[kMaxLaunches];
  uint64_t grids[kMaxLaunches];
  for (size_t k = 0; k < launches.size(); ++k) {
    AggArgs& a = args[k];
    a.rowptr = rowptr;
    a.colidx = colidx;
    a.edge_w = edge_w;
    a.row_scale = row_scale;
    a.X = X;
    a.out = out;
    a.out_bf16 = (out_dtype == GNNAGG_BF16);
    a.order = row_order;
    a.F = F;
    a.x_pitch = x_pitch;
    a.out_pitch = out_pitch;
    a.N = N;
    a.sl = launches[k];
    a.mean = (op == GNNAGG_MEAN);
    a.ws = ws;
    a.e_begin = blk.e_begin;
    a.e_end = blk.e_end;
    a.pin = blk.pin;
    a.pout = blk.pout;
    a.p_pitch = blk.p_pitch;
    a.bias = up.bias;
    a.W2 = up.W2;
    a.H2 = up.H2;
    a.relu = up.relu;
    const int forced = forced_workgroup_cap.load(std::memory_order_relaxed);
    a.lds_per_workgroup = lds_claim(forced >= 0 ? forced
                                                : resident_workgroup_cap(class_off, N, a.sl.g_log2,
                                                                         active_lanes_per_wave(a.sl), opk == OPK_WSUM));
    int rc = build_segments(class_off, N, a.sl.g_log2, ws != nullptr, &a.segs);
    if (rc != GNNAGG_OK) return rc;
    grids[k] = (uint64_t)a.segs.blocks_per_slice * (uint64_t)a.sl.n_chunks * (uint64_t)a.sl.n_sub;
    if (grids[k] == 0 || grids[k] > 0x7fffffffull) return GNNAGG_EUNSUPPORTED;
  }
  for (size_t k = 0; k < launches.size(); ++k) {
    int rc = (x_dtype == GNNAGG_F32) ? launch_op<float>(opk, args[k], grids[k], stream)
                                     : launch_op<bf16_t>(opk, args[k], grids[k], stream);
    if (rc != GNNAGG_OK) return rc;
  }
  if (ws && args[0].segs.ws_slots > 0) {
    // the split runs are the same in every launch: they depend on the degree classes only
    MergeArgs m;
    m.rowptr = rowptr;
    m.order = row_order;
    m.out = out;
    m.ws = ws;
    m.F = F;
    m.out_pitch = out_pitch;
    m.out_bf16 = (out_dtype == GNNAGG_BF16);
    m.mean = (op == GNNAGG_MEAN);
    m.row_scale = row_scale;
    m.bias = up.bias;
    m.W2 = up.W2;
    m.H2 = up.H2;
    m.relu = up.relu;
    m.pin = blk.pin;
    m.pout = blk.pout;
    m.p_pitch = blk.p_pitch;
    m.nrun = 0;
    m.rows = 0;
    const SegTable& st = args[0].segs;
    for (int k = 0; k < st.nseg; ++k) {
      if (st.seg[k].split_log2 == 0) continue;
      if (m.nrun >= kMaxSplitSeg) return GNNAGG_EUNSUPPORTED;  // cannot happen: build_segments caps them
      m.run[m.nrun++] = st.seg[k];
      m.rows += (int64_t)st.seg[k].row_end - st.seg[k].row_begin;
    }
    const int64_t blocks = ceil_div(m.rows * (int64_t)(up.W2 ? up.H2 : F), kBlock);
    if (blocks > 0x7fffffffll) return GNNAGG_EUNSUPPORTED;
    const dim3 grid((unsigned)blocks), block(kBlock);
    if (up.W2) {
      if (opk == OPK_MAX) hipLaunchKernelGGL(split_merge_fused_kernel<OPK_MAX>, grid, block, 0, stream, m);
      else hipLaunchKernelGGL(split_merge_fused_kernel<OPK_SUM>, grid, block, 0, stream, m);
    } else {
      if (opk == OPK_MAX) hipLaunchKernelGGL(split_merge_kernel<OPK_MAX>, grid, block, 0, stream, m);
      else hipLaunchKernelGGL(split_merge_kernel<OPK_SUM>, grid, block, 0, stream, m);
    }
    if (hipGetLastError() != hipSuccess) return GNNAGG_EDEVICE;
  }
  return GNNAGG_OK;
}

}  // namespace

extern "C" int gnnagg_aggregate(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                                const float* edge_w, const void* X, int x_dtype, void* out, int out_dtype,
                                int32_t F, int32_t f_chunk, const int32_t* row_order, const int64_t* class_off,
                                void* stream_) {
  bool nothing;
  int rc = check_aggregate_args(op, N, rowptr, colidx, edge_w, X, x_dtype, out, out_dtype, F, f_chunk, row_order,
                                class_off, &nothing);
  if (rc != GNNAGG_OK || nothing) return rc;
  return aggregate_impl(op, N, rowptr, colidx, edge_w, X, x_dtype, F, out, out_dtype, F, F, f_chunk, row_order,
                        class_off, nullptr, Update(), (hipStream_t)stream_);
}

extern "C" int gnnagg_aggregate_ws(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                                   const float* edge_w, const void* X, int x_dtype, int64_t x_pitch, void* out,
                                   int out_dtype, int64_t out_pitch, int32_t F, int32_t f_chunk,
                                   const int32_t* row_order, const int64_t* class_off, void* workspace,
                                   size_t* workspace_bytes, void* stream_) {
  if (!workspace_bytes) return GNNAGG_ENULL;
  size_t need = 0;
  int rc = check_pitches_and_plan(N, F, F, &x_pitch, &out_pitch, row_order, class_off, &need);
  if (rc != GNNAGG_OK) return rc;
  if (!workspace) {
    *workspace_bytes = need;
    return GNNAGG_OK;
  }
  if (*workspace_bytes < need || ((uintptr_t)workspace & 255u)) return GNNAGG_EWORKSPACE;
  bool nothing;
  rc = check_aggregate_args(op, N, rowptr, colidx, edge_w, X, x_dtype, out, out_dtype, F, f_chunk, row_order,
                            class_off, &nothing);
  if (rc != GNNAGG_OK || nothing) return rc;
  return aggregate_impl(op, N, rowptr, colidx, edge_w, X, x_dtype, x_pitch, out, out_dtype, out_pitch, F, f_chunk,
                        row_order, class_off, need > 0 ? static_cast<double*>(workspace) : nullptr, Update(),
                        (hipStream_t)stream_);
}

extern "C" int gnnagg_aggregate_update(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                                       const float* edge_w, const void* X, int x_dtype, int64_t x_pitch,
                                       int32_t F, int32_t f_chunk, const float* W2, int32_t H2, const float* bias,
                                       int relu, void* out, int out_dtype, int64_t out_pitch,
                                       const int32_t* row_order, const int64_t* class_off, void* workspace,
                                       size_t* workspace_bytes, void* stream_) {
  if (!workspace_bytes) return GNNAGG_ENULL;
  if (relu != 0 && relu != 1) return GNNAGG_EINVAL;
  if (W2 ? (H2 <= 0 || H2 > GNNAGG_FUSED_MAX_COLS) : (H2 != 0)) return GNNAGG_EINVAL;
  if (W2 && F > 0 && F > GNNAGG_FUSED_MAX_ROW) return GNNAGG_EUNSUPPORTED;
  if (W2 && f_chunk > 0 && f_chunk < F) return GNNAGG_EINVAL;  // the dense layer contracts whole rows
  size_t need = 0;
  int rc = check_pitches_and_plan(N, F, W2 ? H2 : F, &x_pitch, &out_pitch, row_order, class_off, &need);
  if (rc != GNNAGG_OK) return rc;
  if (!workspace) {
    *workspace_bytes = need;
    return GNNAGG_OK;
  }
  if (*workspace_bytes < need || ((uintptr_t)workspace & 255u)) return GNNAGG_EWORKSPACE;
  bool nothing;
  rc = check_aggregate_args(op, N, rowptr, colidx, edge_w, X, x_dtype, out, out_dtype, F, f_chunk, row_order,
                            class_off, &nothing);
  if (rc != GNNAGG_OK || nothing) return rc;
  if ((W2 && ((uintptr_t)W2 % 4)) || (bias && ((uintptr_t)bias % 4))) return GNNAGG_EINVAL;
  Update up;
  up.bias = bias;
  up.W2 = W2;
  up.H2 = W2 ? H2 : 0;
  up.relu = relu;
  return aggregate_impl(op, N, rowptr, colidx, edge_w, X, x_dtype, x_pitch, out, out_dtype, out_pitch, F, f_chunk,
                        row_order, class_off, need > 0 ? static_cast<double*>(workspace) : nullptr, up,
                        (hipStream_t)stream_);
}

extern "C" int gnnagg_aggregate_noalloc(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                                        const float* edge_w, const void* X, int x_dtype, int64_t x_pitch,
                                        void* out, int out_dtype, int64_t out_pitch, int32_t F, int32_t f_chunk,
                                        const int32_t* row_order, const int64_t* class_off, void* stream_) {
  size_t need = 0;
  int rc = check_pitches_and_plan(N, F, F, &x_pitch, &out_pitch, row_order, class_off, &need);
  if (rc != GNNAGG_OK) return rc;
  if (need > (size_t)GNNAGG_NOALLOC_SCRATCH_BYTES) return GNNAGG_EWORKSPACE;  // the plan's split rows do not fit
  bool nothing;
  rc = check_aggregate_args(op, N, rowptr, colidx, edge_w, X, x_dtype, out, out_dtype, F, f_chunk, row_order,
                            class_off, &nothing);
  if (rc != GNNAGG_OK || nothing) return rc;
  void* ws = nullptr;
  if (need > 0) {
    rc = scratch_for_current_device(&ws);
    if (rc != GNNAGG_OK) return rc;
  }
  // every slot a piece owns is written in full before the merge kernel reads it: nothing to clear
  return aggregate_impl(op, N, rowptr, colidx, edge_w, X, x_dtype, x_pitch, out, out_dtype, out_pitch, F, f_chunk,
                        row_order, class_off, static_cast<double*>(ws), Update(), (hipStream_t)stream_);
}

namespace {

// gnnagg_aggregate_blocked after its argument checks: f_chunk resolved, workspace carved.
struct BlockedCall {
  int op;
  int64_t N;
  const int64_t* rowptr;
  const int32_t* colidx;
  const float* edge_w;
  const void* X;
  int x_dtype;
  int64_t x_pitch;
  void* out;
  int out_dtype;
  int64_t out_pitch;
  int32_t F, B;
  const int64_t* block_ptr;
  const int32_t* row_order;
  const int64_t* class_off;
  double* state[2];
  double* ws;
  int64_t p_pitch;
};

int run_blocked(const BlockedCall& c, int32_t f_chunk, hipStream_t stream) {
  constexpr int kOffs = GNNAGG_PLAN_CLASSES + 1;
  for (int32_t b = 0; b < c.B; ++b) {
    Block blk;
    blk.e_begin = c.block_ptr + (int64_t)b * c.N;
    blk.e_end = c.block_ptr + (int64_t)(b + 1) * c.N;
    blk.pin = b > 0 ? c.state[(b - 1) & 1] : nullptr;
    blk.pout = b + 1 < c.B ? c.state[b & 1] : nullptr;
    blk.p_pitch = c.p_pitch;
    int rc = aggregate_impl(c.op, c.N, c.rowptr, c.colidx, c.edge_w, c.X, c.x_dtype, c.x_pitch, c.out, c.out_dtype,
                            c.out_pitch, c.F, f_chunk, c.row_order + (int64_t)b * c.N,
                            c.class_off + (size_t)b * kOffs, c.ws, Update(), stream, blk);
    if (rc != GNNAGG_OK) return rc;
  }
  return GNNAGG_OK;
}

// Checks and workspace protocol shared by gnnagg_aggregate_blocked and gnnagg_tune_blocked.  GNNAGG_OK with
// *done = true: the call is complete (size query answered, or nothing to do).
int prepare_blocked(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx, const float* edge_w,
                    const void* X, int x_dtype, int64_t x_pitch, void* out, int out_dtype, int64_t out_pitch,
                    int32_t F, int32_t f_chunk, int32_t B, const int64_t* block_ptr, const int32_t* row_order,
                    const int64_t* class_off, void* workspace, size_t* workspace_bytes, BlockedCall* c, bool* done) {
  *done = false;
  if (!workspace_bytes) return GNNAGG_ENULL;
  if (B < 1 || B > GNNAGG_MAX_SOURCE_BLOCKS) return GNNAGG_EINVAL;
  if (!class_off || !row_order || (N > 0 && !block_ptr)) return GNNAGG_ENULL;
  constexpr int kOffs = GNNAGG_PLAN_CLASSES + 1;
  size_t need_split = 0;
  for (int32_t b = 0; b < B; ++b) {  // the blocks run one after another and share the split rows' slots
    size_t need_b = 0;
    int rc = check_pitches_and_plan(N, F, F, &x_pitch, &out_pitch, row_order, class_off + (size_t)b * kOffs, &need_b);
    if (rc != GNNAGG_OK) return rc;
    if (need_b > need_split) need_split = need_b;
  }
  const int64_t p_pitch = ceil_div(F, 16) * 16;  // rows of the states in transit start on 128-byte lines
  const size_t state_bytes = align_up((size_t)N * (size_t)p_pitch * sizeof(double));
  const int n_state = B - 1 < 2 ? B - 1 : 2;
  const size_t need = (size_t)n_state * state_bytes + need_split;
  if (!workspace) {
    *workspace_bytes = need;
    *done = true;
    return GNNAGG_OK;
  }
  if (*workspace_bytes < need || ((uintptr_t)workspace & 255u)) return GNNAGG_EWORKSPACE;
  bool nothing;
  int rc = check_aggregate_args(op, N, rowptr, colidx, edge_w, X, x_dtype, out, out_dtype, F, f_chunk, row_order,
                                class_off, &nothing);
  if (rc != GNNAGG_OK) return rc;
  if (nothing) {
    *done = true;
    return GNNAGG_OK;
  }
  if ((uintptr_t)block_ptr % 8) return GNNAGG_EINVAL;
  char* base = static_cast<char*>(workspace);
  *c = BlockedCall{op, N, rowptr, colidx, edge_w, X, x_dtype, x_pitch, out, out_dtype, out_pitch, F, B, block_ptr,
                   row_order, class_off,
                   {reinterpret_cast<double*>(base), reinterpret_cast<double*>(base + state_bytes)},
                   need_split > 0 ? reinterpret_cast<double*>(base + (size_t)n_state * state_bytes) : nullptr, p_pitch};
  return GNNAGG_OK;
}

// Row pieces of two lines when the rows of X start on lines and are at least two pieces long, else one chunk.
int32_t blocked_auto_f_chunk(const void* X, int x_dtype, int64_t x_pitch, int32_t F) {
  const int64_t xs = (x_dtype == GNNAGG_F32) ? 4 : 2;
  const bool rows_on_lines = ((uintptr_t)X % 128) == 0 && ((uint64_t)x_pitch * (uint64_t)xs) % 128 == 0;
  const int32_t piece = (x_dtype == GNNAGG_F32) ? 64 : 128;
  return (rows_on_lines && F >= 2 * piece) ? piece : 0;
}

}  // namespace

extern "C" int gnnagg_aggregate_blocked(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                                        const float* edge_w, const void* X, int x_dtype, int64_t x_pitch,
                                        void* out, int out_dtype, int64_t out_pitch, int32_t F, int32_t f_chunk,
                                        int32_t B, const int64_t* block_ptr, const int32_t* row_order,
                                        const int64_t* class_off, void* workspace, size_t* workspace_bytes,
                                        void* stream_) {
  BlockedCall c;
  bool done;
  int rc = prepare_blocked(op, N, rowptr, colidx, edge_w, X, x_dtype, x_pitch, out, out_dtype, out_pitch, F, f_chunk,
                           B, block_ptr, row_order, class_off, workspace, workspace_bytes, &c, &done);
  if (rc != GNNAGG_OK || done) return rc;
  if (f_chunk == GNNAGG_F_CHUNK_AUTO) f_chunk = blocked_auto_f_chunk(c.X, c.x_dtype, c.x_pitch, F);
  return run_blocked(c, f_chunk, (hipStream_t)stream_);
}

extern "C" int gnnagg_tune_blocked(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                                   const float* edge_w, const void* X, int x_dtype, int64_t x_pitch, void* out,
                                   int out_dtype, int64_t out_pitch, int32_t F, int32_t B, const int64_t* block_ptr,
                                   const int32_t* row_order, const int64_t* class_off, void* workspace,
                                   size_t* workspace_bytes, void* stream_, int32_t* best_f_chunk, float* best_ms) {
  BlockedCall c;
  bool done;
  int rc = prepare_blocked(op, N, rowptr, colidx, edge_w, X, x_dtype, x_pitch, out, out_dtype, out_pitch, F, 0, B,
                           block_ptr, row_order, class_off, workspace, workspace_bytes, &c, &done);
  if (rc != GNNAGG_OK) return rc;
  if (done && !workspace) return GNNAGG_OK;  // size query
  if (!best_f_chunk) return GNNAGG_ENULL;
  if (done) {
    *best_f_chunk = F;
    if (best_ms) *best_ms = 0.0f;
    return GNNAGG_OK;
  }
  hipStream_t stream = (hipStream_t)stream_;
  // candidates: the blocked call's own choice and row pieces of 1, 2 and 4 lines
  const int32_t line_cols = (x_dtype == GNNAGG_F32) ? 32 : 64;
  int32_t cand[4];
  int n_cand = 0;
  auto add = [&](int32_t w) {
    if (w <= 0 || w >= F) w = F;
    for (int k = 0; k < n_cand; ++k)
      if (cand[k] == w) return;
    cand[n_cand++] = w;
  };
  add(blocked_auto_f_chunk(c.X, c.x_dtype, c.x_pitch, F));
  for (int32_t lines = 1; lines <= 4; lines *= 2) add(lines * line_cols);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return GNNAGG_EDEVICE;
  if (hipEventCreate(&e1) != hipSuccess) {
    (void)hipEventDestroy(e0);
    return GNNAGG_EDEVICE;
  }
  constexpr int kTimedCalls = 3;
  float best = 0.0f;
  int32_t best_w = cand[0];
  for (int k = 0; k < n_cand && rc == GNNAGG_OK; ++k) {
    float ms = 0.0f;
    for (int rep = 0; rep <= kTimedCalls && rc == GNNAGG_OK; ++rep) {  // call 0 warms caches and code
      if (rep == 1 && hipEventRecord(e0, stream) != hipSuccess) rc = GNNAGG_EDEVICE;
      if (rc == GNNAGG_OK) rc = run_blocked(c, cand[k], stream);
    }
    if (rc == GNNAGG_OK && (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                            hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
      rc = GNNAGG_EDEVICE;
    if (rc == GNNAGG_OK && (k == 0 || ms < best)) {
      best = ms;
      best_w = cand[k];
    }
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != GNNAGG_OK) return rc;
  if (hipStreamSynchronize(stream) != hipSuccess) return GNNAGG_EDEVICE;
  *best_f_chunk = best_w;
  if (best_ms) *best_ms = best / (float)kTimedCalls;
  return GNNAGG_OK;
}

extern "C" int gnnagg_tune_f_chunk(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                                   const float* edge_w, const void* X, int x_dtype, int64_t x_pitch, void* out,
                                   int out_dtype, int64_t out_pitch, int32_t F, const int32_t* row_order,
                                   const int64_t* class_off, void* workspace, size_t* workspace_bytes,
                                   void* stream_, int32_t* best_f_chunk, float* best_ms) {
  if (!workspace_bytes) return GNNAGG_ENULL;
  size_t need = 0;
  int rc = check_pitches_and_plan(N, F, F, &x_pitch, &out_pitch, row_order, class_off, &need);
  if (rc != GNNAGG_OK) return rc;
  if (!workspace) {
    *workspace_bytes = need;
    return GNNAGG_OK;
  }
  if (!best_f_chunk) return GNNAGG_ENULL;
  if (*workspace_bytes < need || ((uintptr_t)workspace & 255u)) return GNNAGG_EWORKSPACE;
  bool nothing;
  rc = check_aggregate_args(op, N, rowptr, colidx, edge_w, X, x_dtype, out, out_dtype, F, 0, row_order, class_off,
                            &nothing);
  if (rc != GNNAGG_OK) return rc;
  if (nothing) {
    *best_f_chunk = F;
    if (best_ms) *best_ms = 0.0f;
    return GNNAGG_OK;
  }
  hipStream_t stream = (hipStream_t)stream_;
  double* ws = need > 0 ? static_cast<double*>(workspace) : nullptr;
  // candidates: one chunk, the rule's choice, and pieces of 1, 2, 4, 8 lines (a quarter line and a half
  // line for rows of at most two lines)
  const int32_t xs = (x_dtype == GNNAGG_F32) ? 4 : 2, line_cols = 128 / xs;
  const bool rows_on_lines = ((uintptr_t)X % 128) == 0 && ((uint64_t)x_pitch * (uint64_t)xs) % 128 == 0;
  int32_t cand[8];
  int n_cand = 0;
  auto add = [&](int32_t w) {
    if (w <= 0 || w > F) return;
    for (int k = 0; k < n_cand; ++k)
      if (cand[k] == w) return;
    cand[n_cand++] = w;
  };
  add(F);
  add(auto_f_chunk(N, F, xs, rows_on_lines, class_off));
  for (int32_t lines = 1; lines <= 8; lines *= 2) add(lines * line_cols);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return GNNAGG_EDEVICE;
  if (hipEventCreate(&e1) != hipSuccess) {
    (void)hipEventDestroy(e0);
    return GNNAGG_EDEVICE;
  }
  constexpr int kTimedCalls = 3;
  float best = 0.0f;
  int32_t best_w = F;
  rc = GNNAGG_OK;
  for (int k = 0; k < n_cand && rc == GNNAGG_OK; ++k) {
    float ms = 0.0f;
    for (int rep = 0; rep <= kTimedCalls && rc == GNNAGG_OK; ++rep) {  // call 0 warms caches and code
      if (rep == 1 && hipEventRecord(e0, stream) != hipSuccess) rc = GNNAGG_EDEVICE;
      if (rc == GNNAGG_OK)
        rc = aggregate_impl(op, N, rowptr, colidx, edge_w, X, x_dtype, x_pitch, out, out_dtype, out_pitch, F, cand[k],
                            row_order, class_off, ws, Update(), stream);
    }
    if (rc == GNNAGG_OK && (hipEventRecord(e1, stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                            hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
      rc = GNNAGG_EDEVICE;
    if (rc == GNNAGG_OK && (k == 0 || ms < best)) {
      best = ms;
      best_w = cand[k];
    }
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != GNNAGG_OK) return rc;
  if (hipStreamSynchronize(stream) != hipSuccess) return GNNAGG_EDEVICE;
  *best_f_chunk = best_w;
  if (best_ms) *best_ms = best / (float)kTimedCalls;
  return GNNAGG_OK;
}

extern "C" int gnnagg_set_workgroup_cap(int cap) {
  if (cap < -1 || cap == 1 || cap > 16) return GNNAGG_EINVAL;  // one workgroup would need more LDS than a launch may claim
  forced_workgroup_cap.store(cap, std::memory_order_relaxed);
  return GNNAGG_OK;
}

extern "C" int64_t gnnagg_row_pitch(int32_t F, int dtype) {
  if (F <= 0 || (dtype != GNNAGG_F32 && dtype != GNNAGG_BF16)) return 0;
  const int64_t elem = (dtype == GNNAGG_F32) ? 4 : 2, bytes = (int64_t)F * elem;
  int64_t padded;
  if (bytes <= 128) {
    padded = elem;
    while (padded < bytes) padded *= 2;  // a power-of-two fraction of a line never straddles one
  } else {
    padded = ceil_div(bytes, 128) * 128;
  }
  return padded / elem;
}

extern "C" int32_t gnnagg_auto_source_blocks(int op, int64_t N, int32_t F, int x_dtype, int64_t x_pitch,
                                             const int64_t* class_off) {
  if (op < GNNAGG_SUM || op > GNNAGG_SUM_SCALED) return 0;
  if (N < 0 || F <= 0 || (x_dtype != GNNAGG_F32 && x_dtype != GNNAGG_BF16)) return 0;
  const int elem = x_dtype == GNNAGG_F32 ? 4 : 2;
  if (x_pitch == 0) x_pitch = F;
  if (x_pitch < F) return 0;
  if (class_off) {
    if (class_off[0] != 0 || class_off[GNNAGG_PLAN_CLASSES] != N) return 0;
    for (int k = 0; k < GNNAGG_PLAN_CLASSES; ++k)
      if (class_off[k] > class_off[k + 1]) return 0;
  }
  return auto_source_blocks(N, F, elem, ((uint64_t)x_pitch * (uint64_t)elem) % 128 == 0, op == GNNAGG_WSUM, class_off);
}

extern "C" int32_t gnnagg_auto_f_chunk(int64_t N, int32_t F, int x_dtype, int64_t x_pitch, const int64_t* class_off) {
  if (N < 0 || F <= 0 || (x_dtype != GNNAGG_F32 && x_dtype != GNNAGG_BF16)) return 0;
  const int elem = x_dtype == GNNAGG_F32 ? 4 : 2;
  if (x_pitch == 0) x_pitch = F;
  if (x_pitch < F) return 0;
  if (class_off) {
    if (class_off[0] != 0 || class_off[GNNAGG_PLAN_CLASSES] != N) return 0;
    for (int k = 0; k < GNNAGG_PLAN_CLASSES; ++k)
      if (class_off[k] > class_off[k + 1]) return 0;
  }
  return auto_f_chunk(N, F, elem, ((uint64_t)x_pitch * (uint64_t)elem) % 128 == 0, class_off);
}
