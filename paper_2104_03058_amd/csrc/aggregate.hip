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
#include "common.hpp"
#include "schedule.hpp"
#include "device_utils.hpp"

namespace gnnagg {
namespace {

enum { OPK_SUM = 0, OPK_WSUM = 1, OPK_MAX = 2 };
constexpr int kUnroll = 8;  // independent gathers in flight per lane

struct AggArgs {
  const int64_t* rowptr;
  const int32_t* colidx;
  const float* edge_w;
  const void* X;
  float* out;
  const int32_t* order;
  int64_t F;
  int64_t N;
  SliceLaunch sl;
  int32_t mean;
  uint32_t lds_per_workgroup;  // host only: LDS each workgroup should occupy (0 = no cap)
  SegTable segs;
};

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
      const double x = (MASKED && !ok) ? 0.0 : (double)v[k];
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
  __device__ inline float result(int k, int64_t deg, bool mean) const {
    return (float)((mean && deg > 0) ? acc[k] / (double)deg : acc[k]);
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
  __device__ inline float result(int k, int64_t deg, bool) const { return deg > 0 ? key_value(key[k]) : 0.0f; }
};

typedef int32_t i32x4_u __attribute__((ext_vector_type(4), aligned(4)));

__device__ inline int64_t uniform64(int64_t v) {  // v is the same in every lane: move it to scalar registers
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

// One gather + accumulate batch: kUnroll independent 16-byte row loads issued back to back, then the
// accumulates.  Straight-line code: an entry that does not exist (OKEXPR false, only in MASKED
// batches) re-reads the row JSAFE, which does exist, and enters the reduction with weight 0 (sums)
// or the lowest key (max), so no load sits behind a branch.
#define GNNAGG_BATCH(UN, MASKED, OKEXPR, JEXPR, WEXPR, JSAFE)                                     \
  {                                                                                           \
    typename Raw<T, VEC>::type raw[(UN)];                                                  \
    float wv[(UN)];                                                                        \
    bool okv[(UN)];                                                                        \
    _Pragma("unroll") for (int u = 0; u < (UN); ++u) {                                     \
      okv[u] = (MASKED) ? (bool)(OKEXPR) : true;                                              \
      const int64_t jj = okv[u] ? (int64_t)(JEXPR) : (int64_t)(JSAFE);                        \
      const float wsel = (OPK == OPK_WSUM) ? (float)(WEXPR) : 1.0f;                           \
      wv[u] = okv[u] ? wsel : 0.0f;                                                           \
      raw[u] = load_raw<T, VEC>(reinterpret_cast<const T*>(xb + jj * rowbytes + lane_off));   \
    }                                                                                         \
    _Pragma("unroll") for (int u = 0; u < (UN); ++u) {                                     \
      float v[VEC];                                                                           \
      unpack(raw[u], v);                                                                      \
      st.template add<(MASKED)>(v, wv[u], okv[u]);                                            \
    }                                                                                         \
  }

// How a row's edge list is dealt out to its P = 2^p_log2 neighbour slots: in rounds of 8*P consecutive
// edges, slot ng taking edges [8*ng, 8*ng + 8) of every round - one gather batch.  All slots of a row
// therefore work on the same 8*P-edge stretch of the (source-sorted) list at any time, and rows that
// run side by side advance through the source ids together: this keeps the set of X rows in flight
// small enough for L2 to serve a row to several destinations.
//
// Slot = a whole wavefront (64 lanes span the slice).  The wave reads the edge indices (and weights) of
// its next eight batches with one load each, then walks them: the source row of an entry is broadcast
// with v_readlane, so row addresses live in scalar registers.  [e0, e1), ng are the same in every lane.
template <typename T, int OPK, int VEC, int U>
__device__ inline void gather_wave(const AggArgs& a, State<OPK, VEC>& st, int64_t e0, int64_t e1, int ng,
                                   int p_log2, int col, int lane) {
  const int64_t e0_u = uniform64(e0), e1_u = uniform64(e1);
  const int ng_u = __builtin_amdgcn_readfirstlane(ng);
  static_assert(U == 4 || U == 8 || U == 16, "a batch is 4, 8 or 16 gathers");
  constexpr int u_log2 = (U == 4) ? 2 : (U == 8 ? 3 : 4);
  const int shift = u_log2 + p_log2;                  // log2 of the round length (U edges per slot)
  const int64_t outer = (int64_t)kWave << p_log2;     // edges the row advances per index load
  const int64_t lane_pos = ((int64_t)(lane >> u_log2) << shift) + (ng_u << u_log2) + (lane & (U - 1));
  const char* __restrict__ xb = static_cast<const char*>(a.X);
  const int64_t rowbytes = a.F * (int64_t)sizeof(T);
  const uint32_t lane_off = (uint32_t)col * (uint32_t)sizeof(T);
  int32_t idx_c = 0;
  float w_c = 1.0f;
  if (e0_u + lane_pos < e1_u) {
    idx_c = a.colidx[e0_u + lane_pos];
    if (OPK == OPK_WSUM) w_c = a.edge_w[e0_u + lane_pos];
  }
  for (int64_t e = e0_u; e < e1_u; e += outer) {
    int32_t idx_n = 0;  // the next eight batches' indices are requested before this block's rows
    float w_n = 1.0f;
    if (e + outer + lane_pos < e1_u) {
      idx_n = a.colidx[e + outer + lane_pos];
      if (OPK == OPK_WSUM) w_n = a.edge_w[e + outer + lane_pos];
    }
    for (int k = 0; k < kWave / U; ++k) {
      const int64_t left = e1_u - (e + ((int64_t)k << shift) + (ng_u << u_log2));
      if (left <= 0) break;
      const int l0 = k * U;
      if (left >= U) {
        GNNAGG_BATCH(U, false, true, __builtin_amdgcn_readlane(idx_c, l0 + u),
                     __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_c), l0 + u)), 0)
      } else {
        GNNAGG_BATCH(U, true, u < left, __builtin_amdgcn_readlane(idx_c, l0 + u),
                     __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_c), l0 + u)),
                     __builtin_amdgcn_readlane(idx_c, l0))
      }
    }
    idx_c = idx_n;
    w_c = w_n;
  }
}

// Slot = 2^g lanes, 8 <= 2^g <= 32.  The lanes of a slot read the indices of the slot's next 2^g / 8
// batches with one load and hand them round with cross-lane shuffles.  All lanes of a slot run the loop
// together; lanes without columns of their own hold indices for the others and re-read the slice's
// last columns (role.col is always a valid column) rather than branching around the gathers.
template <typename T, int OPK, int VEC>
__device__ inline void gather_wide(const AggArgs& a, State<OPK, VEC>& st, int64_t e0, int64_t e1, int ng,
                                   int p_log2, int col, int lane, int g) {
  const int G = 1 << g;
  const int gl = lane & (G - 1), slot_base = lane & ~(G - 1);
  const int shift = 3 + p_log2;
  const int64_t outer = (int64_t)G << p_log2;
  const int64_t lane_pos = ((int64_t)(gl >> 3) << shift) + (ng << 3) + (gl & 7);
  const char* __restrict__ xb = static_cast<const char*>(a.X);
  const int64_t rowbytes = a.F * (int64_t)sizeof(T);
  const uint32_t lane_off = (uint32_t)col * (uint32_t)sizeof(T);
  int32_t idx_c = -1;
  float w_c = 0.0f;
  if (e0 + lane_pos < e1) {
    idx_c = a.colidx[e0 + lane_pos];
    if (OPK == OPK_WSUM) w_c = a.edge_w[e0 + lane_pos];
  }
  for (int64_t e = e0; e < e1; e += outer) {
    int32_t idx_n = -1;
    float w_n = 0.0f;
    if (e + outer + lane_pos < e1) {
      idx_n = a.colidx[e + outer + lane_pos];
      if (OPK == OPK_WSUM) w_n = a.edge_w[e + outer + lane_pos];
    }
    for (int k = 0; k < (G >> 3); ++k) {
      if (e + ((int64_t)k << shift) + (ng << 3) >= e1) break;  // same for every lane of the slot
      int32_t j[kUnroll];
      float wj[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        j[u] = __shfl(idx_c, slot_base + k * kUnroll + u, kWave);
        wj[u] = (OPK == OPK_WSUM) ? __shfl(w_c, slot_base + k * kUnroll + u, kWave) : 1.0f;
      }
      GNNAGG_BATCH(kUnroll, true, j[u] >= 0, j[u], wj[u], j[0])
    }
    idx_c = idx_n;
    w_c = w_n;
  }
}

// Slot = 1, 2 or 4 lanes (slices of at most 16 fp32 / 32 bf16 columns).  Every lane reads the next
// eight edge indices of its slot's range itself, as two 16-byte loads (the lanes of a slot read the
// same addresses, which the memory pipeline merges).  The loads may run past the end of the slot's
// range into the following entries of colidx, never past nnz.
template <typename T, int OPK, int VEC>
__device__ inline void gather_narrow(const AggArgs& a, State<OPK, VEC>& st, int64_t es, int64_t ee,
                                     int64_t stride, int col, int64_t nnz) {
  const char* __restrict__ xb = static_cast<const char*>(a.X);
  const int64_t rowbytes = a.F * (int64_t)sizeof(T);
  const uint32_t lane_off = (uint32_t)col * (uint32_t)sizeof(T);
  for (int64_t e = es; e < ee; e += stride) {
    int32_t j[kUnroll];
    float wj[kUnroll];
    if (e + kUnroll <= nnz) {
      const i32x4_u i0 = *reinterpret_cast<const i32x4_u*>(a.colidx + e);
      const i32x4_u i1 = *reinterpret_cast<const i32x4_u*>(a.colidx + e + 4);
      j[0] = i0.x; j[1] = i0.y; j[2] = i0.z; j[3] = i0.w;
      j[4] = i1.x; j[5] = i1.y; j[6] = i1.z; j[7] = i1.w;
      if (OPK == OPK_WSUM) {
        const f32x4_u w0 = *reinterpret_cast<const f32x4_u*>(a.edge_w + e);
        const f32x4_u w1 = *reinterpret_cast<const f32x4_u*>(a.edge_w + e + 4);
        wj[0] = w0.x; wj[1] = w0.y; wj[2] = w0.z; wj[3] = w0.w;
        wj[4] = w1.x; wj[5] = w1.y; wj[6] = w1.z; wj[7] = w1.w;
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
        if (e + u >= ee) j[u] = -1;
    } else {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const bool ok = e + u < ee;
        j[u] = ok ? a.colidx[e + u] : -1;
        if (OPK == OPK_WSUM) wj[u] = ok ? a.edge_w[e + u] : 0.0f;
      }
    }
    if (OPK != OPK_WSUM) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) wj[u] = 1.0f;
    }
    GNNAGG_BATCH(kUnroll, true, j[u] >= 0, j[u], wj[u], j[0])
  }
}

enum { MODE_WAVE = 0, MODE_WIDE = 1, MODE_NARROW = 2 };  // 64 / 8..32 / 1..4 lanes per slice (fixed per launch)

template <typename T, int OPK, int VEC, int MODE>
__global__ __launch_bounds__(kBlock) void aggregate_kernel(const AggArgs a) {
  static_assert(kUnroll == 8, "gather_narrow reads eight indices as two 16-byte loads");
  __shared__ double lds[(kWavesPerBlock - 1) * kWave * VEC];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;

  const LaneRole role = lane_role(a.sl, a.segs, blockIdx.x, tid);
  const int g = role.g, col = role.col;
  const bool hub = role.hub, row_ok = role.row_ok, col_ok = role.col_ok;
  int64_t r = 0, e0 = 0, e1 = 0;
  if (row_ok) {
    r = a.order ? (int64_t)a.order[role.ridx] : role.ridx;
    e0 = a.rowptr[r];
    e1 = a.rowptr[r + 1];
  }
  const int64_t deg = e1 - e0;
  const int p_log2 = (hub ? 8 : role.L) - g;  // log2 of the row's neighbour slots

  State<OPK, VEC> st;
  st.init();
  if constexpr (MODE == MODE_WAVE) {
    gather_wave<T, OPK, VEC, kUnroll>(a, st, e0, e1, role.ng, p_log2, col, lane);
  } else if constexpr (MODE == MODE_WIDE) {
    gather_wide<T, OPK, VEC>(a, st, e0, e1, role.ng, p_log2, col, lane, g);
  } else {
    const int64_t nnz = a.rowptr[a.N];
    if (col_ok)
      gather_narrow<T, OPK, VEC>(a, st, e0 + (int64_t)role.ng * kUnroll, e1, (int64_t)kUnroll << p_log2, col, nnz);
  }

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
  if (role.writer) {
    float res[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) res[k] = st.result(k, deg, a.mean != 0);
    store_row<VEC>(a.out + r * a.F + col, res);
  }
}

template <typename T, int OPK, int VEC, int MODE>
int launch_one(const AggArgs& a, uint64_t grid, hipStream_t stream) {
  // Unused dynamic LDS is how the number of resident workgroups per compute unit is capped (see
  // resident_workgroup_cap): a workgroup that claims 1/k of the LDS leaves room for k of them.
  const size_t static_lds = sizeof(double) * (kWavesPerBlock - 1) * kWave * VEC;
  const size_t dyn_lds = a.lds_per_workgroup > static_lds ? a.lds_per_workgroup - static_lds : 0;
  hipLaunchKernelGGL((aggregate_kernel<T, OPK, VEC, MODE>), dim3((unsigned)grid), dim3(kBlock), dyn_lds, stream, a);
  return hipGetLastError() == hipSuccess ? GNNAGG_OK : GNNAGG_EDEVICE;
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

extern "C" int gnnagg_aggregate(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                                const float* edge_w, const void* X, int x_dtype, void* out, int out_dtype,
                                int32_t F, int32_t f_chunk, const int32_t* row_order, const int64_t* class_off,
                                void* stream_) {
  if (op < GNNAGG_SUM || op > GNNAGG_MAX) return GNNAGG_EINVAL;
  if (N < 0 || F <= 0 || f_chunk < 0) return GNNAGG_EINVAL;
  if (x_dtype != GNNAGG_F32 && x_dtype != GNNAGG_BF16) return GNNAGG_EINVAL;
  if (out_dtype != GNNAGG_F32) return out_dtype == GNNAGG_BF16 ? GNNAGG_EUNSUPPORTED : GNNAGG_EINVAL;
  if (N >= (1ll << 31)) return GNNAGG_EUNSUPPORTED;
  if ((row_order == nullptr) != (class_off == nullptr)) return GNNAGG_EINVAL;
  if (N == 0) return GNNAGG_OK;
  if (!rowptr || !X || !out) return GNNAGG_ENULL;
  if (op == GNNAGG_WSUM && !edge_w) return GNNAGG_ENULL;
  // colidx may only be NULL for a graph without edges, which the host cannot see; require it
  if (!colidx) return GNNAGG_ENULL;
  const size_t xs = (x_dtype == GNNAGG_F32) ? 4 : 2;
  if (((uintptr_t)X % xs) || ((uintptr_t)out % 4) || ((uintptr_t)rowptr % 8) || ((uintptr_t)colidx % 4) ||
      (edge_w && ((uintptr_t)edge_w % 4)))
    return GNNAGG_EINVAL;
  if (X == out) return GNNAGG_EINVAL;

  std::vector<SliceLaunch> launches;
  plan_columns(F, f_chunk, (int)(16 / xs), 0, &launches);
  hipStream_t stream = (hipStream_t)stream_;
  const int opk = (op == GNNAGG_WSUM) ? OPK_WSUM : (op == GNNAGG_MAX ? OPK_MAX : OPK_SUM);

  // build and validate every launch before the first one is enqueued
  std::vector<AggArgs> args(launches.size());
  std::vector<uint64_t> grids(launches.size());
  for (size_t k = 0; k < launches.size(); ++k) {
    AggArgs& a = args[k];
    a.rowptr = rowptr;
    a.colidx = colidx;
    a.edge_w = edge_w;
    a.X = X;
    a.out = static_cast<float*>(out);
    a.order = row_order;
    a.F = F;
    a.N = N;
    a.sl = launches[k];
    a.mean = (op == GNNAGG_MEAN);
    a.lds_per_workgroup = lds_claim(resident_workgroup_cap(class_off, N, a.sl.g_log2));
    int rc = build_segments(class_off, N, a.sl.g_log2, &a.segs);
    if (rc != GNNAGG_OK) return rc;
    grids[k] = (uint64_t)a.segs.blocks_per_slice * (uint64_t)a.sl.n_chunks * (uint64_t)a.sl.n_sub;
    if (grids[k] == 0 || grids[k] > 0x7fffffffull) return GNNAGG_EUNSUPPORTED;
  }
  for (size_t k = 0; k < launches.size(); ++k) {
    int rc = (x_dtype == GNNAGG_F32) ? launch_op<float>(opk, args[k], grids[k], stream)
                                     : launch_op<bf16_t>(opk, args[k], grids[k], stream);
    if (rc != GNNAGG_OK) return rc;
  }
  return GNNAGG_OK;
}
