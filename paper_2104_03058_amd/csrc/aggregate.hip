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
#include "gather.hpp"

namespace gnnagg {
namespace {

enum { OPK_SUM = 0, OPK_WSUM = 1, OPK_MAX = 2 };

struct AggArgs {
  const int64_t* rowptr;
  const int32_t* colidx;
  const float* edge_w;
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
  // partial result of one piece of a split row, one double per column
  __device__ inline void dump(double* p) const {
#pragma unroll
    for (int k = 0; k < VEC; ++k) p[k] = acc[k];
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
  __device__ inline void dump(double* p) const {  // an int32 key is exact in a double
#pragma unroll
    for (int k = 0; k < VEC; ++k) p[k] = (double)key[k];
  }
};

// Accumulator policy of the walk in gather.hpp: one 16-byte piece of the source row per edge.
template <typename T, int OPK, int VEC>
struct AggAcc {
  static constexpr bool kWeighted = (OPK == OPK_WSUM);
  State<OPK, VEC> st;
  const char* __restrict__ xb;  // X plus this lane's column offset, in bytes
  int64_t rowbytes;
  typename Raw<T, VEC>::type raw[kUnroll];
  __device__ inline void fetch(int u, int64_t j) {
    raw[u] = load_raw<T, VEC>(reinterpret_cast<const T*>(xb + j * rowbytes));
  }
  template <bool MASKED>
  __device__ inline void use(int u, float w, bool ok) {
    float v[VEC];
    unpack(raw[u], v);
    st.template add<MASKED>(v, w, ok);
  }
};

template <typename T, int OPK, int VEC, int MODE>
__global__ __launch_bounds__(kBlock) void aggregate_kernel(const AggArgs a) {
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
  if (role.split_log2 > 0) {  // this workgroup walks one piece of the row
    e0 += (int64_t)role.piece << kSplitLenLog2;
    if (e0 > e1) e0 = e1;
    if (e1 - e0 > ((int64_t)1 << kSplitLenLog2)) e1 = e0 + ((int64_t)1 << kSplitLenLog2);
  }
  AggAcc<T, OPK, VEC> acc;
  acc.st.init();
  acc.xb = static_cast<const char*>(a.X) + (int64_t)col * (int64_t)sizeof(T);
  acc.rowbytes = a.x_pitch * (int64_t)sizeof(T);
  const int64_t nnz = (MODE == MODE_NARROW) ? a.rowptr[a.N] : 0;
  gather_row<MODE>(acc, a.colidx, a.edge_w, e0, e1, role.ng, g, role.L, col_ok, lane, nnz);
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
  } else if (role.writer) {
    float res[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) res[k] = st.result(k, deg, a.mean != 0);
    if (a.out_bf16) store_row_bf16<VEC>(static_cast<uint16_t*>(a.out) + r * a.out_pitch + col, res);
    else store_row<VEC>(static_cast<float*>(a.out) + r * a.out_pitch + col, res);
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
  const float res = st.result(0, deg, a.mean != 0);
  if (a.out_bf16) static_cast<uint16_t*>(a.out)[r * a.out_pitch + col] = (uint16_t)bf16_bits(res);
  else static_cast<float*>(a.out)[r * a.out_pitch + col] = res;
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

namespace {

// Argument checks shared by the two aggregation entry points; GNNAGG_OK with *nothing = true means
// there is nothing to do.
int check_aggregate_args(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx, const float* edge_w,
                         const void* X, int x_dtype, void* out, int out_dtype, int32_t F, int32_t f_chunk,
                         const int32_t* row_order, const int64_t* class_off, bool* nothing) {
  *nothing = false;
  if (op < GNNAGG_SUM || op > GNNAGG_MAX) return GNNAGG_EINVAL;
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
  if (op == GNNAGG_WSUM && !edge_w) return GNNAGG_ENULL;
  // colidx may only be NULL for a graph without edges, which the host cannot see; require it
  if (!colidx) return GNNAGG_ENULL;
  const size_t xs = (x_dtype == GNNAGG_F32) ? 4 : 2;
  if (((uintptr_t)X % xs) || ((uintptr_t)out % (out_dtype == GNNAGG_F32 ? 4 : 2)) || ((uintptr_t)rowptr % 8) ||
      ((uintptr_t)colidx % 4) || (edge_w && ((uintptr_t)edge_w % 4)))
    return GNNAGG_EINVAL;
  if (X == out) return GNNAGG_EINVAL;
  return GNNAGG_OK;
}

// ws == nullptr: no row is split.  Otherwise ws holds segs.ws_slots * F doubles.
int aggregate_impl(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx, const float* edge_w,
                   const void* X, int x_dtype, int64_t x_pitch, void* out, int out_dtype, int64_t out_pitch,
                   int32_t F, int32_t f_chunk, const int32_t* row_order, const int64_t* class_off, double* ws,
                   hipStream_t stream) {
  const size_t xs = (x_dtype == GNNAGG_F32) ? 4 : 2;
  const bool rows_on_lines = ((uintptr_t)X % 128) == 0 && ((uint64_t)x_pitch * xs) % 128 == 0;
  if (f_chunk == GNNAGG_F_CHUNK_AUTO) f_chunk = auto_f_chunk(N, F, (int)xs, rows_on_lines, class_off);
  std::vector<SliceLaunch> launches;
  const bool capped = resident_workgroup_cap(class_off, N, 6, kWave, true) > 0;  // dense graph: caps in play
  plan_columns(F, f_chunk, (int)(16 / xs), 0, rows_on_lines ? (int)(128 / xs) : 0, capped, &launches);
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
    a.lds_per_workgroup =
        lds_claim(resident_workgroup_cap(class_off, N, a.sl.g_log2, active_lanes_per_wave(a.sl), opk == OPK_WSUM));
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
  if (ws && !args.empty() && args[0].segs.ws_slots > 0) {
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
    m.nrun = 0;
    m.rows = 0;
    const SegTable& st = args[0].segs;
    for (int k = 0; k < st.nseg; ++k) {
      if (st.seg[k].split_log2 == 0) continue;
      if (m.nrun >= kMaxSplitSeg) return GNNAGG_EUNSUPPORTED;  // cannot happen: build_segments caps them
      m.run[m.nrun++] = st.seg[k];
      m.rows += (int64_t)st.seg[k].row_end - st.seg[k].row_begin;
    }
    const int64_t blocks = ceil_div(m.rows * (int64_t)F, kBlock);
    if (blocks > 0x7fffffffll) return GNNAGG_EUNSUPPORTED;
    if (opk == OPK_MAX) hipLaunchKernelGGL(split_merge_kernel<OPK_MAX>, dim3((unsigned)blocks), dim3(kBlock), 0, stream, m);
    else hipLaunchKernelGGL(split_merge_kernel<OPK_SUM>, dim3((unsigned)blocks), dim3(kBlock), 0, stream, m);
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
                        class_off, nullptr, (hipStream_t)stream_);
}

extern "C" int gnnagg_aggregate_ws(int op, int64_t N, const int64_t* rowptr, const int32_t* colidx,
                                   const float* edge_w, const void* X, int x_dtype, int64_t x_pitch, void* out,
                                   int out_dtype, int64_t out_pitch, int32_t F, int32_t f_chunk,
                                   const int32_t* row_order, const int64_t* class_off, void* workspace,
                                   size_t* workspace_bytes, void* stream_) {
  if (!workspace_bytes) return GNNAGG_ENULL;
  if (N < 0 || F <= 0) return GNNAGG_EINVAL;
  if (x_pitch == 0) x_pitch = F;
  if (out_pitch == 0) out_pitch = F;
  if (x_pitch < F || out_pitch < F || x_pitch > (1ll << 40) || out_pitch > (1ll << 40)) return GNNAGG_EINVAL;
  if ((row_order == nullptr) != (class_off == nullptr)) return GNNAGG_EINVAL;
  if (N >= (1ll << 31)) return GNNAGG_EUNSUPPORTED;
  SegTable probe;
  int rc = build_segments(class_off, N, 6, true, &probe);  // the split runs do not depend on the slice width
  if (rc != GNNAGG_OK) return rc;
  const size_t need = (size_t)probe.ws_slots * (size_t)F * sizeof(double);
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
                        row_order, class_off, need > 0 ? static_cast<double*>(workspace) : nullptr,
                        (hipStream_t)stream_);
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
