// gnnagg_gat_attention: edge scores, softmax over each destination's in-edges
// and the per-head weighted sum, in one pass over the neighbour rows.
//
// The attention logits need whole head vectors, so the two per-vertex score
// arrays are computed once up front; chunks are whole heads (the paper's GAT
// chunk width 8, Section III, is one head at 8 channels) and every chunk sees
// the same weights.  The softmax is kept online: a lane carries (reference logit,
// running denominator, running weighted sum) for the head its columns belong
// to, one exp per edge, and the states of a row's neighbour slots are merged
// with cross-lane shuffles (hub rows: across waves through LDS).
//
// Where a head spans at most four lanes (4, 8 or 16 channels per head) the source's score is not
// gathered from the score array but recomputed from the feature-row piece the lanes hold anyway
// (a few fp64 FMAs and quad-local lane exchanges): one line request less per edge.  The score kernel
// sums in the same order, so both routes give the same bits.
#include <math.h>

#include "common.hpp"
#include "device_utils.hpp"
#include "gather.hpp"
#include "schedule.hpp"

namespace gnnagg {
namespace {

struct GatArgs {
  const int64_t* rowptr;
  const int32_t* colidx;
  const float* H;
  const float* a_src;
  const float* a_dst;
  const float* s_src;  // score arrays; both null when every score is recomputed in registers (LH > 0, no alpha)
  const float* s_dst;
  float* alpha;
  float* out;
  const int32_t* order;
  int32_t heads, C;
  float slope;
  int64_t N;
  double* pieces;  // partial softmax states of split rows: [slot][heads * C sums | heads references | heads denominators]
  SliceLaunch sl;
  SegTable segs;
};

// s_src[j,h] = a_src[h,:] . H[j,h,:],  s_dst[j,h] = a_dst[h,:] . H[j,h,:]   (fp64, rounded once).
// Summation order: partial sums over consecutive groups of `grp` channels (grp divides C, C / grp is
// 1, 2 or 4), each a chain of FMAs from zero, then a pairwise tree - the order the aggregation kernel
// reproduces when it recomputes a source score from the row pieces of a head's lanes.
__global__ __launch_bounds__(kBlock) void gat_scores_kernel(const float* __restrict__ H,
                                                            const float* __restrict__ a_src,
                                                            const float* __restrict__ a_dst, int64_t n_vh,
                                                            int32_t heads, int32_t C, int32_t grp,
                                                            float* __restrict__ s_src, float* __restrict__ s_dst) {
  const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (t >= n_vh) return;
  const int h = (int)(t % heads);
  const float* __restrict__ x = H + t * C;
  const float* __restrict__ as = a_src + (int64_t)h * C;
  const float* __restrict__ ad = a_dst + (int64_t)h * C;
  double ps[4] = {0.0, 0.0, 0.0, 0.0}, pd[4] = {0.0, 0.0, 0.0, 0.0};
  const int n_grp = C / grp;
  for (int q = 0; q < n_grp; ++q) {
    double s = 0.0, d = 0.0;
    for (int c = q * grp; c < (q + 1) * grp; ++c) {
      const double v = (double)x[c];
      s = __builtin_fma((double)as[c], v, s);
      d = __builtin_fma((double)ad[c], v, d);
    }
    ps[q] = s;
    pd[q] = d;
  }
  double s = ps[0], d = pd[0];
  if (n_grp == 2) {
    s = ps[0] + ps[1];
    d = pd[0] + pd[1];
  } else if (n_grp == 4) {
    s = (ps[0] + ps[1]) + (ps[2] + ps[3]);
    d = (pd[0] + pd[1]) + (pd[2] + pd[3]);
  }
  s_src[t] = (float)s;
  s_dst[t] = (float)d;
}

// x of the lane whose index differs in bit 0 (XOR1) or bit 1 (XOR2): a DPP move inside each quad of lanes
constexpr int kQuadXor1 = 0xB1;  // quad_perm [1,0,3,2]
constexpr int kQuadXor2 = 0x4E;  // quad_perm [2,3,0,1]
template <int CTRL>
__device__ inline double quad_exchange(double x) {
  const uint64_t b = (uint64_t)__double_as_longlong(x);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, 0xF, 0xF, false);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, 0xF, 0xF, false);
  return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// exp through the hardware exp2 (argument scaled by log2 e in fp32): relative error about 1e-7 |x|, i.e.
// below 2e-6 for every term within e^-16 of a row's largest, against a parity bar of 1e-5; a fraction of
// the instructions of the correctly rounded routine, which showed in the run time (about 10 %).
__device__ inline float exp_fast(float x) { return __expf(x); }

template <int VEC>
struct SoftState {
  float m;          // reference logit: within kLazy of the maximum seen, or above it
  double l;         // sum of exp(logit - m)
  double acc[VEC];  // sum of exp(logit - m) * H   (fp64: hub rows add thousands of terms)
  __device__ inline void init() {
    m = -INFINITY;
    l = 0.0;
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = 0.0;
  }
  // The reference m only has to keep exp(logit - m) in range, it need not be the exact maximum: it is
  // moved (and the sums rescaled) only when a logit exceeds it by more than kLazy, which after the
  // first edge is rare, so a wavefront almost always runs the short branch alone.
  static constexpr float kLazy = 8.0f;
  __device__ inline void add(float logit, const float (&v)[VEC]) {
    const float d = logit - m;
    if (d > kLazy) {  // first edge (m = -inf, exp(-inf) = 0) or a jump
      const double ex = (double)exp_fast(-d);
      l = __builtin_fma(l, ex, 1.0);
#pragma unroll
      for (int k = 0; k < VEC; ++k) acc[k] = __builtin_fma(acc[k], ex, (double)v[k]);
      m = logit;
    } else {
      const double ex = (double)exp_fast(d);  // at most e^kLazy
      l += ex;
#pragma unroll
      for (int k = 0; k < VEC; ++k) acc[k] = __builtin_fma(ex, (double)v[k], acc[k]);
    }
  }
  __device__ inline void merge(const SoftState& o) {
    const float mm = fmaxf(m, o.m);
    const double sa = (m == mm) ? 1.0 : (double)exp_fast(m - mm);
    const double sb = (o.m == mm) ? 1.0 : (double)exp_fast(o.m - mm);
    l = l * sa + o.l * sb;
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = acc[k] * sa + o.acc[k] * sb;
    m = mm;
  }
  __device__ inline SoftState shuffled_xor(int stride) const {
    SoftState o;
    o.m = __shfl_xor(m, stride, kWave);
    o.l = __shfl_xor(l, stride, kWave);
#pragma unroll
    for (int k = 0; k < VEC; ++k) o.acc[k] = __shfl_xor(acc[k], stride, kWave);
    return o;
  }
};

// Accumulator policy of the walk in gather.hpp: per edge, the source's score for this lane's head and
// one 16-byte piece of its feature row.  LH == 0: the score is gathered from s_src.  LH = 1, 2, 4: a
// head is held by LH adjacent lanes (aligned to LH) that always run together, and the score is their
// dot product with a_src, summed in the order of gat_scores_kernel.
template <int VEC, int LH>
struct GatAcc {
  static constexpr bool kWeighted = false;
  SoftState<VEC> st;
  const char* __restrict__ hb;  // H plus this lane's column offset, in bytes
  int64_t rowbytes;
  const float* __restrict__ s_src_h;  // s_src plus this lane's head
  int32_t heads;
  float sd, slope;
  double av[VEC];  // a_src at this lane's columns (LH > 0)
  typename Raw<float, VEC>::type raw[kUnroll];
  float ss[kUnroll];
  __device__ inline void fetch(int u, int32_t j) {
    if constexpr (LH == 0) ss[u] = s_src_h[(int64_t)j * heads];
    // j is a vertex id and a row of H is shorter than 2^32 bytes: one 32 x 32 -> 64 bit multiply-add
    raw[u] = load_raw<float, VEC>(
        reinterpret_cast<const float*>(hb + (uint64_t)(uint32_t)j * (uint64_t)(uint32_t)rowbytes));
  }
  __device__ inline void fetch_uniform(int u, int64_t j) {
    if constexpr (LH == 0) ss[u] = s_src_h[j * heads];
    raw[u] = load_raw<float, VEC>(reinterpret_cast<const float*>(hb + j * rowbytes));
  }
  template <bool MASKED>
  __device__ inline void use(int u, float, bool ok) {
    float v[VEC];
    unpack(raw[u], v);
    float sj;
    if constexpr (LH == 0) {
      sj = ss[u];
    } else {  // before the mask test: the lanes of a head exchange partial sums
      double p = 0.0;
#pragma unroll
      for (int k = 0; k < VEC; ++k) p = __builtin_fma(av[k], (double)v[k], p);
      if constexpr (LH >= 2) p += quad_exchange<kQuadXor1>(p);
      if constexpr (LH >= 4) p += quad_exchange<kQuadXor2>(p);
      sj = (float)p;
    }
    if (MASKED && !ok) return;
    const float s = sj + sd;
    st.add(s >= 0.0f ? s : slope * s, v);
  }
};

template <int VEC, int MODE, int LH>
__global__ __launch_bounds__(kBlock) void gat_aggregate_kernel(const GatArgs a) {
  __shared__ double lds[(kWavesPerBlock - 1) * kWave * (2 + VEC)];
  __shared__ double fin[2 * kWave];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;

  const LaneRole role = lane_role(a.sl, a.segs, blockIdx.x, tid);
  const int g = role.g, ng = role.ng, P = role.P, col = role.col;  // slice widths are multiples of VEC here
  const bool hub = role.hub, row_ok = role.row_ok, col_ok = role.col_ok;
  int64_t r = 0, e0 = 0, e1 = 0;
  if (row_ok) {
    r = a.order ? (int64_t)a.order[role.ridx] : role.ridx;
    e0 = a.rowptr[r];
    e1 = a.rowptr[r + 1];
  }
  const int head = col / a.C;  // VEC divides C, so the lane's columns lie in one head
  const int64_t HC = (int64_t)a.heads * a.C;
  const bool split = role.split_log2 > 0;  // this workgroup walks one piece of a very long row
  if (split) {
    e0 += (int64_t)role.piece << kSplitLenLog2;
    if (e0 > e1) e0 = e1;
    if (e1 - e0 > ((int64_t)1 << kSplitLenLog2)) e1 = e0 + ((int64_t)1 << kSplitLenLog2);
  }

  GatAcc<VEC, LH> acc;
  acc.st.init();
#pragma unroll
  for (int k = 0; k < VEC; ++k) acc.av[k] = (LH > 0) ? (double)a.a_src[col + k] : 0.0;  // a_src is [heads, C]: same flat index as the column
  acc.hb = reinterpret_cast<const char*>(a.H + col);
  acc.rowbytes = HC * (int64_t)sizeof(float);
  acc.s_src_h = a.s_src + head;
  acc.heads = a.heads;
  acc.slope = a.slope;
  if (LH > 0 && !a.s_dst) {
    // the destination's score from its own feature row, summed in the order of gat_scores_kernel (the lanes
    // of a head hold the same row and run together; a lane without a row computes on row 0 and drops it)
    float hv[VEC];
    unpack(load_raw<float, VEC>(a.H + r * HC + col), hv);
    double p = 0.0;
#pragma unroll
    for (int k = 0; k < VEC; ++k) p = __builtin_fma((double)a.a_dst[col + k], (double)hv[k], p);
    if constexpr (LH >= 2) p += quad_exchange<kQuadXor1>(p);
    if constexpr (LH >= 4) p += quad_exchange<kQuadXor2>(p);
    acc.sd = (float)p;
  } else {
    acc.sd = row_ok ? a.s_dst[r * a.heads + head] : 0.0f;
  }
  const float sd = acc.sd;
  const int64_t nnz = (MODE == MODE_NARROW) ? a.rowptr[a.N] : 0;
  gather_row<MODE>(acc, a.colidx, nullptr, e0, e1, ng, g, role.L, col_ok, lane, nnz);
  SoftState<VEC>& st = acc.st;

  const int lanes_in_wave = hub ? kWave : (1 << role.L);
  for (int stride = 1 << g; stride < lanes_in_wave; stride <<= 1) st.merge(st.shuffled_xor(stride));
  if (hub) {
    if (wv > 0) {
      double* p = lds + ((wv - 1) * kWave + lane) * (2 + VEC);
      p[0] = (double)st.m;
      p[1] = st.l;
#pragma unroll
      for (int k = 0; k < VEC; ++k) p[2 + k] = st.acc[k];
    }
    __syncthreads();
    if (wv == 0) {
      for (int ww = 1; ww < kWavesPerBlock; ++ww) {
        const double* p = lds + ((ww - 1) * kWave + lane) * (2 + VEC);
        SoftState<VEC> o;
        o.m = (float)p[0];
        o.l = p[1];
#pragma unroll
        for (int k = 0; k < VEC; ++k) o.acc[k] = p[2 + k];
        st.merge(o);
      }
      fin[lane] = (double)st.m;
      fin[kWave + lane] = st.l;
    }
    __syncthreads();
    st.m = (float)fin[lane];  // every wave now knows the row's final maximum and denominator
    st.l = fin[kWave + lane];
  }

  if (split) {
    // leave the piece's state in its workspace slot; the merge kernels finish the row
    if (role.writer) {
      double* p = a.pieces + (int64_t)role.ws_slot * (HC + 2 * a.heads);
#pragma unroll
      for (int k = 0; k < VEC; ++k) p[col + k] = st.acc[k];
      if ((col % a.C) == 0) {
        p[HC + head] = (double)st.m;
        p[HC + a.heads + head] = st.l;
      }
    }
    return;
  }
  if (a.out && role.writer) {
    float res[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) res[k] = (e1 > e0) ? (float)(st.acc[k] / st.l) : 0.0f;
    store_row<VEC>(a.out + r * HC + col, res);
  }
  // softmax weights, written by the first lane of every head; the row's edges are dealt to the slots
  // one at a time here
  if (a.alpha && row_ok && col_ok && (col % a.C) == 0) {
    for (int64_t e = e0 + ng; e < e1; e += P) {
      const float s = a.s_src[(int64_t)a.colidx[e] * a.heads + head] + sd;
      const float logit = s >= 0.0f ? s : a.slope * s;
      a.alpha[e * a.heads + head] = (float)((double)exp_fast(logit - st.m) / st.l);
    }
  }
}

// Split rows: fold the pieces of a row in piece order.  One thread per (split row, column); the first
// column of a head also records the row's final reference and denominator for the weights.
struct GatMergeArgs {
  const int64_t* rowptr;
  const int32_t* colidx;
  const int32_t* order;
  const float* s_src;
  const float* s_dst;
  float* alpha;
  float* out;
  const double* pieces;
  double* fin;   // [split row][head][reference, denominator]
  int64_t rows;  // split rows in all runs together
  int32_t heads, C, nrun;
  float slope;
  Seg run[kMaxSplitSeg];
};

__device__ inline int find_run(const GatMergeArgs& a, int64_t* i) {
  int k = 0;
  while (k + 1 < a.nrun && *i >= (int64_t)a.run[k].row_end - a.run[k].row_begin) {
    *i -= (int64_t)a.run[k].row_end - a.run[k].row_begin;
    ++k;
  }
  return k;
}

__global__ __launch_bounds__(kBlock) void gat_split_merge_kernel(const GatMergeArgs a) {
  const int64_t HC = (int64_t)a.heads * a.C;
  const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (t >= a.rows * HC) return;
  const int64_t row_i = t / HC;
  const int64_t col = t - row_i * HC;
  const int head = (int)(col / a.C);
  int64_t i = row_i;
  const Seg run = a.run[find_run(a, &i)];
  const int64_t r = a.order[run.row_begin + i];
  const int64_t n_pieces = (int64_t)1 << run.split_log2;
  const int64_t pitch = HC + 2 * a.heads;
  const double* p = a.pieces + ((int64_t)run.ws_begin + i * n_pieces) * pitch;
  SoftState<1> st;
  st.init();
  for (int64_t q = 0; q < n_pieces; ++q, p += pitch) {
    SoftState<1> o;
    o.m = (float)p[HC + head];
    o.l = p[HC + a.heads + head];
    o.acc[0] = p[col];
    st.merge(o);
  }
  if (a.out) a.out[r * HC + col] = st.l > 0.0 ? (float)(st.acc[0] / st.l) : 0.0f;
  if (col == (int64_t)head * a.C) {
    a.fin[(row_i * a.heads + head) * 2] = (double)st.m;
    a.fin[(row_i * a.heads + head) * 2 + 1] = st.l;
  }
}

// Softmax weights of the split rows: blockIdx.y strides over the rows, the threads of a block row over
// (edge, head) pairs.
__global__ __launch_bounds__(kBlock) void gat_split_alpha_kernel(const GatMergeArgs a) {
  for (int64_t row_i = blockIdx.y; row_i < a.rows; row_i += gridDim.y) {
    int64_t i = row_i;
    const Seg run = a.run[find_run(a, &i)];
    const int64_t r = a.order[run.row_begin + i];
    const int64_t e0 = a.rowptr[r], n = (a.rowptr[r + 1] - e0) * a.heads;
    for (int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x; t < n; t += (int64_t)gridDim.x * kBlock) {
      const int64_t e = e0 + t / a.heads;
      const int head = (int)(t % a.heads);
      const float s = a.s_src[(int64_t)a.colidx[e] * a.heads + head] + a.s_dst[r * a.heads + head];
      const float logit = s >= 0.0f ? s : a.slope * s;
      const double m = a.fin[(row_i * a.heads + head) * 2], l = a.fin[(row_i * a.heads + head) * 2 + 1];
      a.alpha[e * a.heads + head] = (float)((double)exp_fast(logit - (float)m) / l);
    }
  }
}

template <int VEC, int LH>
int launch_gat(const GatArgs& a, uint64_t grid, hipStream_t stream) {
  const int g = a.sl.g_log2;
  if (g == 6) {
    hipLaunchKernelGGL((gat_aggregate_kernel<VEC, MODE_WAVE, LH>), dim3((unsigned)grid), dim3(kBlock), 0, stream, a);
  } else if (g >= 3) {
    hipLaunchKernelGGL((gat_aggregate_kernel<VEC, MODE_WIDE, LH>), dim3((unsigned)grid), dim3(kBlock), 0, stream, a);
  } else {
    hipLaunchKernelGGL((gat_aggregate_kernel<VEC, MODE_NARROW, LH>), dim3((unsigned)grid), dim3(kBlock), 0, stream,
                       a);
  }
  return hipGetLastError() == hipSuccess ? GNNAGG_OK : GNNAGG_EDEVICE;
}

// Lanes per head when the source score can be recomputed in registers, else 0.  Needs 16-byte lanes, a
// head of 1, 2 or 4 lanes, and slices that are whole heads (then a head's lanes are adjacent, aligned,
// and either all own columns or none does).
inline int lanes_per_head_fused(const SliceLaunch& sl, int32_t C) {
  if (sl.vec != 4 || C % 4) return 0;
  const int lh = C / 4;
  if (lh != 1 && lh != 2 && lh != 4) return 0;
  if (sl.sub_w % C || sl.chunk_w % C || sl.c_begin % C || sl.chunk_stride % C) return 0;
  return lh;
}

}  // namespace
}  // namespace gnnagg

using namespace gnnagg;

extern "C" int gnnagg_gat_attention(int64_t N, const int64_t* rowptr, const int32_t* colidx, const float* H,
                                    const float* a_src, const float* a_dst, int32_t heads, int32_t C,
                                    float negative_slope, float* alpha, float* out, int32_t f_chunk,
                                    const int32_t* row_order, const int64_t* class_off, void* workspace,
                                    size_t* workspace_bytes, void* stream_) {
  if (N < 0 || heads <= 0 || C <= 0 || f_chunk < 0) return GNNAGG_EINVAL;
  if ((int64_t)heads * C > 0x3fffffffll) return GNNAGG_EINVAL;  // a row of H stays below 2^32 bytes
  if (!(negative_slope == negative_slope)) return GNNAGG_EINVAL;
  const int32_t F = heads * C;
  if (f_chunk > 0 && f_chunk < F && (f_chunk % C) != 0) return GNNAGG_EINVAL;  // a chunk may not split a head
  if (!workspace_bytes) return GNNAGG_ENULL;
  if (N >= (1ll << 31)) return GNNAGG_EUNSUPPORTED;
  if ((row_order == nullptr) != (class_off == nullptr)) return GNNAGG_EINVAL;
  // rows long enough to be split (they exist only with a plan): slots for the pieces, finals per row
  SegTable probe;
  {
    int rc = build_segments(class_off, N, 6, true, &probe);  // the split runs do not depend on the slice width
    if (rc != GNNAGG_OK) return rc;
  }
  int64_t split_rows = 0;
  for (int k = 0; k < probe.nseg; ++k)
    if (probe.seg[k].split_log2 > 0) split_rows += (int64_t)probe.seg[k].row_end - probe.seg[k].row_begin;
  Carver carve(workspace);
  float* s_src = carve.take<float>((size_t)(N > 0 ? N : 1) * heads);
  float* s_dst = carve.take<float>((size_t)(N > 0 ? N : 1) * heads);
  double* pieces = nullptr;
  double* fin = nullptr;
  if (probe.ws_slots > 0) {
    pieces = carve.take<double>((size_t)probe.ws_slots * ((size_t)F + 2 * (size_t)heads));
    fin = carve.take<double>((size_t)split_rows * (size_t)heads * 2);
  }
  if (!workspace) {
    *workspace_bytes = carve.used;
    return GNNAGG_OK;
  }
  if (*workspace_bytes < carve.used || ((uintptr_t)workspace & 255u)) return GNNAGG_EWORKSPACE;
  if (N == 0) return GNNAGG_OK;
  if (!rowptr || !colidx || !H || !a_src || !a_dst) return GNNAGG_ENULL;
  if (!alpha && !out) return GNNAGG_OK;
  if (((uintptr_t)H % 4) || ((uintptr_t)rowptr % 8) || ((uintptr_t)colidx % 4) || ((uintptr_t)a_src % 4) ||
      ((uintptr_t)a_dst % 4) || (out && ((uintptr_t)out % 4)) || (alpha && ((uintptr_t)alpha % 4)))
    return GNNAGG_EINVAL;
  if (out == H) return GNNAGG_EINVAL;

  LaunchList launches;
  plan_columns(F, f_chunk, 4, C, 0, false, &launches);
  if (launches.overflow || launches.empty()) return GNNAGG_EUNSUPPORTED;
  // Heads of 4, 8 or 16 channels: both scores of an edge are recomputed from the row pieces the lanes hold,
  // so without alpha (whose second pass reads the score arrays) the score kernel and its arrays drop out
  // and the call is a single launch.
  bool need_scores = alpha != nullptr;
  for (size_t k = 0; k < launches.size(); ++k)
    if (!lanes_per_head_fused(launches[k], C)) need_scores = true;
  GatArgs args[kMaxLaunches];
  uint64_t grids[kMaxLaunches];
  for (size_t k = 0; k < launches.size(); ++k) {
    GatArgs& a = args[k];
    a.rowptr = rowptr;
    a.colidx = colidx;
    a.H = H;
    a.a_src = a_src;
    a.a_dst = a_dst;
    a.s_src = need_scores ? s_src : nullptr;
    a.s_dst = need_scores ? s_dst : nullptr;
    a.alpha = alpha;
    a.out = out;
    a.order = row_order;
    a.heads = heads;
    a.C = C;
    a.slope = negative_slope;
    a.N = N;
    a.pieces = pieces;
    a.sl = launches[k];
    if (a.sl.sub_w % a.sl.vec || a.sl.chunk_w % a.sl.vec) return GNNAGG_EINVAL;  // cannot happen: vec divides C
    int rc = build_segments(class_off, N, a.sl.g_log2, pieces != nullptr, &a.segs);
    if (rc != GNNAGG_OK) return rc;
    grids[k] = (uint64_t)a.segs.blocks_per_slice * (uint64_t)a.sl.n_chunks * (uint64_t)a.sl.n_sub;
    if (grids[k] == 0 || grids[k] > 0x7fffffffull) return GNNAGG_EUNSUPPORTED;
  }
  hipStream_t stream = (hipStream_t)stream_;
  const int64_t n_vh = N * heads;
  // one summation order for the whole call: groups of 4 channels if any launch recomputes scores
  int32_t grp = C;
  for (size_t k = 0; k < launches.size(); ++k)
    if (lanes_per_head_fused(launches[k], C)) grp = 4;
  if (need_scores) {
    hipLaunchKernelGGL(gat_scores_kernel, dim3((unsigned)ceil_div(n_vh, kBlock)), dim3(kBlock), 0, stream, H, a_src,
                       a_dst, n_vh, heads, C, grp, s_src, s_dst);
    GNNAGG_HIP_TRY(hipGetLastError());
  }
  for (size_t k = 0; k < launches.size(); ++k) {
    int rc;
    switch (args[k].sl.vec) {
      case 1: rc = launch_gat<1, 0>(args[k], grids[k], stream); break;
      case 2: rc = launch_gat<2, 0>(args[k], grids[k], stream); break;
      default:
        switch (lanes_per_head_fused(args[k].sl, C)) {
          case 1: rc = launch_gat<4, 1>(args[k], grids[k], stream); break;
          case 2: rc = launch_gat<4, 2>(args[k], grids[k], stream); break;
          case 4: rc = launch_gat<4, 4>(args[k], grids[k], stream); break;
          default: rc = launch_gat<4, 0>(args[k], grids[k], stream); break;
        }
        break;
    }
    if (rc != GNNAGG_OK) return rc;
  }
  if (pieces) {
    GatMergeArgs m;
    m.rowptr = rowptr;
    m.colidx = colidx;
    m.order = row_order;
    m.s_src = s_src;
    m.s_dst = s_dst;
    m.alpha = alpha;
    m.out = out;
    m.pieces = pieces;
    m.fin = fin;
    m.rows = split_rows;
    m.heads = heads;
    m.C = C;
    m.slope = negative_slope;
    m.nrun = 0;
    int max_split = 0;
    for (int k = 0; k < probe.nseg; ++k) {
      if (probe.seg[k].split_log2 == 0) continue;
      if (m.nrun >= kMaxSplitSeg) return GNNAGG_EUNSUPPORTED;  // cannot happen: build_segments caps them
      m.run[m.nrun++] = probe.seg[k];
      if (probe.seg[k].split_log2 > max_split) max_split = probe.seg[k].split_log2;
    }
    const int64_t blocks = ceil_div(split_rows * (int64_t)F, kBlock);
    if (blocks > 0x7fffffffll) return GNNAGG_EUNSUPPORTED;
    hipLaunchKernelGGL(gat_split_merge_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, stream, m);
    GNNAGG_HIP_TRY(hipGetLastError());
    if (alpha) {
      // enough blocks per row for the longest row a run can hold, capped; the kernel strides over the rest
      int64_t bx = ceil_div(((int64_t)1 << (max_split + kSplitLenLog2)) * heads, kBlock);
      if (bx > 4096) bx = 4096;
      const int64_t by = split_rows < 65535 ? split_rows : 65535;
      hipLaunchKernelGGL(gat_split_alpha_kernel, dim3((unsigned)bx, (unsigned)by), dim3(kBlock), 0, stream, m);
      GNNAGG_HIP_TRY(hipGetLastError());
    }
  }
  return GNNAGG_OK;
}
