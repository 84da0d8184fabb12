// Host-side scheduling shared by the aggregation and attention launches:
// how a column range is cut into feature slices, and how the degree classes of
// a row plan map onto lane groups.
//
// Feature decomposition (paper Algorithm 1) becomes a tiling of the launch
// grid: a work item is (row group, feature slice), and the slices of one chunk
// are enumerated chunk-major, so the hardware dispatcher walks the chunks in
// the paper's chunk-outer / vertex-inner order and the rows of X touched at
// any time are restricted to the current chunk's columns.
#pragma once
#include "common.hpp"

namespace gnnagg {

constexpr int kMaxSeg = 16;
constexpr int kMaxSplitSeg = 7;     // runs of split rows per table (the rest of kMaxSeg: 0..6 and 8 lanes log2)
constexpr int kSplitClass = 16;     // rows of degree class >= 16 (2^15 edges or more) may be split
constexpr int kSplitLenLog2 = 13;   // ... into pieces of 2^13 consecutive edges, one workgroup each

// A run of rows (positions in the row plan) handled with 2^lr_log2 lanes per
// row: lr_log2 in [g_log2, 6] = that many lanes of one wave; 8 = a whole
// 256-thread workgroup per row (hub rows; partials meet in LDS).
// split_log2 > 0 (only with lr_log2 == 8, only when the caller gave a workspace): every row of the run
// is walked by 2^split_log2 workgroups, piece p taking edges [p, p + 1) * 2^kSplitLenLog2 of the row;
// each piece leaves its partial result in workspace slot ws_begin + (row - row_begin) * 2^split_log2 + p
// and a merge kernel folds the slots in order.  Without this a row of millions of edges is one
// workgroup's serial walk and sets the run time of the whole call.
struct Seg {
  int32_t row_begin, row_end;
  int32_t blk_begin;  // first workgroup of this run inside one slice's block range
  int32_t lr_log2;
  int32_t split_log2;
  int32_t ws_begin;
};

struct SegTable {
  int32_t nseg;
  uint32_t blocks_per_slice;
  int32_t ws_slots;  // partial-result slots the split runs need (0: nothing is split)
  Seg seg[kMaxSeg];
};

// One launch: n_chunks chunks of equal width chunk_w starting every
// chunk_stride columns from c_begin; each chunk is cut into n_sub slices of
// sub_w columns (the last one may be narrower, never narrower than vec).
// A lane owns vec consecutive columns; 2^g_log2 lanes span one slice.
struct SliceLaunch {
  int32_t c_begin, chunk_stride, chunk_w, n_chunks, sub_w, n_sub, vec, g_log2;
};

// The launches of one call: a fixed-capacity list, so that planning a call touches no heap (a chunk
// yields at most two groups of columns, a group at most one sliver group, a group at most two launches).
constexpr int kMaxLaunches = 16;
struct LaunchList {
  SliceLaunch v[kMaxLaunches];
  int n = 0;
  bool overflow = false;
  void clear() { n = 0; overflow = false; }
  void push_back(const SliceLaunch& s) {
    if (n < kMaxLaunches) v[n++] = s;
    else overflow = true;
  }
  size_t size() const { return (size_t)n; }
  bool empty() const { return n == 0; }
  const SliceLaunch& operator[](size_t k) const { return v[k]; }
  const SliceLaunch* begin() const { return v; }
  const SliceLaunch* end() const { return v + n; }
};

// What one thread of a launch does: which row (position in the plan), which
// columns, which neighbour slot.  The same function runs in the kernels and in
// the host-side coverage test.
struct LaneRole {
  int64_t ridx;   // position in the row plan (valid if row_ok)
  int32_t col;    // first of the lane's vec columns
  int32_t W;      // width of the slice this workgroup works on
  int32_t ng;     // neighbour slot: the lane visits edges e0+ng, e0+ng+P, ...
  int32_t P;      // neighbour slots per row
  int32_t L;      // log2 lanes per row (8 = whole workgroup)
  int32_t g;      // log2 lanes per slice
  bool row_ok;    // the lane has a row
  bool col_ok;    // the lane has columns
  bool hub;       // the row owns the whole workgroup
  bool writer;    // the lane stores the merged result for its columns
  int32_t split_log2;  // > 0: the workgroup walks one piece of a split row ...
  int32_t piece;       // ... this piece ...
  int32_t ws_slot;     // ... and stores its partial result in this workspace slot instead of `out`
};

__host__ __device__ inline LaneRole lane_role(const SliceLaunch& sl, const SegTable& segs, uint32_t block,
                                              int tid) {
  LaneRole r;
  const int lane = tid & (kWave - 1), wv = tid / kWave;
  const uint32_t slice = block / segs.blocks_per_slice;
  uint32_t lb = block - slice * segs.blocks_per_slice;
  const int chunk = (int)(slice / (uint32_t)sl.n_sub);
  const int sub = (int)(slice - (uint32_t)chunk * (uint32_t)sl.n_sub);
  const int w_off = sub * sl.sub_w;
  const int rest = sl.chunk_w - w_off;
  r.W = sl.sub_w < rest ? sl.sub_w : rest;
  const int c0 = sl.c_begin + chunk * sl.chunk_stride + w_off;

  int32_t row_begin = segs.seg[0].row_begin, row_end = segs.seg[0].row_end;
  int32_t blk_begin = segs.seg[0].blk_begin, L = segs.seg[0].lr_log2;
  int32_t split = segs.seg[0].split_log2, ws_begin = segs.seg[0].ws_begin;
#pragma unroll
  for (int k = 1; k < kMaxSeg; ++k) {
    if (k < segs.nseg && lb >= (uint32_t)segs.seg[k].blk_begin) {
      row_begin = segs.seg[k].row_begin;
      row_end = segs.seg[k].row_end;
      blk_begin = segs.seg[k].blk_begin;
      L = segs.seg[k].lr_log2;
      split = segs.seg[k].split_log2;
      ws_begin = segs.seg[k].ws_begin;
    }
  }
  lb -= (uint32_t)blk_begin;
  r.L = L;
  r.g = sl.g_log2;
  r.hub = (L == 8);
  r.split_log2 = split;
  r.piece = (int32_t)(lb & ((1u << split) - 1u));
  r.ws_slot = ws_begin + (int32_t)lb;  // (row - row_begin) * 2^split + piece
  int64_t slot;
  int sub_lane;
  if (r.hub) {
    slot = lb >> split;
    sub_lane = tid;
  } else {
    slot = ((((int64_t)lb * kWavesPerBlock) + wv) << (6 - L)) + (lane >> L);
    sub_lane = lane & ((1 << L) - 1);
  }
  const int gl = sub_lane & ((1 << r.g) - 1);  // position inside the slice
  r.ng = sub_lane >> r.g;
  r.P = (r.hub ? kBlock : (1 << L)) >> r.g;
  r.ridx = (int64_t)row_begin + slot;
  r.row_ok = r.ridx < (int64_t)row_end;
  r.col_ok = sl.vec * gl < r.W;
  // the last lane of a ragged slice re-reads the slice's final vec columns
  const int shift = sl.vec * gl < r.W - sl.vec ? sl.vec * gl : r.W - sl.vec;
  r.col = c0 + shift;
  r.writer = r.row_ok && r.col_ok && r.ng == 0;
  return r;
}

inline int pow2_ceil_log2(int64_t x) {
  int l = 0;
  while ((1ll << l) < x) ++l;
  return l;
}

// Cuts [0,F) into chunks of width f_chunk (0 or >= F: one chunk) and every
// chunk into slices of at most 64 lanes x vec columns.  max_vec is the widest
// per-lane vector (16 bytes of input); vec_multiple forces vec to divide it
// (attention: a lane must stay inside one head) or is 0; line_cols is the number
// of columns in a 128-byte line if every row of the input starts on a line
// boundary, else 0; tail_launch asks for a separate launch for a narrower last
// slice (worth its launch only where the resident-workgroup cap is in play).
inline void plan_columns(int32_t F, int32_t f_chunk, int max_vec, int vec_multiple, int line_cols,
                         bool tail_launch, LaunchList* out) {
  out->clear();
  const int32_t width = (f_chunk <= 0 || f_chunk >= F) ? F : f_chunk;
  struct Group { int32_t c_begin, n_chunks, chunk_w; };
  Group groups[4];  // the full-width chunks, the narrower last chunk, and at most one sliver of the group in work
  int n_groups = 0;
  if (F / width > 0) groups[n_groups++] = {0, F / width, width};
  if (F % width) groups[n_groups++] = {(F / width) * width, 1, F % width};
  while (n_groups > 0) {
    Group gr = groups[--n_groups];
    int vec = max_vec;
    while (vec > 1 && (vec > gr.chunk_w || (vec_multiple && vec_multiple % vec))) vec >>= 1;
    const int32_t cap = kWave * vec;
    int32_t n_sub = (int32_t)ceil_div(gr.chunk_w, cap);
    int32_t sub_w = (int32_t)(ceil_div(ceil_div(gr.chunk_w, n_sub), vec) * vec);
    if (line_cols > 0 && n_sub > 1 && gr.c_begin % line_cols == 0 && (gr.n_chunks == 1 || width % line_cols == 0)) {
      // rows start on 128-byte lines: cut the slices at line boundaries too, so that no line is fetched
      // by two slice passes (F=602 fp32: 224/224/154 columns = 7+7+5 lines instead of 3 x 7)
      const int32_t al = (int32_t)(ceil_div(ceil_div(gr.chunk_w, n_sub), line_cols) * line_cols);
      if (al <= cap && al % vec == 0 && gr.chunk_w - (n_sub - 1) * al >= vec) sub_w = al;
    }
    int32_t last = gr.chunk_w - (n_sub - 1) * sub_w;
    if (last < vec) {  // balanced cut left a sliver: use full-width slices instead
      sub_w = cap;
      n_sub = (int32_t)ceil_div(gr.chunk_w, cap);
      last = gr.chunk_w - (n_sub - 1) * sub_w;
      if (last < vec) {  // give the sliver a launch of its own with a narrower vector
        // the sliver repeats once per chunk, chunk_stride apart: it keeps the stride of the parent
        groups[n_groups++] = {gr.c_begin + (n_sub - 1) * sub_w, gr.n_chunks, last};
        gr.chunk_w = (n_sub - 1) * sub_w;
        n_sub -= 1;
      }
    }
    SliceLaunch sl;
    sl.c_begin = gr.c_begin;
    sl.chunk_stride = width;
    sl.chunk_w = gr.chunk_w;
    sl.n_chunks = gr.n_chunks;
    sl.sub_w = sub_w;
    sl.n_sub = n_sub;
    sl.vec = vec;
    sl.g_log2 = pow2_ceil_log2(ceil_div(sub_w, vec));
    if (tail_launch && sl.n_sub > 1 && sl.n_chunks == 1 && last < sub_w) {
      // the narrower last slice gets a launch of its own, after the others: its waves have fewer active
      // lanes, so its best number of resident workgroups differs (resident_workgroup_cap)
      SliceLaunch tail = sl;
      sl.chunk_w = (n_sub - 1) * sub_w;
      sl.n_sub = n_sub - 1;
      tail.c_begin = sl.c_begin + sl.chunk_w;
      tail.chunk_w = last;
      tail.sub_w = last;
      tail.n_sub = 1;
      tail.g_log2 = pow2_ceil_log2(ceil_div(last, vec));
      out->push_back(sl);
      out->push_back(tail);
      continue;
    }
    out->push_back(sl);
  }
}

// Maps degree classes to lane groups for slices spanned by 2^g_log2 lanes.
// A row of degree d gets about d/8 to d/64 neighbour slots (a power of two; the wider the slot, the more
// edges it should walk before its partial result is worth a merge); beyond what a wave offers the row moves
// to a whole workgroup.  Without a plan every row gets one wave.
inline int build_segments(const int64_t* class_off, int64_t N, int g_log2, bool allow_split, SegTable* t) {
  t->nseg = 0;
  t->ws_slots = 0;
  int64_t blocks = 0, ws = 0;
  int n_split = 0;
  auto rows_per_block = [](int L) -> int64_t { return L == 8 ? 1 : (int64_t)kWavesPerBlock << (6 - L); };
  auto push = [&](int64_t rb, int64_t re, int L, int split) {
    if (re <= rb) return;
    if (t->nseg > 0) {
      // extend the previous run if it is of the same kind.  A split run is extended only when the table
      // has no room for another one (the rows added are shorter, so its piece count covers them).
      Seg& s = t->seg[t->nseg - 1];
      const bool same = s.lr_log2 == L && ((split == 0 && s.split_log2 == 0) ||
                                           (split > 0 && s.split_log2 > 0 && n_split >= kMaxSplitSeg));
      if (same) {
        blocks = s.blk_begin;
        ws = s.ws_begin;
        s.row_end = (int32_t)re;
        const int64_t rows = (int64_t)s.row_end - s.row_begin;
        if (s.split_log2 > 0) {
          blocks += rows << s.split_log2;
          ws += rows << s.split_log2;
        } else {
          blocks += ceil_div(rows, rows_per_block(L));
        }
        return;
      }
    }
    Seg& s = t->seg[t->nseg++];
    s.row_begin = (int32_t)rb;
    s.row_end = (int32_t)re;
    s.blk_begin = (int32_t)blocks;
    s.lr_log2 = L;
    s.split_log2 = split;
    s.ws_begin = (int32_t)ws;
    if (split > 0) {
      ++n_split;
      blocks += (re - rb) << split;
      ws += (re - rb) << split;
    } else {
      blocks += ceil_div(re - rb, rows_per_block(L));
    }
  };
  if (!class_off) {
    push(0, N, 6, 0);
  } else {
    if (class_off[0] != 0 || class_off[GNNAGG_PLAN_CLASSES] != N) return GNNAGG_EINVAL;
    for (int k = 0; k < GNNAGG_PLAN_CLASSES; ++k)
      if (class_off[k] > class_off[k + 1]) return GNNAGG_EINVAL;
    for (int k = 0; k < GNNAGG_PLAN_CLASSES; ++k) {
      const int c = 32 - k;                      // rows with 2^(c-1) <= degree < 2^c
      // edges a neighbour slot should at least walk (log2): 8 where a slot is 1-4 lanes, 32 where it is 8-32
      // lanes, 64 where it is a whole wavefront - measured: against 8 everywhere, 5-8 % on the two large
      // benchmark graphs and on attention; slots of 1-4 lanes lose 1-2 % with more than 8
      const int per_slot_log2 = g_log2 <= 2 ? 3 : (g_log2 == 6 ? 6 : 5);
      const int p_log2 = c > per_slot_log2 ? c - 1 - per_slot_log2 : 0;
      int L = g_log2 + p_log2;
      L = (L >= 8) ? 8 : (L > 6 ? 6 : L);
      const int split = (allow_split && L == 8 && c >= kSplitClass) ? c - kSplitLenLog2 : 0;
      push(class_off[k], class_off[k + 1], L, split);
      if (blocks > 0x7fffffffll || ws > 0x7fffffffll) return GNNAGG_EUNSUPPORTED;
    }
  }
  if (blocks > 0x7fffffffll || t->nseg > kMaxSeg) return GNNAGG_EUNSUPPORTED;
  t->blocks_per_slice = (uint32_t)blocks;
  t->ws_slots = (int32_t)ws;
  return GNNAGG_OK;
}

// Mean degree and the share of all edges that end in the `hot_rows` longest rows, both estimated from
// the plan's degree classes (a row of class c counts as 1.5 * 2^(c-1) - 0.5 edges).
inline void degree_profile(const int64_t* class_off, int64_t N, int64_t hot_rows, double* mean_degree,
                           double* hot_share) {
  double edges = 0.0, hot = 0.0;
  int64_t left = hot_rows;
  for (int k = 0; k < GNNAGG_PLAN_CLASSES; ++k) {  // classes 32 down to 0: longest rows first
    const int c = 32 - k;
    if (c == 0) continue;
    const double mid = 1.5 * (double)(1ull << (c - 1)) - 0.5;
    const int64_t rows = class_off[k + 1] - class_off[k];
    edges += mid * (double)rows;
    const int64_t take = rows < left ? rows : left;
    hot += mid * (double)take;
    left -= take;
  }
  *mean_degree = N > 0 ? edges / (double)N : 0.0;
  *hot_share = edges > 0.0 ? hot / edges : 0.0;
}

// Chunk width for GNNAGG_F_CHUNK_AUTO: the paper leaves the number of layers to the memory capacity of
// the device and the character of the dataset (Section II-B).  What the sweeps on MI355X say (power-law
// graphs of 45,000-2,400,000 rows, mean degree 8-600, 64-2048 columns; bench.py --validate-auto prints the
// regret of this choice per shape, for the benchmark graphs and for shapes the rule was not derived on):
//  (1) Rows on 128-byte lines, at least four lines wide, more than 32,768 rows (as many as one 4 MB L2 holds
//      lines), mean degree >= 16 and hubs that matter (the 32,768 longest rows take >= 40 % of the edges):
//      row pieces of one or a few LINES.  A pass then gathers from a column slice of N x piece bytes in
//      which the hubs' lines stay in L2.
//        - fp32: one line per piece (10-40 % faster than one chunk at 45,000-1,500,000 rows; two-line
//          pieces are up to 10 % ahead of it where they win and up to 23 % behind where they lose);
//        - short rows: every pass pays a chain of dependent loads per row (plan, row pointer, indices) that
//          few edges do not amortise - at mean degree 50 and 45-64 passes two- to four-line pieces are
//          3-12 % faster than one-line ones - so at least ~75 / (mean degree) lines (a power of two), but
//          only while the slice stays within about half the 256 MB Infinity Cache (700,000 rows of mean
//          degree 30: one line, a 90 MB slice, is 14-27 % faster than two or four);
//        - bf16: two lines (a one-line pass accumulates eight columns per lane in fp64 and is bound by that
//          arithmetic, 4-7 % slower on the largest bf16 shapes) - two lines are within 7 % of the
//          best width on every bf16 shape tried).
//  (2) Otherwise, X beyond ~1 GiB (several times the Infinity Cache; 2.4 M rows x 256-512 fp32 columns):
//      chunks whose column slice is ~300-600 MB are 13-17 % faster than one chunk, row pieces under 128
//      bytes twice slower than either -> power-of-two width with a ~384 MB slice, >= 128-byte pieces.
//  (3) Otherwise one chunk: uniform graphs (hot share < 0.2) lose 3-9 % to the extra passes over the edge
//      list, and without line-aligned rows a piece straddles an extra line and every pass costs more.
inline int64_t pow2_floor(double x) {
  int64_t p = 1;
  while ((double)(2 * p) <= x) p *= 2;
  return p;
}

inline int32_t auto_f_chunk(int64_t N, int32_t F, int elem_bytes, bool rows_on_lines, const int64_t* class_off) {
  const double x_bytes = (double)N * (double)F * (double)elem_bytes;
  if (N <= 0) return F;
  constexpr int64_t kLinesPerL2 = 4 * 1024 * 1024 / 128;
  const int64_t line_cols = 128 / elem_bytes;
  if (rows_on_lines && F >= 4 * line_cols && class_off && N > kLinesPerL2) {
    double mean_degree, hot_share;
    degree_profile(class_off, N, kLinesPerL2, &mean_degree, &hot_share);
    if (mean_degree >= 16.0 && hot_share >= 0.4) {
      const double line_slice = (double)N * 128.0;  // bytes of a column slice one line wide
      int64_t lines = 1;
      while (lines < 8 && (double)lines * mean_degree < 75.0) lines *= 2;
      const int64_t in_cache = pow2_floor(128.0e6 / line_slice);
      if (lines > in_cache) lines = in_cache;
      if (elem_bytes < 4 && lines < 2) lines = 2;
      const int64_t w = lines * line_cols;
      return (int32_t)(w >= F ? F : w);
    }
  }
  if (x_bytes > 1024.0 * 1024.0 * 1024.0) {
    const int64_t min_w = 128 / elem_bytes;                                  // 128-byte row pieces
    const int64_t p = pow2_floor(384.0 * 1024.0 * 1024.0 / ((double)N * elem_bytes) / (double)min_w) * min_w;
    return (int32_t)(p >= F ? F : p);  // a power of two keeps every chunk on full 16-byte lanes
  }
  return F;
}

// Whether a graph is worth aggregating over source blocks (gnnagg_aggregate_blocked), and over how many.
// A blocked run re-reads B times fewer rows of X per pass, so more of the gathers hit L2, and pays for it
// with the states in transit: 16 bytes per output element and block boundary, written and read back.  The
// gathers outweigh that only when a row has many edges: on power-law graphs of 50,000-1,500,000 rows
// (bench.py --validate-auto times 2, 4 and 8 blocks at pieces of 1, 2 and 4 lines next to the plain call)
// fp32 shapes of mean degree 200-600 and at least 100,000 rows run 3-23 % faster blocked, with two-line
// pieces, than the plain call at its best width; at mean degree 150 and below, on smaller graphs and with
// bf16 rows (whose plain passes are not bound by L2 misses) the plain call wins, by 5-70 %.
// How many: the plain call already keeps the hubs' lines in L2, so what blocks add depends on how much of
// the graph is NOT hubs.  Where the longest tenth of the rows holds under 60 % of the edges (flat degree
// distributions: the third benchmark graph shape, exponents above 2) 4 blocks beat 2 by 5-30 %; where it
// holds over 70 % 2 blocks beat 4 by 4-11 %.  In between the weighted sum is level (its passes also stream
// the edge weights, which blocks do not help), while sum, mean and max still gain 3-9 % from 4.  8 and more
// lose to the traffic of the states everywhere.  Returns 1 for "do not block".
inline int32_t auto_source_blocks(int64_t N, int64_t F, int elem_bytes, bool rows_on_lines, bool weighted,
                                  const int64_t* class_off) {
  if (!class_off || !rows_on_lines || elem_bytes != 4 || F < 128 || N < 100000) return 1;
  double mean_degree, top_tenth_share;
  degree_profile(class_off, N, N / 10, &mean_degree, &top_tenth_share);
  if (mean_degree < 200.0) return 1;
  return top_tenth_share < (weighted ? 0.6 : 0.7) ? 4 : 2;
}

// How many workgroups of the aggregation kernel should share a compute unit.  Every resident wave
// keeps eight row gathers in flight, and every line in flight occupies L2; at full occupancy the lines
// in flight alone (256 CUs x 16-20 waves x 8 x ~7 lines x 128 B = ~30 MB) are as large as the whole L2
// (8 x 4 MB), so nothing that was fetched stays long enough to serve a second destination.  On dense
// graphs, where a row of X is gathered hundreds of times, fewer resident waves mean more L2 hits and
// a shorter run; on sparse graphs and narrow slices the parallelism is worth more.
//
// What the sweeps on MI355X show (dense graphs, mean degree 190-600, 128 to 602 fp32 / 200 to 512 bf16
// columns, caps 2-5 and none) is an optimum in BYTES IN FLIGHT PER COMPUTE UNIT: a workgroup has
// 4 waves x 8 loads x (active lanes per wave) x 16 B in flight, and the best cap is the one that
// brings cap x that to about 56 KB for the weighted sum (whose loop also streams the edge weights)
// and about 78 KB for sum / mean / max.  64 active lanes: 2 and 2; 56: 2 and 3; 48: 2 and 3; 39: 3 and 4
// - each the measured best, by 5-25 % over its neighbours.  Slices of at most 16 lanes (wide mode with
// four or more rows per wave) ran best uncapped.  The mean degree is estimated from the plan's degree
// classes; active_lanes is the launch's average over its slices.  Returns 0 for "no cap".
inline int resident_workgroup_cap(const int64_t* class_off, int64_t N, int g_log2, int active_lanes,
                                  bool weighted) {
  if (!class_off || N <= 0 || g_log2 < 5 || active_lanes <= 0) return 0;
  double edges = 0.0;
  for (int k = 0; k < GNNAGG_PLAN_CLASSES; ++k) {
    const int c = 32 - k;  // rows with 2^(c-1) <= degree < 2^c
    if (c == 0) continue;
    const double mid = 1.5 * (double)(1ull << (c - 1)) - 0.5;
    edges += mid * (double)(class_off[k + 1] - class_off[k]);
  }
  const double mean_degree = edges / (double)N;
  if (mean_degree < (g_log2 == 6 ? 96.0 : 384.0)) return 0;
  const double target = (g_log2 == 6 && weighted) ? 56.0 * 1024.0 : 78.0 * 1024.0;
  const double per_workgroup = (double)kWavesPerBlock * 8.0 * (double)active_lanes * 16.0;
  int cap = (int)(target / per_workgroup + 0.5);
  return cap < 2 ? 2 : (cap > 4 ? 4 : cap);
}

// Active lanes per wave of a launch, averaged over its slices: lanes that own columns, times the rows a
// wave holds side by side when a slice is narrower than the wave.
inline int active_lanes_per_wave(const SliceLaunch& sl) {
  const int64_t lanes_per_chunk = ceil_div(sl.chunk_w, sl.vec);
  const int per_slice = (int)ceil_div(lanes_per_chunk, sl.n_sub);  // <= 2^g_log2
  return per_slice << (6 - sl.g_log2);
}

// LDS a workgroup has to occupy so that exactly `cap` workgroups fit in the 160 KB of a gfx950
// compute unit (cap + 1 must not fit; 1 KB of slack covers the allocation granularity).
inline uint32_t lds_claim(int cap) {
  constexpr uint32_t kLdsPerCu = 160 * 1024;
  if (cap <= 0) return 0;
  const uint32_t claim = kLdsPerCu / (uint32_t)(cap + 1) + 1024;
  return claim > 64 * 1024 ? 64 * 1024 : claim;  // what a launch may request without opting in to more
}

}  // namespace gnnagg
