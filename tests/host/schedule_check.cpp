// Host-side check of the launch geometry used by the aggregation kernels:
// replays lane_role() for every thread of every workgroup of every launch and
// verifies that (1) every (row, column) of the output has a writer, (2) columns
// written twice come only from the ragged tail lane of the same workgroup,
// (3) for every row and slice position the neighbour slots 0..P-1 each appear
// exactly once, and (4) every column a lane touches lies inside [0, F).  With use_plan == 2 rows of the
// long degree classes are split into pieces: then (5) such a row has no writer into the output, its
// 2^split pieces each cover every column in a workspace slot of their own, and slots are unique.
//
// usage: schedule_check F f_chunk max_vec vec_multiple[:line_cols] N use_plan [class counts ...]
//        (use_plan: 0 none, 1 plan, 2 plan with split rows; class counts: rows in class 32, 31, ..., 0;
//        must add up to N)
#include <cstdio>
#include <cstdlib>
#include <map>
#include <vector>

#include "schedule.hpp"

using namespace gnnagg;

int main(int argc, char** argv) {
  if (argc < 7) return 2;
  const int32_t F = atoi(argv[1]), f_chunk = atoi(argv[2]);
  const int max_vec = atoi(argv[3]), vec_multiple = atoi(argv[4]);
  int line_cols = 0;
  for (const char* c = argv[4]; *c; ++c)
    if (*c == ':') line_cols = atoi(c + 1);
  const int64_t N = atoll(argv[5]);
  const int use_plan = atoi(argv[6]);
  int64_t class_off[GNNAGG_PLAN_CLASSES + 1];
  if (use_plan) {
    if (argc != 7 + GNNAGG_PLAN_CLASSES) return 2;
    class_off[0] = 0;
    for (int k = 0; k < GNNAGG_PLAN_CLASSES; ++k) class_off[k + 1] = class_off[k] + atoll(argv[7 + k]);
    if (class_off[GNNAGG_PLAN_CLASSES] != N) { printf("FAIL class counts do not add up\n"); return 1; }
  }
  LaunchList launches;
  plan_columns(F, f_chunk, max_vec, vec_multiple, line_cols, use_plan != 0, &launches);
  if (launches.overflow || launches.empty()) { printf("FAIL launch list overflow or empty\n"); return 1; }
  if (line_cols)
    for (const SliceLaunch& sl : launches)
      if (sl.n_sub > 1 && sl.c_begin % line_cols == 0 && (sl.n_chunks == 1 || sl.chunk_stride % line_cols == 0) &&
          sl.sub_w % line_cols) {
        // not an error in itself (the aligned width may not fit), but the cases this test passes all fit
        printf("FAIL slices of %d columns do not end on lines of %d\n", sl.sub_w, line_cols);
        return 1;
      }
  std::vector<int> writers((size_t)N * F, 0);
  std::vector<char> is_split((size_t)N, 0);
  std::map<int32_t, std::pair<int64_t, int>> slot_owner;   // workspace slot -> (row, piece)
  std::map<std::pair<int32_t, int>, int> slot_cols;        // (slot, column) -> writers
  int32_t ws_slots = -1;
  for (const SliceLaunch& sl : launches) {
    if (sl.vec < 1 || sl.sub_w < sl.vec || (1 << sl.g_log2) * sl.vec < sl.sub_w || sl.g_log2 > 6) {
      printf("FAIL bad slice launch vec=%d sub_w=%d g=%d\n", sl.vec, sl.sub_w, sl.g_log2);
      return 1;
    }
    if (sl.chunk_w - (sl.n_sub - 1) * sl.sub_w < sl.vec) { printf("FAIL last slice narrower than vec\n"); return 1; }
    if (vec_multiple && (vec_multiple % sl.vec)) { printf("FAIL vec does not divide %d\n", vec_multiple); return 1; }
    SegTable segs;
    int rc = build_segments(use_plan ? class_off : nullptr, N, sl.g_log2, use_plan == 2, &segs);
    if (rc != 0) { printf("FAIL build_segments rc=%d\n", rc); return 1; }
    if (segs.nseg < 1 || segs.nseg > kMaxSeg) { printf("FAIL nseg=%d\n", segs.nseg); return 1; }
    if (ws_slots >= 0 && ws_slots != segs.ws_slots) { printf("FAIL slot count differs between launches\n"); return 1; }
    ws_slots = segs.ws_slots;
    if (use_plan != 2 && ws_slots != 0) { printf("FAIL split without permission\n"); return 1; }
    const uint64_t grid = (uint64_t)segs.blocks_per_slice * sl.n_chunks * sl.n_sub;
    for (uint64_t b = 0; b < grid; ++b) {
      // (row position, first column) -> list of neighbour slots seen, within this workgroup
      std::map<std::pair<int64_t, int>, std::vector<int>> slots;
      std::map<std::pair<int64_t, int>, int> wcount;  // (row, column) -> writers inside this workgroup
      for (int tid = 0; tid < kBlock; ++tid) {
        const LaneRole r = lane_role(sl, segs, (uint32_t)b, tid);
        if (r.L < r.g || r.L > 8 || r.L == 7) { printf("FAIL L=%d g=%d\n", r.L, r.g); return 1; }
        if (!r.row_ok || !r.col_ok) {
          if (r.writer) { printf("FAIL idle lane marked writer\n"); return 1; }
          continue;
        }
        if (r.ridx < 0 || r.ridx >= N) { printf("FAIL row %lld out of range\n", (long long)r.ridx); return 1; }
        if (r.col < 0 || r.col + sl.vec > F) { printf("FAIL col %d out of range\n", r.col); return 1; }
        if (r.ng < 0 || r.ng >= r.P) { printf("FAIL slot %d of %d\n", r.ng, r.P); return 1; }
        if (vec_multiple && (r.col / vec_multiple) != ((r.col + sl.vec - 1) / vec_multiple)) {
          printf("FAIL lane straddles a head at col %d\n", r.col);
          return 1;
        }
        // the lane position inside the slice is what distinguishes groups; use (ridx, tid mod 2^g)
        slots[{r.ridx, tid & ((1 << r.g) - 1)}].push_back(r.ng);
        if (r.split_log2 > 0) {
          if (!r.hub) { printf("FAIL split row is not a hub row\n"); return 1; }
          if (r.piece < 0 || r.piece >= (1 << r.split_log2)) { printf("FAIL piece %d\n", r.piece); return 1; }
          if (r.ws_slot < 0 || r.ws_slot >= segs.ws_slots) { printf("FAIL slot %d of %d\n", r.ws_slot, segs.ws_slots); return 1; }
          is_split[(size_t)r.ridx] = 1;
          auto own = slot_owner.find(r.ws_slot);
          if (own == slot_owner.end()) slot_owner[r.ws_slot] = {r.ridx, r.piece};
          else if (own->second != std::make_pair(r.ridx, (int)r.piece)) { printf("FAIL slot %d shared\n", r.ws_slot); return 1; }
          // the piece must lie where the row's degree class says: piece * 2^kSplitLenLog2 < 2^class
          if (r.writer)
            for (int k = 0; k < sl.vec; ++k) slot_cols[{r.ws_slot, r.col + k}] += 1;
          continue;
        }
        if (r.writer) {
          if (r.hub && tid >= kWave) { printf("FAIL hub writer outside wave 0\n"); return 1; }
          for (int k = 0; k < sl.vec; ++k) {
            writers[(size_t)r.ridx * F + r.col + k] += 1;
            wcount[{r.ridx, r.col + k}] += 1;
          }
        }
      }
      for (auto& kv : slots) {
        std::vector<int>& v = kv.second;
        std::vector<int> seen(v.size(), 0);
        const LaneRole any = lane_role(sl, segs, (uint32_t)b, 0);
        (void)any;
        for (int s : v) {
          if (s >= (int)v.size() || seen[s]) { printf("FAIL neighbour slots not a permutation\n"); return 1; }
          seen[s] = 1;
        }
      }
      for (auto& kv : wcount)
        if (kv.second > 2) { printf("FAIL column written %d times in one workgroup\n", kv.second); return 1; }
    }
  }
  // split rows: every piece of every such row covers every column in its slot
  long long split_rows = 0;
  if (use_plan == 2) {
    if ((int64_t)slot_owner.size() != ws_slots) { printf("FAIL %zu slots used of %d\n", slot_owner.size(), ws_slots); return 1; }
    for (auto& kv : slot_owner)
      for (int32_t c = 0; c < F; ++c) {
        auto it = slot_cols.find({kv.first, c});
        if (it == slot_cols.end() || it->second > 2) { printf("FAIL slot %d column %d\n", kv.first, c); return 1; }
      }
    // a row of class c (position known from class_off) must own 2^(c - kSplitLenLog2) pieces or more
    std::map<int64_t, int> pieces;
    for (auto& kv : slot_owner) pieces[kv.second.first] += 1;
    for (int k = 0; k < GNNAGG_PLAN_CLASSES; ++k) {
      const int c = 32 - k;
      for (int64_t r = class_off[k]; r < class_off[k + 1]; ++r) {
        if (c >= kSplitClass) {
          if (!is_split[(size_t)r] || pieces[r] < (1 << (c - kSplitLenLog2))) { printf("FAIL row %lld class %d has %d pieces\n", (long long)r, c, pieces[r]); return 1; }
          ++split_rows;
        } else if (is_split[(size_t)r]) { printf("FAIL short row %lld split\n", (long long)r); return 1; }
      }
    }
  }
  long long twice = 0;
  for (size_t i = 0; i < writers.size(); ++i) {
    if (is_split[i / F]) {
      if (writers[i] != 0) { printf("FAIL split row written directly\n"); return 1; }
      continue;
    }
    if (writers[i] < 1) { printf("FAIL (row %zu, col %zu) has no writer\n", i / F, i % F); return 1; }
    if (writers[i] > 2) { printf("FAIL (row %zu, col %zu) has %d writers\n", i / F, i % F, writers[i]); return 1; }
    twice += writers[i] == 2;
  }
  printf("OK launches=%zu twice=%lld split_rows=%lld slots=%d\n", launches.size(), twice, split_rows, ws_slots < 0 ? 0 : ws_slots);
  return 0;
}
