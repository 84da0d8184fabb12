// The neighbour walk shared by the aggregation and attention kernels: how a row's edge list is dealt
// out to lanes, how edge indices and weights reach them, and the gather batch.
//
// An accumulator policy `Acc` says what is fetched per edge and how it enters the reduction:
//   static constexpr bool kWeighted      - the walk also delivers edge_w
//   void fetch(int u, int32_t j)          - issue the loads for source row j into slot u of the batch
//   void fetch_uniform(int u, int64_t j)  - the same when j is the same in every lane (it lives in scalar
//                                           registers: the row address is scalar arithmetic plus one add)
//   template <bool MASKED> void use(int u, float w, bool ok)
//                                         - fold slot u in; ok == false (MASKED batches only) means
//                                           the entry does not exist and must not change the result
#pragma once
#include "common.hpp"
#include "device_utils.hpp"

namespace gnnagg {

constexpr int kUnroll = 8;  // gathers in flight per lane = one batch

typedef int32_t i32x4_u __attribute__((ext_vector_type(4), aligned(4)));

__device__ inline int64_t uniform64(int64_t v) {  // v is the same in every lane: move it to scalar registers
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

// One gather + accumulate batch: kUnroll independent row loads issued back to back, then the
// accumulates.  Straight-line code: an entry that does not exist (only in MASKED batches) re-reads the
// row `jsafe`, which does exist, and is folded in with ok == false, so no load sits behind a branch.
// ok(u), j(u), w(u) describe entry u.
template <bool MASKED, bool UNIFORM_J = false, typename Acc, typename OkF, typename JF, typename WF>
__device__ inline void gather_batch(Acc& acc, OkF ok, JF j, WF w, int64_t jsafe) {
  float wv[kUnroll];
  bool okv[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    okv[u] = MASKED ? (bool)ok(u) : true;
    wv[u] = Acc::kWeighted ? (float)w(u) : 1.0f;
    if constexpr (UNIFORM_J) {
      acc.fetch_uniform(u, okv[u] ? (int64_t)j(u) : jsafe);
    } else {  // vertex ids are 32-bit: the select and the address arithmetic stay 32-bit
      acc.fetch(u, okv[u] ? (int32_t)j(u) : (int32_t)jsafe);
    }
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) acc.template use<MASKED>(u, wv[u], okv[u]);
}

// How a row's edge list is dealt out to its P = 2^p_log2 neighbour slots: in rounds of 8*P consecutive
// edges, slot ng taking edges [8*ng, 8*ng + 8) of every round - one gather batch.  All slots of a row
// therefore work on the same 8*P-edge stretch of the (source-sorted) list at any time.
//
// Slot = a whole wavefront (64 lanes span the slice).  The wave reads the edge indices (and weights) of
// its next eight batches with one load each, then walks them: the source row of an entry is broadcast
// with v_readlane, so row addresses live in scalar registers.  [e0, e1), ng are the same in every lane.
template <typename Acc>
__device__ inline void gather_wave(Acc& acc, const int32_t* __restrict__ colidx, const float* __restrict__ edge_w,
                                   int64_t e0, int64_t e1, int ng, int p_log2, int lane) {
  const int64_t e0_u = uniform64(e0), e1_u = uniform64(e1);
  const int ng_u = __builtin_amdgcn_readfirstlane(ng);
  const int shift = 3 + p_log2;                    // log2 of the round length
  const int64_t outer = (int64_t)kWave << p_log2;  // edges the row advances per index load
  const int64_t lane_pos = ((int64_t)(lane >> 3) << shift) + (ng_u << 3) + (lane & 7);
  int32_t idx_c = 0;
  float w_c = 1.0f;
  if (e0_u + lane_pos < e1_u) {
    idx_c = colidx[e0_u + lane_pos];
    if (Acc::kWeighted) w_c = edge_w[e0_u + lane_pos];
  }
  for (int64_t e = e0_u; e < e1_u; e += outer) {
    int32_t idx_n = 0;  // the next eight batches' indices are requested before this block's rows
    float w_n = 1.0f;
    if (e + outer + lane_pos < e1_u) {
      idx_n = colidx[e + outer + lane_pos];
      if (Acc::kWeighted) w_n = edge_w[e + outer + lane_pos];
    }
    for (int k = 0; k < kWave / kUnroll; ++k) {
      const int64_t left = e1_u - (e + ((int64_t)k << shift) + (ng_u << 3));
      if (left <= 0) break;
      const int l0 = k * kUnroll;
      auto jf = [&](int u) { return __builtin_amdgcn_readlane(idx_c, l0 + u); };
      auto wf = [&](int u) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_c), l0 + u)); };
      if (left >= kUnroll) {
        gather_batch<false, true>(acc, [](int) { return true; }, jf, wf, 0);
      } else {
        gather_batch<true, true>(acc, [&](int u) { return u < left; }, jf, wf,
                                 (int64_t)__builtin_amdgcn_readlane(idx_c, l0));
      }
    }
    idx_c = idx_n;
    w_c = w_n;
  }
}

// Value of lane `slot_base + SRC` for every lane of a slot of G lanes (8, 16 or 32; slots are aligned to G, so
// they lie inside one half of the wave): a swizzle with an immediate pattern - lane' = (lane & ~(G-1)) | SRC
// on the low five lane bits - which needs no address register and no vector instruction to form one.
template <int G, int SRC>
__device__ inline int32_t slot_broadcast(int32_t v) {
  static_assert(G == 8 || G == 16 || G == 32, "slots of 8, 16 or 32 lanes");
  static_assert(SRC >= 0 && SRC < G, "source lane inside the slot");
  constexpr int kAnd = 0x1f & ~(G - 1), kOr = SRC;
  return __builtin_amdgcn_ds_swizzle(v, (kOr << 5) | kAnd);
}

template <int G, int K, typename Acc>
__device__ inline void wide_batch(Acc& acc, int32_t idx_c, float w_c) {
  int32_t j[kUnroll];
  float wj[kUnroll];
  j[0] = slot_broadcast<G, K * kUnroll + 0>(idx_c);
  j[1] = slot_broadcast<G, K * kUnroll + 1>(idx_c);
  j[2] = slot_broadcast<G, K * kUnroll + 2>(idx_c);
  j[3] = slot_broadcast<G, K * kUnroll + 3>(idx_c);
  j[4] = slot_broadcast<G, K * kUnroll + 4>(idx_c);
  j[5] = slot_broadcast<G, K * kUnroll + 5>(idx_c);
  j[6] = slot_broadcast<G, K * kUnroll + 6>(idx_c);
  j[7] = slot_broadcast<G, K * kUnroll + 7>(idx_c);
  if constexpr (Acc::kWeighted) {
    const int32_t wb = __float_as_int(w_c);
    wj[0] = __int_as_float(slot_broadcast<G, K * kUnroll + 0>(wb));
    wj[1] = __int_as_float(slot_broadcast<G, K * kUnroll + 1>(wb));
    wj[2] = __int_as_float(slot_broadcast<G, K * kUnroll + 2>(wb));
    wj[3] = __int_as_float(slot_broadcast<G, K * kUnroll + 3>(wb));
    wj[4] = __int_as_float(slot_broadcast<G, K * kUnroll + 4>(wb));
    wj[5] = __int_as_float(slot_broadcast<G, K * kUnroll + 5>(wb));
    wj[6] = __int_as_float(slot_broadcast<G, K * kUnroll + 6>(wb));
    wj[7] = __int_as_float(slot_broadcast<G, K * kUnroll + 7>(wb));
  } else {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) wj[u] = 1.0f;
  }
  gather_batch<true>(acc, [&](int u) { return j[u] >= 0; }, [&](int u) { return j[u]; },
                     [&](int u) { return wj[u]; }, (int64_t)j[0]);
}

// Slot = G lanes, G = 8, 16 or 32.  The lanes of a slot read the indices of the slot's next G / 8 batches with
// one load and hand them round with swizzles.  All lanes of a slot run the loop together; lanes without
// columns of their own hold indices for the others and re-read the slice's last columns (their column offset
// is always valid) rather than branching around the gathers.
template <int G, typename Acc>
__device__ inline void gather_wide(Acc& acc, const int32_t* __restrict__ colidx, const float* __restrict__ edge_w,
                                   int64_t e0, int64_t e1, int ng, int p_log2, int lane) {
  static_assert(kUnroll == 8, "a batch is eight entries");
  const int gl = lane & (G - 1);
  const int shift = 3 + p_log2;
  const int64_t outer = (int64_t)G << p_log2;
  const int64_t lane_pos = ((int64_t)(gl >> 3) << shift) + (ng << 3) + (gl & 7);
  int32_t idx_c = -1;
  float w_c = 0.0f;
  if (e0 + lane_pos < e1) {
    idx_c = colidx[e0 + lane_pos];
    if (Acc::kWeighted) w_c = edge_w[e0 + lane_pos];
  }
  for (int64_t e = e0; e < e1; e += outer) {
    int32_t idx_n = -1;
    float w_n = 0.0f;
    if (e + outer + lane_pos < e1) {
      idx_n = colidx[e + outer + lane_pos];
      if (Acc::kWeighted) w_n = edge_w[e + outer + lane_pos];
    }
    // batch k of the block exists for this slot if its first edge does (same for every lane of the slot)
    const int64_t first = e + (ng << 3);
    if (first < e1) wide_batch<G, 0>(acc, idx_c, w_c);  // (its first entry then exists: the row every masked entry re-reads)
    if constexpr (G >= 16) {
      if (first + ((int64_t)1 << shift) < e1) wide_batch<G, 1>(acc, idx_c, w_c);
    }
    if constexpr (G >= 32) {
      if (first + ((int64_t)2 << shift) < e1) wide_batch<G, 2>(acc, idx_c, w_c);
      if (first + ((int64_t)3 << shift) < e1) wide_batch<G, 3>(acc, idx_c, w_c);
    }
    idx_c = idx_n;
    w_c = w_n;
  }
}

// The same walk with the indices handed round through LDS instead of swizzles: every lane parks the index
// (and weight) it loaded in its wave's tile, and a batch reads its eight entries back as two 16-byte LDS
// reads per lane.  The lanes of a slot only ever read what lanes of the same slot wrote, and a wave's LDS
// operations execute in order, so a wavefront-scope fence (a scheduling barrier for the compiler) is all
// the synchronisation needed.  tile: 2 * kWave words owned by this wave, 16-byte aligned.
__device__ inline void stage_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int K, typename Acc>
__device__ inline void staged_batch(Acc& acc, const int32_t* slot_tile) {
  typedef int32_t i32x4_a __attribute__((ext_vector_type(4)));
  const i32x4_a a = *reinterpret_cast<const i32x4_a*>(slot_tile + K * kUnroll);
  const i32x4_a b = *reinterpret_cast<const i32x4_a*>(slot_tile + K * kUnroll + 4);
  const int32_t j[kUnroll] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
  float wj[kUnroll];
  if constexpr (Acc::kWeighted) {
    const i32x4_a c = *reinterpret_cast<const i32x4_a*>(slot_tile + kWave + K * kUnroll);
    const i32x4_a d = *reinterpret_cast<const i32x4_a*>(slot_tile + kWave + K * kUnroll + 4);
    wj[0] = __int_as_float(c.x); wj[1] = __int_as_float(c.y); wj[2] = __int_as_float(c.z); wj[3] = __int_as_float(c.w);
    wj[4] = __int_as_float(d.x); wj[5] = __int_as_float(d.y); wj[6] = __int_as_float(d.z); wj[7] = __int_as_float(d.w);
  } else {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) wj[u] = 1.0f;
  }
  gather_batch<true>(acc, [&](int u) { return j[u] >= 0; }, [&](int u) { return j[u]; },
                     [&](int u) { return wj[u]; }, (int64_t)j[0]);
}

template <int G, typename Acc>
__device__ inline void gather_wide_staged(Acc& acc, const int32_t* __restrict__ colidx,
                                          const float* __restrict__ edge_w, int64_t e0, int64_t e1, int ng,
                                          int p_log2, int lane, int32_t* tile) {
  static_assert(kUnroll == 8, "a batch is eight entries");
  const int gl = lane & (G - 1);
  const int32_t* slot_tile = tile + (lane & ~(G - 1));
  const int shift = 3 + p_log2;
  const int64_t outer = (int64_t)G << p_log2;
  const int64_t lane_pos = ((int64_t)(gl >> 3) << shift) + (ng << 3) + (gl & 7);
  int32_t idx_c = -1;
  float w_c = 0.0f;
  if (e0 + lane_pos < e1) {
    idx_c = colidx[e0 + lane_pos];
    if (Acc::kWeighted) w_c = edge_w[e0 + lane_pos];
  }
  for (int64_t e = e0; e < e1; e += outer) {
    int32_t idx_n = -1;
    float w_n = 0.0f;
    if (e + outer + lane_pos < e1) {
      idx_n = colidx[e + outer + lane_pos];
      if (Acc::kWeighted) w_n = edge_w[e + outer + lane_pos];
    }
    tile[lane] = idx_c;
    if (Acc::kWeighted) tile[kWave + lane] = __float_as_int(w_c);
    stage_sync();
    const int64_t first = e + (ng << 3);
    if (first < e1) staged_batch<0>(acc, slot_tile);
    if constexpr (G >= 16) {
      if (first + ((int64_t)1 << shift) < e1) staged_batch<1>(acc, slot_tile);
    }
    if constexpr (G >= 32) {
      if (first + ((int64_t)2 << shift) < e1) staged_batch<2>(acc, slot_tile);
      if (first + ((int64_t)3 << shift) < e1) staged_batch<3>(acc, slot_tile);
    }
    stage_sync();  // the tile is rewritten only after every lane of the slot has read it
    idx_c = idx_n;
    w_c = w_n;
  }
}

// Slot = 1, 2 or 4 lanes (slices of at most 16 fp32 / 32 bf16 columns).  Every lane reads the next
// eight edge indices of its slot itself, as two 16-byte loads (the lanes of a slot read the same
// addresses, which the memory pipeline merges).  The loads may run past the end of the row into the
// following entries of colidx, never past nnz.  es = first edge of the slot, stride = round length.
template <typename Acc>
__device__ inline void gather_narrow(Acc& acc, const int32_t* __restrict__ colidx, const float* __restrict__ edge_w,
                                     int64_t es, int64_t ee, int64_t stride, int64_t nnz) {
  static_assert(kUnroll == 8, "eight indices are read as two 16-byte loads");
  for (int64_t e = es; e < ee; e += stride) {
    int32_t j[kUnroll];
    float wj[kUnroll];
    if (e + kUnroll <= nnz) {
      const i32x4_u i0 = *reinterpret_cast<const i32x4_u*>(colidx + e);
      const i32x4_u i1 = *reinterpret_cast<const i32x4_u*>(colidx + e + 4);
      j[0] = i0.x; j[1] = i0.y; j[2] = i0.z; j[3] = i0.w;
      j[4] = i1.x; j[5] = i1.y; j[6] = i1.z; j[7] = i1.w;
      if (Acc::kWeighted) {
        const f32x4_u w0 = *reinterpret_cast<const f32x4_u*>(edge_w + e);
        const f32x4_u w1 = *reinterpret_cast<const f32x4_u*>(edge_w + e + 4);
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
        j[u] = ok ? colidx[e + u] : -1;
        if (Acc::kWeighted) wj[u] = ok ? edge_w[e + u] : 0.0f;
      }
    }
    if (!Acc::kWeighted) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) wj[u] = 1.0f;
    }
    gather_batch<true>(acc, [&](int u) { return j[u] >= 0; }, [&](int u) { return j[u]; },
                       [&](int u) { return wj[u]; }, (int64_t)j[0]);
  }
}

enum { MODE_WAVE = 0, MODE_WIDE = 1, MODE_NARROW = 2 };  // 64 / 8..32 / 1..4 lanes per slice (fixed per launch)

// Runs the walk of one lane for a row with edges [e0, e1); g, L as in LaneRole (L == 8: hub row).
template <int MODE, typename Acc>
__device__ inline void gather_row(Acc& acc, const int32_t* __restrict__ colidx, const float* __restrict__ edge_w,
                                  int64_t e0, int64_t e1, int ng, int g, int L, bool col_ok, int lane,
                                  int64_t nnz, int32_t* stage = nullptr) {
  const int p_log2 = L - g;  // log2 of the row's neighbour slots
  if constexpr (MODE == MODE_WAVE) {
    gather_wave(acc, colidx, edge_w, e0, e1, ng, p_log2, lane);
  } else if constexpr (MODE == MODE_WIDE) {
    if (stage) {  // indices through LDS (stage: this wave's tile)
      if (g == 3) gather_wide_staged<8>(acc, colidx, edge_w, e0, e1, ng, p_log2, lane, stage);
      else if (g == 4) gather_wide_staged<16>(acc, colidx, edge_w, e0, e1, ng, p_log2, lane, stage);
      else gather_wide_staged<32>(acc, colidx, edge_w, e0, e1, ng, p_log2, lane, stage);
      return;
    }
    if (g == 3) gather_wide<8>(acc, colidx, edge_w, e0, e1, ng, p_log2, lane);
    else if (g == 4) gather_wide<16>(acc, colidx, edge_w, e0, e1, ng, p_log2, lane);
    else gather_wide<32>(acc, colidx, edge_w, e0, e1, ng, p_log2, lane);
  } else {
    if (col_ok) gather_narrow(acc, colidx, edge_w, e0 + (int64_t)ng * kUnroll, e1, (int64_t)kUnroll << p_log2, nnz);
  }
}

}  // namespace gnnagg
