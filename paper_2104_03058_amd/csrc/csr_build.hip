// gnnagg_build_csr and gnnagg_plan_rows: the per-graph steps that precede
// aggregation (paper Section II-C: the edge set arrives in COO form; Section
// III: format conversion is a cost of its own).
//
// CSR build = one stable radix sort of the edges on the key
// (destination, source), so that ties fall in input order (the input position
// travels with the key only when the caller asks for the permutation); row
// pointers come from a search of the sorted keys.  Integer work only, no
// atomics on the outputs: the result is unique.
#include "common.hpp"
#include "radix_sort.hpp"

namespace gnnagg {
namespace {

__global__ void fill_u32_kernel(uint32_t* __restrict__ p, uint32_t v) { *p = v; }

__global__ __launch_bounds__(kBlock) void fill_i64_kernel(int64_t* __restrict__ p, int64_t n, int64_t v) {
  const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (k < n) p[k] = v;
}

// rowptr[r] = first slot whose destination is >= r, one thread per row: a binary search over the sorted
// keys, so that the time does not depend on how the empty rows are distributed.
__global__ __launch_bounds__(kBlock) void rowptr_kernel(const uint64_t* __restrict__ keys, int64_t nnz, int64_t N,
                                                        int src_bits, int64_t* __restrict__ rowptr) {
  const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (r > N) return;
  int64_t lo = 0, hi = nnz;  // first slot in [lo, hi] with destination >= r
  while (lo < hi) {
    const int64_t mid = lo + ((hi - lo) >> 1);
    if ((int64_t)(keys[mid] >> src_bits) >= r) hi = mid;
    else lo = mid + 1;
  }
  rowptr[r] = lo;
}

// colidx, perm and the edge weights from the sorted keys in one pass over them: the source is the low
// src_bits of the key, the destination the rest.  GCN symmetric normalisation: fp64 1/sqrt(d_i d_j), one
// rounding to fp32 (rowptr is complete when this runs).
__global__ __launch_bounds__(kBlock) void csr_from_sorted_kernel(const uint64_t* __restrict__ keys,
                                                                 const uint32_t* __restrict__ vals,
                                                                 int64_t nnz, int src_bits,
                                                                 const int64_t* __restrict__ rowptr, int norm_sym,
                                                                 int32_t* __restrict__ colidx,
                                                                 int64_t* __restrict__ perm,
                                                                 float* __restrict__ edge_w) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= nnz) return;
  const uint64_t key = keys[e];
  const int64_t j = (int64_t)(key & ((1ull << src_bits) - 1ull));
  colidx[e] = (int32_t)j;
  if (perm) perm[e] = (int64_t)vals[e];
  if (edge_w) {
    if (norm_sym) {
      const int64_t i = (int64_t)(key >> src_bits);
      const double di = (double)(rowptr[i + 1] - rowptr[i]);
      const double dj = (double)(rowptr[j + 1] - rowptr[j]);
      edge_w[e] = (float)(1.0 / sqrt(di * dj));
    } else {
      edge_w[e] = 1.0f;
    }
  }
}

// ---- row plan -------------------------------------------------------------
__device__ inline int degree_class(int64_t deg) {  // 0 for empty, else 1 + floor(log2 deg), capped at 32
  if (deg <= 0) return 0;
  const int c = 64 - __clzll((unsigned long long)deg);
  return c > 32 ? 32 : c;
}

// Row r owns the edges [begin[r], end[r]): end = begin + 1 for a whole CSR, two rows of a block table for
// one source block.
__global__ __launch_bounds__(kBlock) void make_degree_keys_kernel(const int64_t* __restrict__ begin,
                                                                  const int64_t* __restrict__ end, int64_t N,
                                                                  uint64_t* __restrict__ keys,
                                                                  uint32_t* __restrict__ vals) {
  const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (r >= N) return;
  int64_t deg = end[r] - begin[r];
  if (deg < 0) deg = 0;
  if (deg > 0xffffffffll) deg = 0xffffffffll;
  keys[r] = 0xffffffffull - (uint64_t)deg;  // ascending key = descending degree
  vals[r] = (uint32_t)r;
}

// Writes row_order and, at every change of degree class along the sorted
// order, the class offsets: class c starts at class_off[32 - c].
__global__ __launch_bounds__(kBlock) void plan_finish_kernel(const uint64_t* __restrict__ keys,
                                                             const uint32_t* __restrict__ vals, int64_t N,
                                                             int32_t* __restrict__ row_order,
                                                             int64_t* __restrict__ class_off) {
  const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (k > N) return;
  // class of the row at sorted position k; position N acts as class -1, position -1 as class 33
  const int c = (k < N) ? degree_class((int64_t)(0xffffffffull - keys[k])) : -1;
  const int cprev = (k == 0) ? GNNAGG_PLAN_CLASSES : degree_class((int64_t)(0xffffffffull - keys[k - 1]));
  for (int cc = cprev - 1; cc > c; --cc) class_off[32 - cc] = k;  // classes with no rows
  if (c >= 0 && c != cprev) class_off[32 - c] = k;
  if (k < N) row_order[k] = (int32_t)vals[k];
  else class_off[GNNAGG_PLAN_CLASSES] = N;
}

// ---- popularity order of the sources -------------------------------------------
__global__ __launch_bounds__(kBlock) void fill_range_u32_kernel(uint32_t* __restrict__ p, int64_t n, uint32_t v) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ __launch_bounds__(kBlock) void count_sources_kernel(const int32_t* __restrict__ colidx, int64_t nnz,
                                                               int64_t N, uint32_t* __restrict__ count) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= nnz) return;
  const int64_t j = colidx[e];
  if (j >= 0 && j < N) atomicAdd(&count[j], 1u);  // integer counts: the result does not depend on the order
}

__global__ __launch_bounds__(kBlock) void make_count_keys_kernel(const uint32_t* __restrict__ count, int64_t N,
                                                                 uint64_t* __restrict__ keys,
                                                                 uint32_t* __restrict__ vals) {
  const int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (j >= N) return;
  keys[j] = 0xffffffffull - (uint64_t)count[j];  // ascending key = descending count; the sort is stable in j
  vals[j] = (uint32_t)j;
}

__global__ __launch_bounds__(kBlock) void rank_from_order_kernel(const uint32_t* __restrict__ order, int64_t N,
                                                                 int32_t* __restrict__ rank) {
  const int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (p < N) rank[order[p]] = (int32_t)p;
}

__global__ __launch_bounds__(kBlock) void rename_sources_kernel(const int32_t* __restrict__ colidx, int64_t nnz,
                                                                int64_t N, const int32_t* __restrict__ rank,
                                                                int32_t* __restrict__ out) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= nnz) return;
  const int64_t j = colidx[e];
  out[e] = (j >= 0 && j < N) ? rank[j] : (int32_t)j;
}

// ---- validity check of a caller's CSR ----------------------------------------------
__global__ __launch_bounds__(kBlock) void check_rowptr_kernel(const int64_t* __restrict__ rowptr, int64_t N,
                                                              int64_t nnz, uint32_t* __restrict__ bad) {
  const int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (r > N) return;
  bool wrong = false;
  if (r == 0) wrong = rowptr[0] != 0 || rowptr[N] != nnz;
  if (r < N) wrong = wrong || rowptr[r] > rowptr[r + 1] || rowptr[r] < 0 || rowptr[r + 1] > nnz;
  if (wrong) atomicOr(bad, 1u);
}

__global__ __launch_bounds__(kBlock) void check_colidx_kernel(const int32_t* __restrict__ colidx, int64_t nnz,
                                                              int64_t N, uint32_t* __restrict__ bad) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= nnz) return;
  const int64_t j = colidx[e];
  if (j < 0 || j >= N) atomicOr(bad, 2u);
}

struct CsrWorkspace {
  uint64_t *keys_a, *keys_b;
  uint32_t *vals_a, *vals_b, *hist, *scan, *bad;
  size_t bytes;
};

CsrWorkspace carve_sort_workspace(void* base, int64_t n) {
  Carver c(base);
  CsrWorkspace w;
  const size_t cnt = (size_t)(n > 0 ? n : 1);
  w.keys_a = c.take<uint64_t>(cnt);
  w.keys_b = c.take<uint64_t>(cnt);
  w.vals_a = c.take<uint32_t>(cnt);
  w.vals_b = c.take<uint32_t>(cnt);
  const size_t hw = sort_hist_words(n > 0 ? n : 1);
  w.hist = c.take<uint32_t>(hw);
  w.scan = c.take<uint32_t>(scan_scratch_words((int64_t)hw));
  w.bad = c.take<uint32_t>(64);
  w.bytes = c.used;
  return w;
}

unsigned grid_for(int64_t n) { return (unsigned)ceil_div(n > 0 ? n : 1, kBlock); }

// ---- source blocks -----------------------------------------------------------
// Flags a row whose sources are not in ascending order: one wave per row, the lanes stride over the
// neighbouring pairs of its edge list.
__global__ __launch_bounds__(kBlock) void rows_ascending_kernel(const int64_t* __restrict__ rowptr,
                                                                const int32_t* __restrict__ colidx, int64_t N,
                                                                uint32_t* __restrict__ bad) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wave = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave;
  const int64_t waves = (int64_t)gridDim.x * kWavesPerBlock;
  bool wrong = false;
  for (int64_t r = wave; r < N; r += waves) {
    const int64_t e0 = rowptr[r], e1 = rowptr[r + 1];
    for (int64_t e = e0 + lane; e + 1 < e1; e += kWave) wrong |= colidx[e] > colidx[e + 1];
  }
  if (wrong) atomicOr(bad, 1u);
}

// block_ptr[b * N + r] = first edge of row r whose source lies in block b or a later one (blocks of
// `per_block` consecutive vertex ids); b = 0 .. B, so that block b of row r is
// [block_ptr[b * N + r], block_ptr[(b + 1) * N + r]).  One thread per entry, a binary search in the row.
__global__ __launch_bounds__(kBlock) void block_bounds_kernel(const int64_t* __restrict__ rowptr,
                                                              const int32_t* __restrict__ colidx, int64_t N,
                                                              int32_t B, int64_t per_block,
                                                              int64_t* __restrict__ block_ptr) {
  const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (t >= N * (int64_t)(B + 1)) return;
  const int64_t b = t / N, r = t - b * N;
  int64_t lo = rowptr[r], hi = rowptr[r + 1];
  if (b == 0) hi = lo;
  else if (b == B) lo = hi;
  const int64_t first_source = b * per_block;
  while (lo < hi) {
    const int64_t mid = lo + ((hi - lo) >> 1);
    if ((int64_t)colidx[mid] >= first_source) hi = mid;
    else lo = mid + 1;
  }
  block_ptr[t] = lo;
}

}  // namespace
}  // namespace gnnagg

using namespace gnnagg;

extern "C" int gnnagg_build_csr(int64_t N, int64_t E, const int32_t* src, const int32_t* dst, uint32_t flags,
                                int64_t* rowptr, int32_t* colidx, float* edge_w, int64_t* perm, void* workspace,
                                size_t* workspace_bytes, void* stream_) {
  if (N < 0 || E < 0) return GNNAGG_EINVAL;
  if (flags & ~(uint32_t)(GNNAGG_SELF_LOOPS | GNNAGG_NORM_SYM)) return GNNAGG_EINVAL;
  if (!workspace_bytes) return GNNAGG_ENULL;
  if (N >= (1ll << 31)) return GNNAGG_EUNSUPPORTED;
  if (N == 0 && E > 0) return GNNAGG_EINVAL;  // no vertex an edge could touch
  const int64_t nnz = E + ((flags & GNNAGG_SELF_LOOPS) ? N : 0);
  if (nnz >= (1ll << 32)) return GNNAGG_EUNSUPPORTED;
  CsrWorkspace w = carve_sort_workspace(workspace, nnz);
  if (!workspace) {
    *workspace_bytes = w.bytes;
    return GNNAGG_OK;
  }
  if (!rowptr || (E > 0 && (!src || !dst)) || (nnz > 0 && !colidx)) return GNNAGG_ENULL;
  if (*workspace_bytes < w.bytes || ((uintptr_t)workspace & 255u)) return GNNAGG_EWORKSPACE;
  hipStream_t stream = (hipStream_t)stream_;

  if (nnz == 0) {
    hipLaunchKernelGGL(fill_i64_kernel, dim3(grid_for(N + 1)), dim3(kBlock), 0, stream, rowptr, N + 1, (int64_t)0);
    GNNAGG_HIP_TRY(hipGetLastError());
    GNNAGG_HIP_TRY(hipStreamSynchronize(stream));
    return GNNAGG_OK;
  }
  const int src_bits = bits_for((uint64_t)(N - 1));
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(1), 0, stream, w.bad, 0u);
  GNNAGG_HIP_TRY(hipGetLastError());
  // one stable sort on (destination, source); the keys of the first pass come straight from the COO arrays,
  // and the input positions travel with the keys only if the caller wants the permutation
  KeySource coo;
  coo.src = src;
  coo.dst = dst;
  coo.E = E;
  coo.N = N;
  coo.src_bits = src_bits;
  coo.bad = w.bad;
  bool in_a = true;
  int rc = radix_sort(coo, w.keys_a, w.vals_a, w.keys_b, w.vals_b, nnz, 0, 2 * src_bits, perm != nullptr, w.hist,
                      w.scan, stream, &in_a);
  if (rc != GNNAGG_OK) return rc;
  const uint64_t* keys = in_a ? w.keys_a : w.keys_b;
  const uint32_t* vals = in_a ? w.vals_a : w.vals_b;
  hipLaunchKernelGGL(rowptr_kernel, dim3(grid_for(N + 1)), dim3(kBlock), 0, stream, keys, nnz, N, src_bits, rowptr);
  hipLaunchKernelGGL(csr_from_sorted_kernel, dim3(grid_for(nnz)), dim3(kBlock), 0, stream, keys, vals, nnz, src_bits,
                     (const int64_t*)rowptr, (int)((flags & GNNAGG_NORM_SYM) != 0), colidx, perm, edge_w);
  GNNAGG_HIP_TRY(hipGetLastError());
  uint32_t bad = 0;
  GNNAGG_HIP_TRY(hipMemcpyAsync(&bad, w.bad, sizeof(bad), hipMemcpyDeviceToHost, stream));
  GNNAGG_HIP_TRY(hipStreamSynchronize(stream));
  return bad ? GNNAGG_EINVAL : GNNAGG_OK;
}

// Row plan of the rows [begin[r], end[r]): degree-descending order and the class offsets (host).  Waits
// for the stream.
static int plan_rows_impl(int64_t N, const int64_t* begin, const int64_t* end, int32_t* row_order, int64_t* d_off,
                          int64_t* class_off, const CsrWorkspace& w, hipStream_t stream) {
  hipLaunchKernelGGL(make_degree_keys_kernel, dim3(grid_for(N)), dim3(kBlock), 0, stream, begin, end, N, w.keys_a,
                     w.vals_a);
  GNNAGG_HIP_TRY(hipGetLastError());
  bool in_a = true;
  KeySource from_a;
  from_a.keys = w.keys_a;
  int rc = radix_sort(from_a, w.keys_a, w.vals_a, w.keys_b, w.vals_b, N, 0, 32, true, w.hist, w.scan, stream, &in_a);
  if (rc != GNNAGG_OK) return rc;
  hipLaunchKernelGGL(plan_finish_kernel, dim3(grid_for(N + 1)), dim3(kBlock), 0, stream,
                     (const uint64_t*)(in_a ? w.keys_a : w.keys_b), (const uint32_t*)(in_a ? w.vals_a : w.vals_b), N,
                     row_order, d_off);
  GNNAGG_HIP_TRY(hipGetLastError());
  GNNAGG_HIP_TRY(hipMemcpyAsync(class_off, d_off, sizeof(int64_t) * (GNNAGG_PLAN_CLASSES + 1),
                                hipMemcpyDeviceToHost, stream));
  GNNAGG_HIP_TRY(hipStreamSynchronize(stream));
  return GNNAGG_OK;
}

extern "C" int gnnagg_plan_rows(int64_t N, const int64_t* rowptr, int32_t* row_order, int64_t* class_off,
                                void* workspace, size_t* workspace_bytes, void* stream_) {
  if (N < 0) return GNNAGG_EINVAL;
  if (!workspace_bytes) return GNNAGG_ENULL;
  if (N >= (1ll << 31)) return GNNAGG_EUNSUPPORTED;
  CsrWorkspace w = carve_sort_workspace(workspace, N);
  Carver extra(workspace ? (char*)workspace + w.bytes : nullptr);
  int64_t* d_off = extra.take<int64_t>(GNNAGG_PLAN_CLASSES + 1);
  const size_t need = w.bytes + extra.used;
  if (!workspace) {
    *workspace_bytes = need;
    return GNNAGG_OK;
  }
  if (!rowptr || !class_off || (N > 0 && !row_order)) return GNNAGG_ENULL;
  if (*workspace_bytes < need || ((uintptr_t)workspace & 255u)) return GNNAGG_EWORKSPACE;
  hipStream_t stream = (hipStream_t)stream_;
  if (N == 0) {
    for (int k = 0; k <= GNNAGG_PLAN_CLASSES; ++k) class_off[k] = 0;
    return GNNAGG_OK;
  }
  return plan_rows_impl(N, rowptr, rowptr + 1, row_order, d_off, class_off, w, stream);
}

extern "C" int gnnagg_plan_source_blocks(int64_t N, const int64_t* rowptr, const int32_t* colidx, int32_t B,
                                         int64_t* block_ptr, int32_t* row_order, int64_t* class_off,
                                         void* workspace, size_t* workspace_bytes, void* stream_) {
  if (N < 0 || B < 1 || B > GNNAGG_MAX_SOURCE_BLOCKS) return GNNAGG_EINVAL;
  if (!workspace_bytes) return GNNAGG_ENULL;
  if (N >= (1ll << 31)) return GNNAGG_EUNSUPPORTED;
  CsrWorkspace w = carve_sort_workspace(workspace, N);
  Carver extra(workspace ? (char*)workspace + w.bytes : nullptr);
  int64_t* d_off = extra.take<int64_t>(GNNAGG_PLAN_CLASSES + 1);
  uint32_t* bad = extra.take<uint32_t>(64);
  const size_t need = w.bytes + extra.used;
  if (!workspace) {
    *workspace_bytes = need;
    return GNNAGG_OK;
  }
  if (!rowptr || !class_off || (N > 0 && (!row_order || !block_ptr || !colidx))) return GNNAGG_ENULL;
  if (*workspace_bytes < need || ((uintptr_t)workspace & 255u)) return GNNAGG_EWORKSPACE;
  if (((uintptr_t)rowptr % 8) || ((uintptr_t)colidx % 4) || ((uintptr_t)block_ptr % 8) || ((uintptr_t)row_order % 4))
    return GNNAGG_EINVAL;
  hipStream_t stream = (hipStream_t)stream_;
  if (N == 0) {
    for (int k = 0; k < B * (GNNAGG_PLAN_CLASSES + 1); ++k) class_off[k] = 0;
    return GNNAGG_OK;
  }
  // the edges of a block are one run of a row only if the row lists its sources in ascending order
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(1), 0, stream, bad, 0u);
  GNNAGG_HIP_TRY(hipGetLastError());
  const int64_t waves = N < (1 << 16) ? N : (1 << 16);
  hipLaunchKernelGGL(rows_ascending_kernel, dim3((unsigned)ceil_div(waves, kWavesPerBlock)), dim3(kBlock), 0, stream,
                     rowptr, colidx, N, bad);
  GNNAGG_HIP_TRY(hipGetLastError());
  uint32_t h_bad = 0;
  GNNAGG_HIP_TRY(hipMemcpyAsync(&h_bad, bad, sizeof(h_bad), hipMemcpyDeviceToHost, stream));
  GNNAGG_HIP_TRY(hipStreamSynchronize(stream));
  if (h_bad) return GNNAGG_EINVAL;
  const int64_t per_block = ceil_div(N, (int64_t)B);  // vertices per source block
  hipLaunchKernelGGL(block_bounds_kernel, dim3(grid_for(N * (int64_t)(B + 1))), dim3(kBlock), 0, stream, rowptr,
                     colidx, N, B, per_block, block_ptr);
  GNNAGG_HIP_TRY(hipGetLastError());
  for (int32_t b = 0; b < B; ++b) {
    int rc = plan_rows_impl(N, block_ptr + (int64_t)b * N, block_ptr + (int64_t)(b + 1) * N,
                            row_order + (int64_t)b * N, d_off, class_off + (int64_t)b * (GNNAGG_PLAN_CLASSES + 1), w,
                            stream);
    if (rc != GNNAGG_OK) return rc;
  }
  return GNNAGG_OK;
}

extern "C" int gnnagg_rank_sources(int64_t N, int64_t nnz, const int32_t* colidx, int32_t* rank,
                                   int32_t* colidx_ranked, void* workspace, size_t* workspace_bytes, void* stream_) {
  if (N < 0 || nnz < 0) return GNNAGG_EINVAL;
  if (!workspace_bytes) return GNNAGG_ENULL;
  if (N >= (1ll << 31) || nnz >= (1ll << 32)) return GNNAGG_EUNSUPPORTED;
  CsrWorkspace w = carve_sort_workspace(workspace, N);
  Carver extra(workspace ? (char*)workspace + w.bytes : nullptr);
  uint32_t* count = extra.take<uint32_t>((size_t)(N > 0 ? N : 1));
  const size_t need = w.bytes + extra.used;
  if (!workspace) {
    *workspace_bytes = need;
    return GNNAGG_OK;
  }
  if (*workspace_bytes < need || ((uintptr_t)workspace & 255u)) return GNNAGG_EWORKSPACE;
  if (N == 0) return nnz == 0 ? GNNAGG_OK : GNNAGG_EINVAL;
  if (!rank || (nnz > 0 && (!colidx || !colidx_ranked))) return GNNAGG_ENULL;
  if (((uintptr_t)rank % 4) || ((uintptr_t)colidx % 4) || ((uintptr_t)colidx_ranked % 4)) return GNNAGG_EINVAL;
  hipStream_t stream = (hipStream_t)stream_;
  hipLaunchKernelGGL(fill_range_u32_kernel, dim3(grid_for(N)), dim3(kBlock), 0, stream, count, N, 0u);
  GNNAGG_HIP_TRY(hipGetLastError());
  if (nnz > 0) {
    hipLaunchKernelGGL(count_sources_kernel, dim3(grid_for(nnz)), dim3(kBlock), 0, stream, colidx, nnz, N, count);
    GNNAGG_HIP_TRY(hipGetLastError());
  }
  hipLaunchKernelGGL(make_count_keys_kernel, dim3(grid_for(N)), dim3(kBlock), 0, stream, (const uint32_t*)count, N,
                     w.keys_a, w.vals_a);
  GNNAGG_HIP_TRY(hipGetLastError());
  bool in_a = true;
  KeySource from_a;
  from_a.keys = w.keys_a;
  int rc = radix_sort(from_a, w.keys_a, w.vals_a, w.keys_b, w.vals_b, N, 0, 32, true, w.hist, w.scan, stream, &in_a);
  if (rc != GNNAGG_OK) return rc;
  hipLaunchKernelGGL(rank_from_order_kernel, dim3(grid_for(N)), dim3(kBlock), 0, stream,
                     (const uint32_t*)(in_a ? w.vals_a : w.vals_b), N, rank);
  GNNAGG_HIP_TRY(hipGetLastError());
  if (nnz > 0) {
    hipLaunchKernelGGL(rename_sources_kernel, dim3(grid_for(nnz)), dim3(kBlock), 0, stream, colidx, nnz, N,
                       (const int32_t*)rank, colidx_ranked);
    GNNAGG_HIP_TRY(hipGetLastError());
  }
  return GNNAGG_OK;
}

extern "C" int gnnagg_check_csr(int64_t N, int64_t nnz, const int64_t* rowptr, const int32_t* colidx, void* workspace,
                                size_t* workspace_bytes, void* stream_) {
  if (N < 0 || nnz < 0) return GNNAGG_EINVAL;
  if (!workspace_bytes) return GNNAGG_ENULL;
  if (N >= (1ll << 31)) return GNNAGG_EUNSUPPORTED;
  Carver carve(workspace);
  uint32_t* bad = carve.take<uint32_t>(64);
  if (!workspace) {
    *workspace_bytes = carve.used;
    return GNNAGG_OK;
  }
  if (*workspace_bytes < carve.used || ((uintptr_t)workspace & 255u)) return GNNAGG_EWORKSPACE;
  if (!rowptr || (nnz > 0 && !colidx)) return GNNAGG_ENULL;
  if (((uintptr_t)rowptr % 8) || ((uintptr_t)colidx % 4)) return GNNAGG_EINVAL;
  hipStream_t stream = (hipStream_t)stream_;
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(1), 0, stream, bad, 0u);
  hipLaunchKernelGGL(check_rowptr_kernel, dim3(grid_for(N + 1)), dim3(kBlock), 0, stream, rowptr, N, nnz, bad);
  if (nnz > 0)
    hipLaunchKernelGGL(check_colidx_kernel, dim3(grid_for(nnz)), dim3(kBlock), 0, stream, colidx, nnz, N, bad);
  GNNAGG_HIP_TRY(hipGetLastError());
  uint32_t flag = 0;
  GNNAGG_HIP_TRY(hipMemcpyAsync(&flag, bad, sizeof(flag), hipMemcpyDeviceToHost, stream));
  GNNAGG_HIP_TRY(hipStreamSynchronize(stream));
  return flag ? GNNAGG_EINVAL : GNNAGG_OK;
}
