// Stable LSD radix sort (8-bit digits) and exclusive scan for gfx950.
//
// One sort pass = three launches: per-workgroup digit histograms, a scan of the
// digit-major histogram table, and a scatter in which every key finds its
// stable rank inside its workgroup tile with wave ballots (64-lane match on the
// digit) and a small LDS table across the four waves; the tile is sorted by digit
// in LDS and leaves it in whole runs.  No global atomics, so the output order is
// unique.
#include "radix_sort.hpp"

namespace gnnagg {
namespace {

__device__ inline uint32_t wave_inclusive_scan(uint32_t x, int lane) {
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    uint32_t t = __shfl_up(x, o, kWave);
    if (lane >= o) x += t;
  }
  return x;
}

// Exclusive prefix of one value per thread over the 256-thread workgroup.
__device__ inline uint32_t block_exclusive_scan(uint32_t x, uint32_t* lds4, uint32_t* total) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const uint32_t inc = wave_inclusive_scan(x, lane);
  if (lane == kWave - 1) lds4[w] = inc;
  __syncthreads();
  uint32_t wbase = 0, tot = 0;
#pragma unroll
  for (int k = 0; k < kWavesPerBlock; ++k) {
    const uint32_t s = lds4[k];
    if (k < w) wbase += s;
    tot += s;
  }
  __syncthreads();
  *total = tot;
  return wbase + inc - x;
}

__global__ __launch_bounds__(kBlock) void scan_reduce_kernel(const uint32_t* __restrict__ in, int64_t n,
                                                             uint32_t* __restrict__ sums) {
  __shared__ uint32_t lds4[kWavesPerBlock];
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItemsPerThread;
  uint32_t s = 0;
#pragma unroll
  for (int k = 0; k < kScanItemsPerThread; ++k)
    if (base + k < n) s += in[base + k];
  uint32_t total;
  block_exclusive_scan(s, lds4, &total);
  if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(kBlock) void scan_apply_kernel(uint32_t* __restrict__ data, int64_t n,
                                                            const uint32_t* __restrict__ offsets) {
  __shared__ uint32_t lds4[kWavesPerBlock];
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItemsPerThread;
  uint32_t v[kScanItemsPerThread];
  uint32_t s = 0;
#pragma unroll
  for (int k = 0; k < kScanItemsPerThread; ++k) {
    v[k] = (base + k < n) ? data[base + k] : 0u;
    s += v[k];
  }
  uint32_t total;
  uint32_t pre = block_exclusive_scan(s, lds4, &total);
  if (offsets) pre += offsets[blockIdx.x];
#pragma unroll
  for (int k = 0; k < kScanItemsPerThread; ++k) {
    if (base + k < n) data[base + k] = pre;
    pre += v[k];
  }
}

__global__ __launch_bounds__(kBlock) void radix_hist_kernel(const uint64_t* __restrict__ keys, int64_t n,
                                                            int shift, uint32_t* __restrict__ hist,
                                                            int64_t nblk) {
  __shared__ uint32_t h[kRadixBins];
  h[threadIdx.x] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll 4
  for (int r = 0; r < kSortItemsPerThread; ++r) {
    const int64_t i = base + (int64_t)r * kBlock + threadIdx.x;
    if (i < n) atomicAdd(&h[(uint32_t)(keys[i] >> shift) & (kRadixBins - 1)], 1u);
  }
  __syncthreads();
  hist[(int64_t)threadIdx.x * nblk + blockIdx.x] = h[threadIdx.x];
}

// One workgroup scatters one tile of kSortTile keys.  The tile is cut into four contiguous quarters, one
// per wave; a wave keeps its 16 x 64 keys in registers.  Phase 1: every wave counts its quarter per digit
// (wave ballots find the lanes that hold the same digit; one lane per group adds the group size to an LDS
// counter).  Thread d then turns the counts of digit d into the place of each wave's keys with that
// digit inside the tile sorted by digit (an exclusive scan over the digits gives where digit d starts).
// Phase 2: every wave walks its rounds again, alone - position = running start of (wave, digit) + rank
// inside the group - and stores key and value at that place IN LDS.  Phase 3: the sorted tile leaves LDS
// in order, so the keys of one digit go to consecutive global addresses (whole lines, not one 8-byte
// store per lane and digit).  Equal digits keep their input order: the sort is stable, and no global
// atomic is involved.
__global__ __launch_bounds__(kBlock) void radix_scatter_kernel(
    const uint64_t* __restrict__ kin, const uint32_t* __restrict__ vin, uint64_t* __restrict__ kout,
    uint32_t* __restrict__ vout, int64_t n, int shift, const uint32_t* __restrict__ hist_scanned,
    int64_t nblk) {
  __shared__ uint64_t lkey[kSortTile];
  __shared__ uint32_t lval[kSortTile];
  __shared__ uint32_t start[kWavesPerBlock][kRadixBins];  // counts in phase 1, running local positions after
  __shared__ uint32_t shift_out[kRadixBins];              // global position minus local position, per digit
  __shared__ uint32_t lds4[kWavesPerBlock];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
#pragma unroll
  for (int k = 0; k < kWavesPerBlock; ++k) start[k][tid] = 0;
  __syncthreads();
  constexpr int kQuarter = kSortTile / kWavesPerBlock;  // keys per wave
  const int64_t tile = (int64_t)blockIdx.x * kSortTile;
  const int64_t first = tile + (int64_t)w * kQuarter + lane;
  const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
  uint64_t key[kSortItemsPerThread];
  uint32_t val[kSortItemsPerThread];
  uint32_t rank_size[kSortItemsPerThread];  // rank inside the group (low 8 bits), group size - 1 (next 8), valid (bit 16)
#pragma unroll
  for (int r = 0; r < kSortItemsPerThread; ++r) {
    const int64_t i = first + (int64_t)r * kWave;
    const bool valid = i < n;
    key[r] = valid ? kin[i] : 0ull;
    val[r] = valid ? vin[i] : 0u;
    const uint32_t d = (uint32_t)(key[r] >> shift) & (kRadixBins - 1);
    uint64_t same = __ballot(valid);  // lanes of this wave that hold the same digit
#pragma unroll
    for (int b = 0; b < kRadixBits; ++b) {
      const bool bit = (d >> b) & 1u;
      const uint64_t bal = __ballot(valid && bit);
      same &= bit ? bal : ~bal;
    }
    const uint32_t rank = (uint32_t)__popcll(same & below), size = (uint32_t)__popcll(same);
    rank_size[r] = rank | ((size - (valid ? 1u : 0u)) << 8) | (valid ? 1u << 16 : 0u);
    if (valid && rank == 0) start[w][d] += size;  // one lane per digit group; groups of a round differ in d
  }
  __syncthreads();
  {
    uint32_t c[kWavesPerBlock], tot = 0;
#pragma unroll
    for (int k = 0; k < kWavesPerBlock; ++k) {
      c[k] = start[k][tid];
      tot += c[k];
    }
    uint32_t all;
    uint32_t b = block_exclusive_scan(tot, lds4, &all);  // where digit `tid` starts in the sorted tile
    shift_out[tid] = hist_scanned[(int64_t)tid * nblk + blockIdx.x] - b;  // modulo 2^32, undone below
#pragma unroll
    for (int k = 0; k < kWavesPerBlock; ++k) {
      start[k][tid] = b;
      b += c[k];
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < kSortItemsPerThread; ++r) {
    const bool valid = (rank_size[r] >> 16) & 1u;
    const uint32_t d = (uint32_t)(key[r] >> shift) & (kRadixBins - 1);
    const uint32_t rank = rank_size[r] & 0xffu, size = ((rank_size[r] >> 8) & 0xffu) + 1u;
    uint32_t pos = 0;
    if (valid) pos = start[w][d] + rank;
    // every lane of a group has read the start before its first lane moves it on: LDS operations of one
    // wave complete in program order
    if (valid && rank == 0) start[w][d] += size;
    if (valid) {
      lkey[pos] = key[r];
      lval[pos] = val[r];
    }
  }
  __syncthreads();
  const int64_t left = n - tile;
  const int count = left < kSortTile ? (int)left : kSortTile;  // keys in this tile
  for (int p = tid; p < count; p += kBlock) {
    const uint64_t k = lkey[p];
    const uint32_t d = (uint32_t)(k >> shift) & (kRadixBins - 1);
    const uint32_t pos = (uint32_t)p + shift_out[d];
    kout[pos] = k;
    vout[pos] = lval[p];
  }
}

size_t round64(size_t x) { return (x + 63) / 64 * 64; }

}  // namespace

size_t scan_scratch_words(int64_t n) {
  size_t total = 64;
  while (n > kScanTile) {
    n = ceil_div(n, kScanTile);
    total += round64((size_t)n);
  }
  return total;
}

int exclusive_scan_u32(uint32_t* data, int64_t n, uint32_t* scratch, hipStream_t stream) {
  if (n <= 0) return GNNAGG_OK;
  const int64_t nb = ceil_div(n, kScanTile);
  if (nb > 0x7fffffff) return GNNAGG_EUNSUPPORTED;
  if (nb == 1) {
    hipLaunchKernelGGL(scan_apply_kernel, dim3(1), dim3(kBlock), 0, stream, data, n, (const uint32_t*)nullptr);
  } else {
    hipLaunchKernelGGL(scan_reduce_kernel, dim3((unsigned)nb), dim3(kBlock), 0, stream, (const uint32_t*)data, n,
                       scratch);
    int rc = exclusive_scan_u32(scratch, nb, scratch + round64((size_t)nb), stream);
    if (rc != GNNAGG_OK) return rc;
    hipLaunchKernelGGL(scan_apply_kernel, dim3((unsigned)nb), dim3(kBlock), 0, stream, data, n,
                       (const uint32_t*)scratch);
  }
  GNNAGG_HIP_TRY(hipGetLastError());
  return GNNAGG_OK;
}

int radix_sort_pairs(uint64_t* keys_a, uint32_t* vals_a, uint64_t* keys_b, uint32_t* vals_b, int64_t n,
                     int bit_begin, int bit_end, uint32_t* hist, uint32_t* scan_scratch, hipStream_t stream,
                     bool* in_a) {
  *in_a = true;
  if (n <= 0) return GNNAGG_OK;
  const int64_t nblk = sort_blocks(n);
  if (nblk > 0x7fffffff) return GNNAGG_EUNSUPPORTED;
  uint64_t* kin = keys_a;
  uint32_t* vin = vals_a;
  uint64_t* kout = keys_b;
  uint32_t* vout = vals_b;
  for (int shift = bit_begin; shift < bit_end; shift += kRadixBits) {
    hipLaunchKernelGGL(radix_hist_kernel, dim3((unsigned)nblk), dim3(kBlock), 0, stream, (const uint64_t*)kin, n,
                       shift, hist, nblk);
    int rc = exclusive_scan_u32(hist, nblk * kRadixBins, scan_scratch, stream);
    if (rc != GNNAGG_OK) return rc;
    hipLaunchKernelGGL(radix_scatter_kernel, dim3((unsigned)nblk), dim3(kBlock), 0, stream, (const uint64_t*)kin,
                       (const uint32_t*)vin, kout, vout, n, shift, (const uint32_t*)hist, nblk);
    GNNAGG_HIP_TRY(hipGetLastError());
    uint64_t* tk = kin; kin = kout; kout = tk;
    uint32_t* tv = vin; vin = vout; vout = tv;
    *in_a = !*in_a;
  }
  return GNNAGG_OK;
}

}  // namespace gnnagg
