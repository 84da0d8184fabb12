// Stable LSD radix sort (digits of up to 9 bits) and exclusive scan for gfx950.
//
// One sort pass = three launches: per-workgroup digit histograms, a scan of the
// digit-major histogram table, and a scatter in which every key finds its
// stable rank inside its workgroup tile with wave ballots (64-lane match on the
// digit) and a small LDS table across the four waves; the tile is sorted by digit
// in LDS and leaves it in whole runs.  No global atomics, so the output order is
// unique.
//
// What a pass moves is what bounds it, so the sort moves as little as it can: the
// digit width is chosen so that the key bits take the fewest passes (36 bits: four
// passes of 9, not five of 8), a sort whose caller does not ask for the permutation
// carries no values at all (a stable sort needs none to keep ties in input order),
// and the first pass of the CSR build forms its keys from the COO arrays on the fly
// instead of reading a key array written by a pass of its own.
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

// Key of element i: from the key array, or (first pass of the CSR build) formed from the COO arrays:
// (destination << src_bits) | source, the appended self-loop i - E for i >= E.  Out-of-range endpoints
// are clamped, so that every later access stays in range, and reported through *bad.
__device__ inline uint64_t load_key(const KeySource& in, int64_t i) {
  if (in.keys) return in.keys[i];
  int64_t s, d;
  if (i < in.E) {
    s = in.src[i];
    d = in.dst[i];
    if (s < 0 || s >= in.N || d < 0 || d >= in.N) {
      *in.bad = 1u;
      s = 0;
      d = 0;
    }
  } else {
    s = d = i - in.E;
  }
  return ((uint64_t)d << in.src_bits) | (uint64_t)s;
}

// Which tile a workgroup takes.  Workgroups are dealt to the eight XCDs round-robin (workgroup b runs on
// XCD b mod 8) and every XCD has an L2 of its own; the tiles are handed out so that each XCD works through
// one contiguous eighth of the array: consecutive tiles - whose histogram entries and whose runs of equal
// digits are neighbours in memory - are then written through the same L2 and leave it as whole lines.
__device__ inline int64_t tile_of_workgroup(uint32_t block, int64_t tiles_per_xcd) {
  return (int64_t)(block & 7u) * tiles_per_xcd + (int64_t)(block >> 3);
}

template <int ITEMS>
__global__ __launch_bounds__(kBlock) void radix_hist_kernel(const KeySource in, int64_t n, int shift, int bits,
                                                            uint32_t* __restrict__ hist, int64_t nblk,
                                                            int64_t tiles_per_xcd) {
  __shared__ uint32_t h[kMaxRadixBins];
  const int64_t t = tile_of_workgroup(blockIdx.x, tiles_per_xcd);
  if (t >= nblk) return;
  const uint32_t mask = (1u << bits) - 1u;
  for (int d = threadIdx.x; d <= (int)mask; d += kBlock) h[d] = 0;
  __syncthreads();
  const int64_t base = t * (kBlock * ITEMS);
  uint32_t d[ITEMS];  // every load is issued before the first counter is touched
#pragma unroll
  for (int r = 0; r < ITEMS; ++r) {
    const int64_t i = base + (int64_t)r * kBlock + threadIdx.x;
    d[r] = (i < n) ? ((uint32_t)(load_key(in, i) >> shift) & mask) : 0xffffffffu;
  }
#pragma unroll
  for (int r = 0; r < ITEMS; ++r)
    if (d[r] != 0xffffffffu) atomicAdd(&h[d[r]], 1u);
  __syncthreads();
  for (int d = threadIdx.x; d <= (int)mask; d += kBlock) hist[(int64_t)d * nblk + t] = h[d];
}

// One workgroup scatters one tile of kBlock * ITEMS keys.  The tile is cut into four contiguous quarters,
// one per wave; a wave keeps its ITEMS x 64 keys in registers.  Phase 1: every wave counts its quarter per
// digit (wave ballots find the lanes that hold the same digit; the first lane of each such group adds the
// group size to an LDS counter).  The digits are then scanned: where digit d starts in the tile sorted by
// digit, and inside that where each wave's keys with that digit go.  Phase 2: every wave walks its rounds
// again, alone - position = running start of (wave, digit) + rank inside the group - and stores key (and
// value) at that place IN LDS.  Phase 3: the sorted tile leaves LDS in order, so the keys of one digit go to
// consecutive global addresses (whole lines, not one 8-byte store per lane and digit).  Equal digits keep
// their input order: the sort is stable, and no global atomic is involved.
//
// LDS hand-off inside a wave: in every round only the first lane of a digit group touches the group's
// counter (groups of one round have different digits, hence different counters) and hands the value to
// the rest of its group with a shuffle; rounds are separated by a wavefront fence, so no lane reads a
// counter another lane is about to write.
template <int ITEMS, bool HAS_VALS>
__global__ __launch_bounds__(kBlock) void radix_scatter_kernel(const KeySource in, const uint32_t* __restrict__ vin,
                                                               uint64_t* __restrict__ kout,
                                                               uint32_t* __restrict__ vout, int64_t n, int shift,
                                                               int bits, const uint32_t* __restrict__ hist_scanned,
                                                               int64_t nblk, int64_t tiles_per_xcd) {
  constexpr int kTile = kBlock * ITEMS;
  const int64_t t = tile_of_workgroup(blockIdx.x, tiles_per_xcd);
  if (t >= nblk) return;
  __shared__ uint64_t lkey[kTile];
  __shared__ uint32_t lval[HAS_VALS ? kTile : 1];
  __shared__ uint32_t start[kWavesPerBlock][kMaxRadixBins];  // counts in phase 1, running local positions after
  __shared__ uint32_t shift_out[kMaxRadixBins];              // global position minus local position, per digit
  __shared__ uint32_t lds4[kWavesPerBlock];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const uint32_t mask = (1u << bits) - 1u;
  const int per = ((int)mask + kBlock) / kBlock;  // digits per thread in the digit scan: 1 (up to 8 bits) or 2
  for (int d = tid; d <= (int)mask; d += kBlock) {
#pragma unroll
    for (int k = 0; k < kWavesPerBlock; ++k) start[k][d] = 0;
  }
  __syncthreads();
  constexpr int kQuarter = kTile / kWavesPerBlock;  // keys per wave
  const int64_t tile = t * kTile;
  const int64_t first = tile + (int64_t)w * kQuarter + lane;
  const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
  uint64_t key[ITEMS];
  uint32_t val[HAS_VALS ? ITEMS : 1];
  uint32_t group[ITEMS];  // rank inside the digit group (bits 0-7), first lane of the group (8-15), group size - 1 (16-23), valid (24)
  // all loads first: the fences of the counting rounds below must not stand between them
#pragma unroll
  for (int r = 0; r < ITEMS; ++r) {
    const int64_t i = first + (int64_t)r * kWave;
    const bool valid = i < n;
    key[r] = valid ? load_key(in, i) : 0ull;
    if constexpr (HAS_VALS) val[r] = valid ? (vin ? vin[i] : (uint32_t)i) : 0u;
  }
#pragma unroll
  for (int r = 0; r < ITEMS; ++r) {
    const bool valid = first + (int64_t)r * kWave < n;
    const uint32_t d = (uint32_t)(key[r] >> shift) & mask;
    uint64_t same = __ballot(valid);  // lanes of this wave that hold the same digit
#pragma unroll
    for (int b = 0; b < kMaxRadixBits; ++b) {
      if (b < bits) {  // uniform
        const bool bit = (d >> b) & 1u;
        const uint64_t bal = __ballot(valid && bit);
        same &= bit ? bal : ~bal;
      }
    }
    const uint32_t rank = (uint32_t)__popcll(same & below), size = (uint32_t)__popcll(same);
    const uint32_t leader = valid ? (uint32_t)(__ffsll((unsigned long long)same) - 1) : 0u;
    group[r] = rank | (leader << 8) | ((size - (valid ? 1u : 0u)) << 16) | (valid ? 1u << 24 : 0u);
    if (valid && rank == 0) start[w][d] += size;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  }
  __syncthreads();
  {
    // thread t owns the digits t * per .. t * per + per - 1 (ascending, so the scan over threads is the scan over digits)
    uint32_t c[2][kWavesPerBlock], tot = 0;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
#pragma unroll
      for (int k = 0; k < kWavesPerBlock; ++k) {
        const int d = tid * per + q;
        c[q][k] = (q < per && d <= (int)mask) ? start[k][d] : 0u;
        tot += c[q][k];
      }
    }
    uint32_t all;
    uint32_t b = block_exclusive_scan(tot, lds4, &all);  // where this thread's first digit starts in the sorted tile
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int d = tid * per + q;
      if (q < per && d <= (int)mask) {
        shift_out[d] = hist_scanned[(int64_t)d * nblk + t] - b;  // modulo 2^32, undone below
#pragma unroll
        for (int k = 0; k < kWavesPerBlock; ++k) {
          start[k][d] = b;
          b += c[q][k];
        }
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < ITEMS; ++r) {
    const bool valid = (group[r] >> 24) & 1u;
    const uint32_t d = (uint32_t)(key[r] >> shift) & mask;
    const uint32_t rank = group[r] & 0xffu, leader = (group[r] >> 8) & 0xffu, size = ((group[r] >> 16) & 0xffu) + 1u;
    uint32_t base = 0;
    if (valid && rank == 0) {  // the group's first lane takes the group's place and moves the counter on
      base = start[w][d];
      start[w][d] = base + size;
    }
    base = __shfl(base, (int)leader, kWave);
    if (valid) {
      lkey[base + rank] = key[r];
      if constexpr (HAS_VALS) lval[base + rank] = val[r];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  }
  __syncthreads();
  const int64_t left = n - tile;
  const int count = left < kTile ? (int)left : kTile;  // keys in this tile
  for (int p = tid; p < count; p += kBlock) {
    const uint64_t k = lkey[p];
    const uint32_t d = (uint32_t)(k >> shift) & mask;
    const uint32_t pos = (uint32_t)p + shift_out[d];
    kout[pos] = k;
    if constexpr (HAS_VALS) vout[pos] = lval[p];
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

int radix_digit_bits(int key_bits) {
  if (key_bits <= 0) return 1;
  const int passes = (key_bits + kMaxRadixBits - 1) / kMaxRadixBits;
  return (key_bits + passes - 1) / passes;  // the narrowest digit that needs no more passes than the widest
}

int radix_sort(const KeySource& first, uint64_t* keys_a, uint32_t* vals_a, uint64_t* keys_b, uint32_t* vals_b,
               int64_t n, int bit_begin, int bit_end, bool with_vals, uint32_t* hist, uint32_t* scan_scratch,
               hipStream_t stream, bool* in_a) {
  *in_a = true;
  if (n <= 0) return GNNAGG_OK;
  const int64_t nblk = sort_blocks(n, with_vals);
  const int64_t tiles_per_xcd = ceil_div(nblk, 8);
  if (8 * tiles_per_xcd > 0x7fffffff) return GNNAGG_EUNSUPPORTED;
  const int digit = radix_digit_bits(bit_end - bit_begin);
  KeySource in = first;         // the first pass reads where the caller says (key array a, or the COO arrays)
  const uint32_t* vin = first.keys ? vals_a : nullptr;  // keys formed on the fly carry their index as the value
  uint64_t* kout = keys_b;
  uint32_t* vout = vals_b;
  bool out_is_b = true;
  for (int shift = bit_begin; shift < bit_end; shift += digit) {
    const int bits = (bit_end - shift < digit) ? bit_end - shift : digit;
    const dim3 grid((unsigned)(8 * tiles_per_xcd)), block(kBlock);
    if (with_vals)
      hipLaunchKernelGGL(radix_hist_kernel<kSortItemsPairs>, grid, block, 0, stream, in, n, shift, bits, hist, nblk,
                         tiles_per_xcd);
    else
      hipLaunchKernelGGL(radix_hist_kernel<kSortItemsKeys>, grid, block, 0, stream, in, n, shift, bits, hist, nblk,
                         tiles_per_xcd);
    int rc = exclusive_scan_u32(hist, nblk << bits, scan_scratch, stream);
    if (rc != GNNAGG_OK) return rc;
    if (with_vals)
      hipLaunchKernelGGL((radix_scatter_kernel<kSortItemsPairs, true>), grid, block, 0, stream, in, vin, kout, vout, n,
                         shift, bits, (const uint32_t*)hist, nblk, tiles_per_xcd);
    else
      hipLaunchKernelGGL((radix_scatter_kernel<kSortItemsKeys, false>), grid, block, 0, stream, in,
                         (const uint32_t*)nullptr, kout, (uint32_t*)nullptr, n, shift, bits, (const uint32_t*)hist,
                         nblk, tiles_per_xcd);
    GNNAGG_HIP_TRY(hipGetLastError());
    in = KeySource();
    in.keys = kout;
    vin = vout;
    *in_a = !out_is_b;
    out_is_b = !out_is_b;
    kout = out_is_b ? keys_b : keys_a;
    vout = out_is_b ? vals_b : vals_a;
  }
  return GNNAGG_OK;
}

}  // namespace gnnagg
