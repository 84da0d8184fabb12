// Stable LSD radix sort of uint64 keys, with or without uint32 values, and an
// exclusive scan, both running entirely in caller-provided device memory.  They serve the
// CSR build (edges sorted by destination, then source, then input position)
// and the degree-sorted row plan.
#pragma once
#include "common.hpp"

namespace gnnagg {

constexpr int kMaxRadixBits = 9;  // digit width: 512 counters per wave in LDS, 9 wave ballots per key
constexpr int kMaxRadixBins = 1 << kMaxRadixBits;
// Keys per thread = tile size / 256.  With values: 2,560-key tiles (36 KB of LDS with the counters, four
// workgroups per compute unit); keys alone: 3,072-key tiles (longer runs per digit leave the tile, and the
// histogram table is shorter).
constexpr int kSortItemsPairs = 10;
constexpr int kSortItemsKeys = 12;

constexpr int kScanItemsPerThread = 16;
constexpr int kScanTile = kBlock * kScanItemsPerThread;

// uint32 scratch words an exclusive scan of n elements needs
size_t scan_scratch_words(int64_t n);

// In-place exclusive scan of n uint32 values (wraps modulo 2^32).
int exclusive_scan_u32(uint32_t* data, int64_t n, uint32_t* scratch, hipStream_t stream);

inline int64_t sort_blocks(int64_t n, bool with_vals) {
  return ceil_div(n, kBlock * (with_vals ? kSortItemsPairs : kSortItemsKeys));
}
// uint32 words of histogram storage a sort of n keys needs (sized for the widest digit and either tile size)
inline size_t sort_hist_words(int64_t n) { return (size_t)sort_blocks(n, true) * kMaxRadixBins; }

// Where the first pass of a sort finds its keys: a key array, or (keys == nullptr) the COO arrays of the CSR
// build, from which key i = (dst[i] << src_bits) | src[i] is formed on the fly; elements E .. n-1 are the
// appended self-loops.  *bad is set if an endpoint is outside [0, N).
struct KeySource {
  const uint64_t* keys = nullptr;
  const int32_t* src = nullptr;
  const int32_t* dst = nullptr;
  int64_t E = 0, N = 0;
  int src_bits = 0;
  uint32_t* bad = nullptr;
};

// Digit width the sort uses for a key of key_bits bits: the narrowest that needs the fewest passes.
int radix_digit_bits(int key_bits);

// Sorts n elements by key bits [bit_begin, bit_end), stable.  The first pass reads `first` (first.keys ==
// keys_a for an ordinary sort) and, with_vals, the values vals_a (or the element index as the value when the
// keys are formed on the fly); passes ping-pong between the b and a buffers; *in_a tells where the result
// ended up.  Without with_vals no value array is touched.  hist needs sort_hist_words(n) words,
// scan_scratch needs scan_scratch_words(that) words.
int radix_sort(const KeySource& first, uint64_t* keys_a, uint32_t* vals_a, uint64_t* keys_b, uint32_t* vals_b,
               int64_t n, int bit_begin, int bit_end, bool with_vals, uint32_t* hist, uint32_t* scan_scratch,
               hipStream_t stream, bool* in_a);

}  // namespace gnnagg
