// Stable LSD radix sort of (uint64 key, uint32 value) pairs and an exclusive
// scan, both running entirely in caller-provided device memory.  They serve the
// CSR build (edges sorted by destination, then source, then input position)
// and the degree-sorted row plan.
#pragma once
#include "common.hpp"

namespace gnnagg {

constexpr int kRadixBits = 8;
constexpr int kRadixBins = 1 << kRadixBits;
constexpr int kSortItemsPerThread = 10;  // 2,560-key tiles: 36 KB of LDS, four workgroups per compute unit (measured best of 4..16)
constexpr int kSortTile = kBlock * kSortItemsPerThread;  // keys per workgroup per pass

constexpr int kScanItemsPerThread = 16;
constexpr int kScanTile = kBlock * kScanItemsPerThread;

// uint32 scratch words an exclusive scan of n elements needs
size_t scan_scratch_words(int64_t n);

// In-place exclusive scan of n uint32 values (wraps modulo 2^32).
int exclusive_scan_u32(uint32_t* data, int64_t n, uint32_t* scratch, hipStream_t stream);

inline int64_t sort_blocks(int64_t n) { return ceil_div(n, kSortTile); }
// uint32 words of histogram storage a sort of n keys needs
inline size_t sort_hist_words(int64_t n) { return (size_t)sort_blocks(n) * kRadixBins; }

// Sorts by key bits [bit_begin, bit_end), stable.  Ping-pongs between the a and
// b buffers; *in_a tells where the result ended up.  hist needs
// sort_hist_words(n) words, scan_scratch needs scan_scratch_words(that) words.
int radix_sort_pairs(uint64_t* keys_a, uint32_t* vals_a, uint64_t* keys_b, uint32_t* vals_b, int64_t n,
                     int bit_begin, int bit_end, uint32_t* hist, uint32_t* scan_scratch, hipStream_t stream,
                     bool* in_a);

}  // namespace gnnagg
