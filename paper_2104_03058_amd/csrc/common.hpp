// Shared host-side helpers of libgnnagg (GPU path only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "gnnagg.h"

namespace gnnagg {

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kBlock = 256;        // threads per workgroup: 4 wavefronts
constexpr int kWavesPerBlock = kBlock / kWave;

#define GNNAGG_HIP_TRY(expr)                    \
  do {                                          \
    hipError_t e__ = (expr);                    \
    if (e__ != hipSuccess) return GNNAGG_EDEVICE; \
  } while (0)

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Carves 256-byte aligned pieces out of a caller-provided workspace.  With a
// null base it only adds up sizes (the size query of the workspace protocol).
struct Carver {
  char* base;
  size_t used = 0;
  explicit Carver(void* p) : base(static_cast<char*>(p)) {}
  template <typename T>
  T* take(size_t count) {
    size_t off = used;
    used += align_up(count * sizeof(T));
    return base ? reinterpret_cast<T*>(base + off) : nullptr;
  }
};

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

inline int bits_for(uint64_t max_value) {  // bits needed to hold values 0..max_value (at least 1)
  int b = 1;
  while (b < 64 && (max_value >> b) != 0) ++b;
  return b;
}

}  // namespace gnnagg
