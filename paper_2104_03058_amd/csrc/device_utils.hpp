// Device-side helpers shared by the aggregation and attention kernels:
// element-aligned vector loads/stores of feature rows.
#pragma once
#include "common.hpp"

namespace gnnagg {

struct bf16_t { uint16_t bits; };

// Under-aligned vector types: rows start at any element boundary (F is
// arbitrary), so vector accesses promise only element alignment.
typedef float f32x2_u __attribute__((ext_vector_type(2), aligned(4)));
typedef float f32x4_u __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x1_h __attribute__((aligned(2)));
typedef uint32_t u32x2_h __attribute__((ext_vector_type(2), aligned(2)));
typedef uint32_t u32x4_h __attribute__((ext_vector_type(4), aligned(2)));

template <typename T, int VEC> struct Raw;
template <> struct Raw<float, 1> { typedef float type; };
template <> struct Raw<float, 2> { typedef f32x2_u type; };
template <> struct Raw<float, 4> { typedef f32x4_u type; };
template <> struct Raw<bf16_t, 1> { typedef uint16_t type; };
template <> struct Raw<bf16_t, 2> { typedef u32x1_h type; };
template <> struct Raw<bf16_t, 4> { typedef u32x2_h type; };
template <> struct Raw<bf16_t, 8> { typedef u32x4_h type; };

template <typename T, int VEC>
__device__ inline typename Raw<T, VEC>::type load_raw(const T* p) {
  return *reinterpret_cast<const typename Raw<T, VEC>::type*>(p);
}

__device__ inline float bf16lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ inline float bf16hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }

__device__ inline void unpack(float r, float (&v)[1]) { v[0] = r; }
__device__ inline void unpack(f32x2_u r, float (&v)[2]) { v[0] = r.x; v[1] = r.y; }
__device__ inline void unpack(f32x4_u r, float (&v)[4]) { v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w; }
__device__ inline void unpack(uint16_t r, float (&v)[1]) { v[0] = __uint_as_float((uint32_t)r << 16); }
__device__ inline void unpack(u32x1_h r, float (&v)[2]) { v[0] = bf16lo(r); v[1] = bf16hi(r); }
__device__ inline void unpack(u32x2_h r, float (&v)[4]) {
  v[0] = bf16lo(r.x); v[1] = bf16hi(r.x); v[2] = bf16lo(r.y); v[3] = bf16hi(r.y);
}
__device__ inline void unpack(u32x4_h r, float (&v)[8]) {
  v[0] = bf16lo(r.x); v[1] = bf16hi(r.x); v[2] = bf16lo(r.y); v[3] = bf16hi(r.y);
  v[4] = bf16lo(r.z); v[5] = bf16hi(r.z); v[6] = bf16lo(r.w); v[7] = bf16hi(r.w);
}

// All-ones for an entry that exists, zero for one that does not, as a value the optimiser cannot see through:
// ANDed into the raw bits of a loaded row piece it makes a missing entry an exact +0 at one integer
// instruction per 32 bits loaded.  (Written as a select on the widened value the same masking costs two
// selects per fp64 value, because the compiler moves a select on the fp32 value behind the conversion.)
__device__ inline uint32_t keep_bits(bool ok) {
  uint32_t m = ok ? 0xffffffffu : 0u;
  asm("" : "+v"(m));
  return m;
}
__device__ inline float and_bits(float r, uint32_t m) { return __uint_as_float(__float_as_uint(r) & m); }
__device__ inline f32x2_u and_bits(f32x2_u r, uint32_t m) {
  f32x2_u o; o.x = and_bits((float)r.x, m); o.y = and_bits((float)r.y, m);
  return o;
}
__device__ inline f32x4_u and_bits(f32x4_u r, uint32_t m) {
  f32x4_u o; o.x = and_bits((float)r.x, m); o.y = and_bits((float)r.y, m); o.z = and_bits((float)r.z, m);
  o.w = and_bits((float)r.w, m);
  return o;
}
__device__ inline uint16_t and_bits(uint16_t r, uint32_t m) { return (uint16_t)(r & m); }
__device__ inline u32x1_h and_bits(u32x1_h r, uint32_t m) { return r & m; }
__device__ inline u32x2_h and_bits(u32x2_h r, uint32_t m) { u32x2_h o; o.x = r.x & m; o.y = r.y & m; return o; }
__device__ inline u32x4_h and_bits(u32x4_h r, uint32_t m) {
  u32x4_h o; o.x = r.x & m; o.y = r.y & m; o.z = r.z & m; o.w = r.w & m;
  return o;
}

template <int VEC>
__device__ inline void store_row(float* p, const float (&v)[VEC]) {
  if constexpr (VEC == 1) {
    p[0] = v[0];
  } else if constexpr (VEC == 2) {
    f32x2_u r; r.x = v[0]; r.y = v[1];
    *reinterpret_cast<f32x2_u*>(p) = r;
  } else {
#pragma unroll
    for (int k = 0; k < VEC; k += 4) {
      f32x4_u r; r.x = v[k]; r.y = v[k + 1]; r.z = v[k + 2]; r.w = v[k + 3];
      *reinterpret_cast<f32x4_u*>(p + k) = r;
    }
  }
}

// fp32 -> bf16 bits, round to nearest even (inputs here are finite or infinite, never NaN by contract;
// a NaN keeps a non-zero mantissa)
__device__ inline uint32_t bf16_bits(float f) {
  const uint32_t b = __float_as_uint(f);
  if ((b & 0x7fffffffu) > 0x7f800000u) return (b >> 16) | 0x40u;
  return (b + 0x7fffu + ((b >> 16) & 1u)) >> 16;
}

template <int VEC>
__device__ inline void store_row_bf16(uint16_t* p, const float (&v)[VEC]) {
  if constexpr (VEC == 1) {
    p[0] = (uint16_t)bf16_bits(v[0]);
  } else {
    typedef uint32_t u32_h __attribute__((aligned(2)));
#pragma unroll
    for (int k = 0; k < VEC; k += 2)
      *reinterpret_cast<u32_h*>(p + k) = bf16_bits(v[k]) | (bf16_bits(v[k + 1]) << 16);
  }
}

}  // namespace gnnagg
