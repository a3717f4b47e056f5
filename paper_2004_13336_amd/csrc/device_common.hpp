// Device-side helpers shared by the kernel files: 128-bit accesses with a per-kernel cache policy,
// bfloat16 rounding, workspace addressing.  Everything is internal linkage.
#pragma once

#include "internal.hpp"

namespace su {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));


// Four consecutive floats held in registers; moved with one 128-bit access.
struct F4 {
  float x, y, z, w;
};

template <int MASK>
struct Policy {
  static constexpr bool RO = (MASK & 4) != 0, RW = (MASK & 2) != 0, ST = (MASK & 1) != 0;
};

template <bool NT, typename T>
__device__ __forceinline__ T ld(const T* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT, typename T>
__device__ __forceinline__ void st(T* p, T x) {
  if constexpr (NT) __builtin_nontemporal_store(x, p);
  else *p = x;
}
template <bool NT>
__device__ __forceinline__ F4 ld4(const float* p) {
  const f4 t = ld<NT>((const f4*)p);
  return F4{t.x, t.y, t.z, t.w};
}
template <bool NT>
__device__ __forceinline__ void st4(float* p, const F4& a) {
  f4 t;
  t.x = a.x; t.y = a.y; t.z = a.z; t.w = a.w;
  st<NT>((f4*)p, t);
}

// ---- bfloat16 ---------------------------------------------------------------------------------
// Round to nearest, ties to even, on the bit pattern; NaN keeps sign and upper payload and gets
// the quiet bit.
__device__ __forceinline__ uint32_t bf16_from_f32_bits(uint32_t b) {
  const uint32_t rounded = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
  const uint32_t quiet = (b >> 16) | 0x0040u;
  return ((b & 0x7FFFFFFFu) > 0x7F800000u) ? quiet : rounded;
}
__device__ __forceinline__ uint32_t bf16_of(float x) { return bf16_from_f32_bits(__float_as_uint(x)); }

template <bool NT>
__device__ __forceinline__ void store_bf16x4(uint16_t* p, const F4& w) {
  u2 o;
  o.x = bf16_of(w.x) | (bf16_of(w.y) << 16);
  o.y = bf16_of(w.z) | (bf16_of(w.w) << 16);
  st<NT>((u2*)p, o);
}

template <typename T>
inline T* ws_at(const shard_plan_t* p, size_t off) {
  return reinterpret_cast<T*>(p->ws.base + off);
}

}  // namespace
}  // namespace su
