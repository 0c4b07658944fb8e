// Streamed access to the moment arrays M^R, V^R (fp32 or bfloat16), shared by the kernels that
// update them (Algorithm 1, step 2).
#pragma once
#include "apollo_internal.h"

namespace apollo {

// VEC consecutive elements of a moment array at element index idx, as floats; the array is fp32
// or bfloat16 (SB16).  Streamed (non-temporal).  idx is a multiple of VEC and the arrays are
// aligned so that the VEC elements form one naturally aligned access.
template <int VEC, bool SB16, bool UA = false>
__device__ __forceinline__ float __attribute__((ext_vector_type(VEC))) load_state(const APOLLO_GLOBAL void* base, size_t idx) {
  typedef float vec_t __attribute__((ext_vector_type(VEC)));
  // UA: idx is any element index; the access is only aligned to its element type (the compiler
  // then picks instructions that are valid for that alignment)
  typedef float vec_ua_t __attribute__((ext_vector_type(VEC), aligned(4)));
  typedef uint32_t u32x2_ua_t __attribute__((ext_vector_type(2), aligned(2)));
  if constexpr (!SB16) {
    if constexpr (UA) {
      const vec_ua_t t = __builtin_nontemporal_load(reinterpret_cast<const APOLLO_GLOBAL vec_ua_t*>(reinterpret_cast<const APOLLO_GLOBAL float*>(base) + idx));
      vec_t v;
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[e] = t[e];
      return v;
    } else {
      return __builtin_nontemporal_load(reinterpret_cast<const APOLLO_GLOBAL vec_t*>(reinterpret_cast<const APOLLO_GLOBAL float*>(base) + idx));
    }
  } else if constexpr (VEC == 4) {
    u32x2_t h;
    if constexpr (UA) {
      const u32x2_ua_t t = __builtin_nontemporal_load(reinterpret_cast<const APOLLO_GLOBAL u32x2_ua_t*>(reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(base) + idx));
      h.x = t.x;
      h.y = t.y;
    } else {
      h = __builtin_nontemporal_load(reinterpret_cast<const APOLLO_GLOBAL u32x2_t*>(reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(base) + idx));
    }
    vec_t v = {__uint_as_float(h.x << 16), __uint_as_float(h.x & 0xFFFF0000u), __uint_as_float(h.y << 16), __uint_as_float(h.y & 0xFFFF0000u)};
    return v;
  } else {
    static_assert(VEC == 1 || VEC == 4, "VEC");
    vec_t v = {bf16_bits_to_f32(reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(base)[idx])};
    return v;
  }
}

// The values are already bfloat16 numbers when SB16 (rounded by the caller): the store truncates.
template <int VEC, bool SB16, bool UA = false>
__device__ __forceinline__ void store_state(APOLLO_GLOBAL void* base, size_t idx, float __attribute__((ext_vector_type(VEC))) v) {
  typedef float vec_t __attribute__((ext_vector_type(VEC)));
  typedef float vec_ua_t __attribute__((ext_vector_type(VEC), aligned(4)));
  typedef uint32_t u32x2_ua_t __attribute__((ext_vector_type(2), aligned(2)));
  if constexpr (!SB16) {
    if constexpr (UA) {
      vec_ua_t t;
#pragma unroll
      for (int e = 0; e < VEC; ++e) t[e] = v[e];
      __builtin_nontemporal_store(t, reinterpret_cast<APOLLO_GLOBAL vec_ua_t*>(reinterpret_cast<APOLLO_GLOBAL float*>(base) + idx));
    } else {
      __builtin_nontemporal_store(v, reinterpret_cast<APOLLO_GLOBAL vec_t*>(reinterpret_cast<APOLLO_GLOBAL float*>(base) + idx));
    }
  } else if constexpr (VEC == 4) {
    u32x2_t h;
    h.x = (__float_as_uint(v[0]) >> 16) | (__float_as_uint(v[1]) & 0xFFFF0000u);
    h.y = (__float_as_uint(v[2]) >> 16) | (__float_as_uint(v[3]) & 0xFFFF0000u);
    if constexpr (UA) {
      u32x2_ua_t t;
      t.x = h.x;
      t.y = h.y;
      __builtin_nontemporal_store(t, reinterpret_cast<APOLLO_GLOBAL u32x2_ua_t*>(reinterpret_cast<APOLLO_GLOBAL uint16_t*>(base) + idx));
    } else {
      __builtin_nontemporal_store(h, reinterpret_cast<APOLLO_GLOBAL u32x2_t*>(reinterpret_cast<APOLLO_GLOBAL uint16_t*>(base) + idx));
    }
  } else {
    reinterpret_cast<APOLLO_GLOBAL uint16_t*>(base)[idx] = (uint16_t)(__float_as_uint(v[0]) >> 16);
  }
}

// The first `cnt` (1..3) of four consecutive elements, one at a time: the ragged end of a row whose
// length is not a multiple of 4.  Elements beyond cnt read as 0 and are not written.
template <bool SB16>
__device__ __forceinline__ f32x4_t load_state_part(const APOLLO_GLOBAL void* base, size_t idx, int cnt) {
  f32x4_t v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int e = 0; e < 3; ++e)
    if (e < cnt) v[e] = load_state<1, SB16>(base, idx + e)[0];
  return v;
}
template <bool SB16>
__device__ __forceinline__ void store_state_part(APOLLO_GLOBAL void* base, size_t idx, f32x4_t v, int cnt) {
  typedef float one_t __attribute__((ext_vector_type(1)));
#pragma unroll
  for (int e = 0; e < 3; ++e)
    if (e < cnt) {
      one_t o = {v[e]};
      store_state<1, SB16>(base, idx + e, o);
    }
}

}  // namespace apollo
