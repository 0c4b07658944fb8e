// Element-wise AdamW for the parameters APOLLO does not project (Section 3.1, Eq. 1, with the
// decoupled decay term of Algorithm 1, step 4).  Pure streaming: per parameter W read + write
// (8 B; 4 B when stored in bfloat16), M and V read + write (16 B; 8 B), G read (2 or 4 B).
//
// One launch covers the whole tensor list: block b looks its tensor up in a table, and works on
// 1024 consecutive elements of it, one thread = four consecutive elements = one 16-byte access
// per array, blocks in memory order, all arrays streamed with non-temporal accesses (the shape
// that moves 6.4 TB/s in the APOLLO weight update).
#include "apollo_internal.h"

namespace apollo {

namespace {

// STORE16: M and V are kept in bfloat16: they are rounded (to nearest even) before anything else
// uses them, so the update is formed from what is stored.
template <bool STORE16>
__device__ __forceinline__ void adamw_element(float g, float& w, float& m, float& v, const AdamwParams& p) {
  m = __builtin_fmaf(p.beta1, m, p.omb1 * g);
  v = __builtin_fmaf(p.beta2, v, p.omb2 * (g * g));
  if (STORE16) {
    m = bf16_bits_to_f32(f32_to_bf16_bits(m));
    v = bf16_bits_to_f32(f32_to_bf16_bits(v));
  }
  // hardware square root and reciprocal (1 ulp each): the kernel only streams otherwise
  const float u = (m * p.inv_bc1) * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(v * p.inv_bc2) + p.eps);
  w = __builtin_fmaf(-p.lr, u, __builtin_fmaf(-p.lr_decay, w, w));
}

// four consecutive elements of a W / M / V array (fp32 or bf16) at element e0 (a multiple of 4), streamed
template <bool STORE16>
__device__ __forceinline__ f32x4_t load_quad(const APOLLO_GLOBAL void* base, uint64_t e0) {
  if constexpr (STORE16) {
    const u32x2_t h = __builtin_nontemporal_load(
        reinterpret_cast<const APOLLO_GLOBAL u32x2_t*>(reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(base) + e0));
    return mk_f4(__uint_as_float(h.x << 16), __uint_as_float(h.x & 0xFFFF0000u), __uint_as_float(h.y << 16),
                 __uint_as_float(h.y & 0xFFFF0000u));
  } else {
    return __builtin_nontemporal_load(
        reinterpret_cast<const APOLLO_GLOBAL f32x4_t*>(reinterpret_cast<const APOLLO_GLOBAL float*>(base) + e0));
  }
}
// the counterpart store; ROUND: the values still have to be rounded to bfloat16 (W), otherwise they
// already are bfloat16 numbers (M, V) and the store truncates
template <bool STORE16, bool ROUND>
__device__ __forceinline__ void store_quad(APOLLO_GLOBAL void* base, uint64_t e0, f32x4_t x) {
  if constexpr (STORE16) {
    uint32_t b[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) b[e] = ROUND ? f32_to_bf16_bits(x[e]) : (__float_as_uint(x[e]) >> 16);
    u32x2_t h = {b[0] | (b[1] << 16), b[2] | (b[3] << 16)};
    __builtin_nontemporal_store(h, reinterpret_cast<APOLLO_GLOBAL u32x2_t*>(reinterpret_cast<APOLLO_GLOBAL uint16_t*>(base) + e0));
  } else {
    __builtin_nontemporal_store(x, reinterpret_cast<APOLLO_GLOBAL f32x4_t*>(reinterpret_cast<APOLLO_GLOBAL float*>(base) + e0));
  }
}
template <bool STORE16>
__device__ __forceinline__ float load_one(const APOLLO_GLOBAL void* base, uint64_t e) {
  if constexpr (STORE16) return bf16_bits_to_f32(reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(base)[e]);
  else return reinterpret_cast<const APOLLO_GLOBAL float*>(base)[e];
}
template <bool STORE16>
__device__ __forceinline__ void store_one(APOLLO_GLOBAL void* base, uint64_t e, float x) {
  if constexpr (STORE16) reinterpret_cast<APOLLO_GLOBAL uint16_t*>(base)[e] = (uint16_t)f32_to_bf16_bits(x);
  else reinterpret_cast<APOLLO_GLOBAL float*>(base)[e] = x;
}

template <bool STORE16>
__device__ __forceinline__ void adamw_block(const AdamwDesc& d, uint64_t e0, const AdamwParams& p) {
  APOLLO_GLOBAL void* w = gptr(d.w);
  APOLLO_GLOBAL void* m = gptr(d.m);
  APOLLO_GLOBAL void* v = gptr(d.v);
  if (e0 + 4 <= d.numel) {
    f32x4_t wv = load_quad<STORE16>(w, e0);
    f32x4_t mv = load_quad<STORE16>(m, e0);
    f32x4_t vv = load_quad<STORE16>(v, e0);
    float g[4];
    if (d.bf16) {
      const u32x2_t gv = __builtin_nontemporal_load(
          reinterpret_cast<const APOLLO_GLOBAL u32x2_t*>(reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(gptr(d.g)) + e0));
      g[0] = __uint_as_float(gv.x << 16);
      g[1] = __uint_as_float(gv.x & 0xFFFF0000u);
      g[2] = __uint_as_float(gv.y << 16);
      g[3] = __uint_as_float(gv.y & 0xFFFF0000u);
    } else {
      const f32x4_t gv = __builtin_nontemporal_load(
          reinterpret_cast<const APOLLO_GLOBAL f32x4_t*>(reinterpret_cast<const APOLLO_GLOBAL float*>(gptr(d.g)) + e0));
      g[0] = gv.x; g[1] = gv.y; g[2] = gv.z; g[3] = gv.w;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float we = wv[e], me = mv[e], ve = vv[e];
      adamw_element<STORE16>(g[e], we, me, ve, p);
      wv[e] = we; mv[e] = me; vv[e] = ve;
    }
    store_quad<STORE16, true>(w, e0, wv);
    store_quad<STORE16, false>(m, e0, mv);
    store_quad<STORE16, false>(v, e0, vv);
  } else {
    // ragged tail of the tensor: up to three elements, one at a time
    const int left = (int)(d.numel - e0);
    for (int e = 0; e < left; ++e) {
      const float g = d.bf16 ? __uint_as_float((uint32_t)reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(gptr(d.g))[e0 + e] << 16)
                             : reinterpret_cast<const APOLLO_GLOBAL float*>(gptr(d.g))[e0 + e];
      float we = load_one<STORE16>(w, e0 + e), me = load_one<STORE16>(m, e0 + e), ve = load_one<STORE16>(v, e0 + e);
      adamw_element<STORE16>(g, we, me, ve, p);
      store_one<STORE16>(w, e0 + e, we);
      store_one<STORE16>(m, e0 + e, me);
      store_one<STORE16>(v, e0 + e, ve);
    }
  }
}

__global__ __launch_bounds__(256) void adamw_kernel(const AdamwDesc* __restrict__ descs,
                                                    const uint32_t* __restrict__ block_tensor, AdamwParams p) {
  const AdamwDesc d = descs[block_tensor[blockIdx.x]];
  const uint64_t e0 = ((uint64_t)(blockIdx.x - d.first_block) * 256u + threadIdx.x) * 4u;
  if (e0 >= d.numel) return;
  if (d.store16) adamw_block<true>(d, e0, p);      // uniform over the block: a tensor has one storage type
  else adamw_block<false>(d, e0, p);
}

}  // namespace

hipError_t launch_adamw(const AdamwDesc* d_descs, const uint32_t* d_block_tensor, uint32_t n_blocks,
                        const AdamwParams& p, hipStream_t st) {
  if (n_blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(adamw_kernel, dim3(n_blocks), dim3(256), 0, st, d_descs, d_block_tensor, p);
  return hipGetLastError();
}

}  // namespace apollo
