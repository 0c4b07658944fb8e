// Element-wise AdamW for the parameters APOLLO does not project (Section 3.1, Eq. 1, with the
// decoupled decay term of Algorithm 1, step 4).  Pure streaming: per parameter W read + write
// (8 B), M and V read + write (16 B), G read (2 or 4 B).
//
// One launch covers the whole tensor list: block b looks its tensor up in a table, and works on
// 1024 consecutive elements of it, one thread = four consecutive elements = one 16-byte access
// per array, blocks in memory order, all arrays streamed with non-temporal accesses (the shape
// that moves 6.4 TB/s in the APOLLO weight update).
#include "apollo_internal.h"

namespace apollo {

namespace {

__device__ __forceinline__ void adamw_element(float g, float& w, float& m, float& v, const AdamwParams& p) {
  m = __builtin_fmaf(p.beta1, m, p.omb1 * g);
  v = __builtin_fmaf(p.beta2, v, p.omb2 * (g * g));
  // hardware square root and reciprocal (1 ulp each): the kernel only streams otherwise
  const float u = (m * p.inv_bc1) * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(v * p.inv_bc2) + p.eps);
  w = __builtin_fmaf(-p.lr, u, __builtin_fmaf(-p.lr_decay, w, w));
}

__global__ __launch_bounds__(256) void adamw_kernel(const AdamwDesc* __restrict__ descs,
                                                    const uint32_t* __restrict__ block_tensor, AdamwParams p) {
  const AdamwDesc d = descs[block_tensor[blockIdx.x]];
  const uint64_t e0 = ((uint64_t)(blockIdx.x - d.first_block) * 256u + threadIdx.x) * 4u;
  if (e0 >= d.numel) return;
  APOLLO_GLOBAL float* w = gptr(d.w) + e0;
  APOLLO_GLOBAL float* m = gptr(d.m) + e0;
  APOLLO_GLOBAL float* v = gptr(d.v) + e0;
  if (e0 + 4 <= d.numel) {
    f32x4_t wv = __builtin_nontemporal_load(reinterpret_cast<APOLLO_GLOBAL f32x4_t*>(w));
    f32x4_t mv = __builtin_nontemporal_load(reinterpret_cast<APOLLO_GLOBAL f32x4_t*>(m));
    f32x4_t vv = __builtin_nontemporal_load(reinterpret_cast<APOLLO_GLOBAL f32x4_t*>(v));
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
      adamw_element(g[e], we, me, ve, p);
      wv[e] = we; mv[e] = me; vv[e] = ve;
    }
    __builtin_nontemporal_store(wv, reinterpret_cast<APOLLO_GLOBAL f32x4_t*>(w));
    __builtin_nontemporal_store(mv, reinterpret_cast<APOLLO_GLOBAL f32x4_t*>(m));
    __builtin_nontemporal_store(vv, reinterpret_cast<APOLLO_GLOBAL f32x4_t*>(v));
  } else {
    // ragged tail of the tensor: up to three elements, one at a time
    const int left = (int)(d.numel - e0);
    for (int e = 0; e < left; ++e) {
      const float g = d.bf16 ? __uint_as_float((uint32_t)reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(gptr(d.g))[e0 + e] << 16)
                             : reinterpret_cast<const APOLLO_GLOBAL float*>(gptr(d.g))[e0 + e];
      float we = w[e], me = m[e], ve = v[e];
      adamw_element(g, we, me, ve, p);
      w[e] = we; m[e] = me; v[e] = ve;
    }
  }
}

}  // namespace

hipError_t launch_adamw(const AdamwDesc* d_descs, const uint32_t* d_block_tensor, uint32_t n_blocks,
                        const AdamwParams& p, hipStream_t st) {
  if (n_blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(adamw_kernel, dim3(n_blocks), dim3(256), 0, st, d_descs, d_block_tensor, p);
  return hipGetLastError();
}

}  // namespace apollo
