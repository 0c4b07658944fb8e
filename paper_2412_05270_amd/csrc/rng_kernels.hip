// Kernels that materialise the random stream: the scratch copy of P that the matrix-core and the
// general projection read (written when the step's refresh interval differs from the one the
// scratch holds, i.e. once per T steps, and kept in between as Algorithm 1 keeps P_t; never state:
// a resumed run writes it again from the seed), and the debug views used by the bit-exact stream
// checks.  (Algorithm 1: "P_t <- N_seed(0, 1/r)".)
#include "apollo_internal.h"

namespace apollo {

// One thread per Philox call = four consecutive columns of one row of P.  Thread t handles
// half h = t & 1 of octet o of row kk with (t >> 1) = o * r + kk, so the stores of a wave are
// one contiguous run of the fragment-major scratch layout (8 bytes per thread for bf16).
template <bool BF16>
__global__ __launch_bounds__(256) void fill_projection_kernel(const TensorDesc* __restrict__ descs,
                                                              StepParams sp_arg, StepState* __restrict__ ss, int m8) {
  if (ss && !ss->regen) return;       // a replayed step whose scratch already holds this epoch's P
  const StepParams sp = step_params(sp_arg, ss);
  const TensorView d(descs[blockIdx.y]);
  const int r = sp.r;
  const size_t total = (size_t)r * (size_t)(m8 >> 2);
  const size_t t = (size_t)blockIdx.x * 256u + threadIdx.x;
  if (t >= total) return;
  const int h = (int)(t & 1u);
  const size_t rk = t >> 1;
  const int kk = (int)(rk % (size_t)r);
  const int o = (int)(rk / (size_t)r);
  const int q = 2 * o + h;
  const int m = d.m;
  const int mq = (m + 3) >> 2;
  float z[4] = {0.f, 0.f, 0.f, 0.f};
  if (q < mq) {
    projection_quad(sp.ks, sp.epoch, (uint32_t)d.tensor_id, (uint64_t)kk * (uint64_t)mq + (uint64_t)q, z);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (4 * q + e >= m) z[e] = 0.f;
  }
  if (BF16) {
    u32x2_t v;
    v.x = f32_to_bf16_bits(z[0]) | (f32_to_bf16_bits(z[1]) << 16);
    v.y = f32_to_bf16_bits(z[2]) | (f32_to_bf16_bits(z[3]) << 16);
    reinterpret_cast<APOLLO_GLOBAL u32x2_t*>(d.P)[t] = v;
  } else {
    reinterpret_cast<APOLLO_GLOBAL f32x4_t*>(d.P)[t] = mk_f4(z[0], z[1], z[2], z[3]);
  }
}

hipError_t launch_fill_projection(const TensorDesc* d_descs, int count, int r, int m8, bool bf16,
                                  const StepArgs& sa, hipStream_t st) {
  const size_t total = (size_t)r * (size_t)(m8 >> 2);
  dim3 grid((unsigned)((total + 255) / 256), (unsigned)count, 1);
  if (bf16)
    hipLaunchKernelGGL(fill_projection_kernel<true>, grid, dim3(256), 0, st, d_descs, sa.host, sa.dev, m8);
  else
    hipLaunchKernelGGL(fill_projection_kernel<false>, grid, dim3(256), 0, st, d_descs, sa.host, sa.dev, m8);
  return hipGetLastError();
}

// Copy of a bf16 gradient whose row length is not a multiple of eight elements into a scratch
// matrix with rows padded (zeros) to ldg elements, so that every row starts on a 16-byte boundary
// as the direct-to-LDS loads of the matrix-core projection need.  One thread per eight output
// elements, read with one element-aligned 16-byte load (the source rows have no common alignment).
__global__ __launch_bounds__(256) void pad_gradient_kernel(const TensorDesc* __restrict__ descs, int rows, int cols,
                                                           int ldg) {
  const TensorView d(descs[blockIdx.y]);
  const int oct_per_row = ldg >> 3;
  const size_t t = (size_t)blockIdx.x * 256u + threadIdx.x;
  if (t >= (size_t)rows * (size_t)oct_per_row) return;
  const int row = (int)(t / (size_t)oct_per_row);
  const int c0 = 8 * (int)(t % (size_t)oct_per_row);
  const APOLLO_GLOBAL uint16_t* src = reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(d.g) + (size_t)row * cols;
  uint32_t h[8];
  if (c0 + 8 <= cols) {
    // one 16-byte load that is only element-aligned (the rows have no common alignment)
    typedef uint16_t u16x8_ua_t __attribute__((ext_vector_type(8), aligned(2)));
    const u16x8_ua_t v = __builtin_nontemporal_load(reinterpret_cast<const APOLLO_GLOBAL u16x8_ua_t*>(src + c0));
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = v[e];
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = c0 + e < cols ? (uint32_t)src[c0 + e] : 0u;
  }
  reinterpret_cast<APOLLO_GLOBAL u32x4_t*>(d.gpad)[t] =
      mk_u4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
}

hipError_t launch_pad_gradient(const TensorDesc* d_descs, int count, int rows, int cols, int ldg, hipStream_t st) {
  const size_t total = (size_t)rows * (size_t)(ldg >> 3);
  dim3 grid((unsigned)((total + 255) / 256), (unsigned)count, 1);
  hipLaunchKernelGGL(pad_gradient_kernel, grid, dim3(256), 0, st, d_descs, rows, cols, ldg);
  return hipGetLastError();
}

// Row-major r x m view of the same stream (debug).
template <bool BF16>
__global__ __launch_bounds__(256) void fill_projection_rowmajor_kernel(void* __restrict__ out, int r, int m,
                                                                       uint32_t tensor_id, StepParams sp) {
  const int mq = (m + 3) >> 2;
  const size_t total = (size_t)r * (size_t)mq;
  const size_t t = (size_t)blockIdx.x * 256u + threadIdx.x;
  if (t >= total) return;
  const int kk = (int)(t / (size_t)mq);
  const int q = (int)(t % (size_t)mq);
  float z[4];
  projection_quad(sp.ks, sp.epoch, tensor_id, t, z);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int i = 4 * q + e;
    if (i < m) {
      const size_t o = (size_t)kk * (size_t)m + (size_t)i;
      if (BF16)
        reinterpret_cast<uint16_t*>(out)[o] = (uint16_t)f32_to_bf16_bits(z[e]);
      else
        reinterpret_cast<float*>(out)[o] = z[e];
    }
  }
}

hipError_t launch_fill_projection_rowmajor(void* out, bool out_bf16, int r, int m, uint32_t tensor_id,
                                           const StepParams& sp, hipStream_t st) {
  const size_t total = (size_t)r * (size_t)((m + 3) >> 2);
  dim3 grid((unsigned)((total + 255) / 256));
  if (out_bf16)
    hipLaunchKernelGGL(fill_projection_rowmajor_kernel<true>, grid, dim3(256), 0, st, out, r, m, tensor_id, sp);
  else
    hipLaunchKernelGGL(fill_projection_rowmajor_kernel<false>, grid, dim3(256), 0, st, out, r, m, tensor_id, sp);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void philox_words_kernel(const uint32_t* __restrict__ ctr, PhiloxKeySchedule ks,
                                                           uint32_t* __restrict__ out, int64_t count) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  uint32_t c[4] = {ctr[4 * i], ctr[4 * i + 1], ctr[4 * i + 2], ctr[4 * i + 3]};
  philox4x32_10(c, ks);
  out[4 * i] = c[0];
  out[4 * i + 1] = c[1];
  out[4 * i + 2] = c[2];
  out[4 * i + 3] = c[3];
}

hipError_t launch_philox_words(const uint32_t* ctr, uint32_t k0, uint32_t k1, uint32_t* out, int64_t count,
                               hipStream_t st) {
  if (count == 0) return hipSuccess;
  const PhiloxKeySchedule ks = philox_key_schedule((uint64_t)k0 | ((uint64_t)k1 << 32));
  hipLaunchKernelGGL(philox_words_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, ctr, ks, out,
                     count);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void gauss_parts_kernel(uint32_t first, int64_t count, float* __restrict__ radius,
                                                          float* __restrict__ cosv, float* __restrict__ sinv) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  const uint32_t word = (first + (uint32_t)i) << 8;
  radius[i] = gauss_radius(word);
  float c, s;
  gauss_cos_sin(word, c, s);
  cosv[i] = c;
  sinv[i] = s;
}

hipError_t launch_gauss_parts(uint32_t first, int64_t count, float* radius, float* cosv, float* sinv,
                              hipStream_t st) {
  if (count == 0) return hipSuccess;
  hipLaunchKernelGGL(gauss_parts_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, first, count,
                     radius, cosv, sinv);
  return hipGetLastError();
}

// A step's scalars into device memory (see StepState), and whether the step has to write P first.
__global__ __launch_bounds__(64) void set_step_kernel(StepState* __restrict__ ss, StepParams sp, int force_regen, int reset) {
  if (threadIdx.x != 0) return;
  if (reset) {
    ss->p_valid = 0;
    ss->p_epoch = 0;
  }
  ss->sp = sp;
  ss->regen = (force_regen || !ss->p_valid || ss->p_epoch != sp.epoch) ? 1 : 0;
}

hipError_t launch_set_step(StepState* d_state, const StepParams& sp, bool force_regen, bool reset, hipStream_t st) {
  hipLaunchKernelGGL(set_step_kernel, dim3(1), dim3(64), 0, st, d_state, sp, force_regen ? 1 : 0, reset ? 1 : 0);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4_t* __restrict__ p, size_t n16) {
  const u32x4_t z = mk_u4(0, 0, 0, 0);
  for (size_t i = (size_t)blockIdx.x * 256u + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256u) p[i] = z;
}

// bytes must be a multiple of 16 and p 16-byte aligned (the state buffer is).
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, st, reinterpret_cast<u32x4_t*>(p), n16);
  return hipGetLastError();
}

// bf16 -> fp32, element by element (debug view of a bfloat16 state).
__global__ __launch_bounds__(256) void bf16_to_f32_kernel(float* __restrict__ dst, const uint16_t* __restrict__ src, size_t count) {
  for (size_t i = (size_t)blockIdx.x * 256u + threadIdx.x; i < count; i += (size_t)gridDim.x * 256u)
    dst[i] = bf16_bits_to_f32(src[i]);
}

hipError_t launch_bf16_to_f32(float* dst, const void* src, size_t count, hipStream_t st) {
  if (count == 0) return hipSuccess;
  size_t blocks = (count + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(bf16_to_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, dst, static_cast<const uint16_t*>(src), count);
  return hipGetLastError();
}

// Plain copy of n16 16-byte words, one per thread (reference kernel of known traffic for
// calibrating hardware byte counters).
__global__ __launch_bounds__(256) void copy_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst,
                                                   size_t n16) {
  const size_t i = (size_t)blockIdx.x * 256u + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t st) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, st,
                     reinterpret_cast<const u32x4_t*>(src), reinterpret_cast<u32x4_t*>(dst), n16);
  return hipGetLastError();
}

}  // namespace apollo
