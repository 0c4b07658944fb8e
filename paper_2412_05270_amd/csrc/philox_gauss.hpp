// Device-side random stream of the projection matrix P (Algorithm 1: "P_t <- N_seed(0, 1/r)").
//
// P is a pure function of (seed, tensor id, refresh epoch, row, column): a Philox4x32-10 call
// (Salmon et al., SC'11) per four consecutive columns of a row, turned into four unit-variance
// Gaussians by a Box-Muller transform whose log / sin / cos are spelled out as a fixed sequence
// of IEEE binary32 operations (exact conversions, single multiplies / adds, fused multiply-adds
// with one rounding, correctly rounded sqrt).  The sequence and its constants are the
// definition of the stream, so a CPU implementation following the same sequence reproduces it
// bit for bit.  Nothing here may be contracted, reassociated or replaced by an approximate
// hardware transcendental.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace apollo {

struct PhiloxKeySchedule {
  uint32_t k0[10];
  uint32_t k1[10];
};

__host__ __device__ inline PhiloxKeySchedule philox_key_schedule(uint64_t seed) {
  PhiloxKeySchedule ks;
  uint32_t a = (uint32_t)(seed & 0xffffffffu), b = (uint32_t)(seed >> 32);
  for (int i = 0; i < 10; ++i) {
    ks.k0[i] = a;
    ks.k1[i] = b;
    a += 0x9E3779B9u;
    b += 0xBB67AE85u;
  }
  return ks;
}

// Ten Philox rounds on counter c[0..3]; the per-round keys are wave-uniform.
__device__ __forceinline__ void philox4x32_10(uint32_t c[4], const PhiloxKeySchedule& ks) {
#pragma unroll
  for (int i = 0; i < 10; ++i) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ ks.k0[i];
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ ks.k1[i];
    c[1] = (uint32_t)p1;
    c[3] = (uint32_t)p0;
    c[0] = n0;
    c[2] = n2;
  }
}

// rho = sqrt(-2 ln u1), u1 = ((xa >> 8) + 1) / 2^24 in (0, 1].
__device__ __forceinline__ float gauss_radius(uint32_t xa) {
#pragma clang fp contract(off)
  const uint32_t n1 = (xa >> 8) + 1u;                 // 1 .. 2^24, exact as float
  const float f = (float)n1;
  const uint32_t bits = __float_as_uint(f);
  const uint32_t mbits = bits & 0x7FFFFFu;
  const bool big = mbits > 0x3504F3u;                 // mantissa above sqrt(2): use mant/2
  const float mant = __uint_as_float(mbits | (big ? 0x3F000000u : 0x3F800000u));
  const int k = (int)(bits >> 23) - 127 + (big ? 1 : 0) - 24;   // u1 = mant * 2^k
  const float t = mant - 1.0f;                        // exact
  // log1p(t) ~ t + t^2 q(t) on [sqrt(1/2)-1, sqrt(2)-1]
  float q = 0x1.6fd5ap-4f;
  q = __builtin_fmaf(q, t, -0x1.2773cap-3f);
  q = __builtin_fmaf(q, t, 0x1.30cecep-3f);
  q = __builtin_fmaf(q, t, -0x1.52fb66p-3f);
  q = __builtin_fmaf(q, t, 0x1.98da68p-3f);
  q = __builtin_fmaf(q, t, -0x1.0006c4p-2f);
  q = __builtin_fmaf(q, t, 0x1.5556e6p-2f);
  q = __builtin_fmaf(q, t, -0x1.fffff4p-2f);
  const float t2 = t * t;
  const float lp = __builtin_fmaf(t2, q, t);
  const float kf = (float)k;
  const float w = __builtin_fmaf(kf, 0x1.62e4p-1f, __builtin_fmaf(kf, 0x1.7f7d1cp-20f, lp));  // ln u1 <= 0
  return __builtin_sqrtf(-2.0f * w);
}

// (cos, sin) of theta = 2 pi u2, u2 = (xb >> 8) / 2^24: nearest quarter turn kq, remainder
// (pi/4) x with x in [-1, 1) exact.
__device__ __forceinline__ void gauss_cos_sin(uint32_t xb, float& c, float& s) {
#pragma clang fp contract(off)
  const uint32_t n2 = xb >> 8;
  const uint32_t kq = (n2 + 0x200000u) >> 22;         // 0 .. 4
  const int fi = (int)n2 - (int)(kq << 22);           // -2^21 .. 2^21-1
  const float x = (float)fi * 0x1p-21f;               // exact
  const float x2 = x * x;
  float sp = -0x1.2d9bb8p-15f;
  sp = __builtin_fmaf(sp, x2, 0x1.465ec6p-9f);
  sp = __builtin_fmaf(sp, x2, -0x1.4abbbap-4f);
  sp = __builtin_fmaf(sp, x2, 0x1.921fb6p-1f);
  const float sn = sp * x;
  float cs = -0x1.4e5ed6p-12f;
  cs = __builtin_fmaf(cs, x2, 0x1.03af5cp-6f);
  cs = __builtin_fmaf(cs, x2, -0x1.3bd392p-2f);
  cs = __builtin_fmaf(cs, x2, 1.0f);
  // rotate by kq quarter turns: (c,s) = (cs,sn), (-sn,cs), (-cs,-sn), (sn,-cs)
  const bool swap = (kq & 1u) != 0u;
  const float cc = swap ? sn : cs;
  const float ss = swap ? cs : sn;
  const uint32_t csign = ((kq + 1u) & 2u) << 30;      // quadrants 1, 2: negative cosine
  const uint32_t ssign = (kq & 2u) << 30;             // quadrants 2, 3: negative sine
  c = __uint_as_float(__float_as_uint(cc) ^ csign);
  s = __uint_as_float(__float_as_uint(ss) ^ ssign);
}

__device__ __forceinline__ void gauss_pair(uint32_t xa, uint32_t xb, float& za, float& zb) {
#pragma clang fp contract(off)
  const float rho = gauss_radius(xa);
  float c, s;
  gauss_cos_sin(xb, c, s);
  za = rho * c;
  zb = rho * s;
}

// The four unit-variance Gaussians z[kk][4q .. 4q+3] of a tensor's projection, where
// idx = kk * ceil(m/4) + q indexes the Philox counter (idx_lo, epoch, tensor_id, idx_hi).
__device__ __forceinline__ void projection_quad(const PhiloxKeySchedule& ks, uint32_t epoch,
                                                uint32_t tensor_id, uint64_t idx, float z[4]) {
  uint32_t c[4] = {(uint32_t)idx, epoch, tensor_id, (uint32_t)(idx >> 32)};
  philox4x32_10(c, ks);
  gauss_pair(c[0], c[1], z[0], z[1]);
  gauss_pair(c[2], c[3], z[2], z[3]);
}

// float -> bfloat16, round to nearest even; returns the 16 bits.  A NaN stays a NaN (its upper bits,
// made quiet): the rounding increment must not carry a NaN's payload into the exponent or sign.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float v) {
  const uint32_t b = __float_as_uint(v);
  const uint32_t rounded = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
  return (b & 0x7FFFFFFFu) > 0x7F800000u ? ((b >> 16) | 0x0040u) : rounded;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

}  // namespace apollo
