// Low-rank Adam moments + scaling factors (Algorithm 1, steps 2-3; Section 4.1, Eq. 4; Section
// 4.2), the per-tensor norm-growth limiter (Section 3.2, Eq. 3) and the scaled weight update
// (Algorithm 1, step 4).
#include <algorithm>
#include <type_traits>

#include "apollo_internal.h"
#include "state_io.hpp"

namespace apollo {

// ---------------------------------------------------------------------------------------------
// Moments and norms.  Block = 64 channel groups x 4 rank lanes; a channel group is 4 consecutive
// channels, so a wave touches 1 KB contiguous per row of R, M^R, V^R (when n is not a multiple of
// 4 the quads are only element-aligned and the last group of a row is ragged).  Thread (c, q) walks rows q, q+4, ... of its channels, accumulating
// a_j = sum R~^2 and b_j = sum R^2 in registers; the four rank lanes are combined through LDS in
// a fixed order, then the channels of the block are reduced to four block partials.  No
// atomics: results are run-to-run identical.  M^R, V^R and R are streamed (non-temporal).
// ---------------------------------------------------------------------------------------------
// RSRC: where R comes from.  0: the projection's scratch R (fp32).  1 / 2: no projection (Section 3.2,
// full-rank moments): "R" is the gradient itself, fp32 / bf16, r = m rows, and the squared channel
// norm of G is b_j; only for tensors whose rows are projected (channels = stored columns), so that
// the gradient has R's own layout.
// Row groups of a block: its 256 threads are kRG groups of kLanes threads; the groups take the rows
// kk = q, q + kRG, ... of the same kLanes * VEC channels.
constexpr int kRG = 4;
constexpr int kLanes = 256 / kRG;

// UA (with VEC = 4): n is not a multiple of 4, so a row of R, M^R, V^R starts at any element: the
// quads are accessed with element alignment only, and the last thread of a row holds 1..3 channels.
template <int VEC, bool SB16, int RSRC, bool UA = false>
__global__ __launch_bounds__(256) void adam_norms_kernel(const TensorDesc* __restrict__ descs, StepParams sp_arg, StepState* __restrict__ ss) {
  const StepParams sp = step_params(sp_arg, ss);
  static_assert(!UA || VEC == 4, "element-aligned quads");
  typedef float vec_t __attribute__((ext_vector_type(VEC)));
  __shared__ float red_a[kRG > 1 ? kRG - 1 : 1][kLanes * VEC], red_b[kRG > 1 ? kRG - 1 : 1][kLanes * VEC];
  __shared__ float blk[4][kLanes];
  const TensorView d(descs[blockIdx.y]);
  const int r = RSRC == 0 ? sp.r : d.m, n = d.n, n_slabs = RSRC == 0 ? d.n_slabs : 1;
  const int c = threadIdx.x % kLanes, q = threadIdx.x / kLanes;
  const int j0 = (blockIdx.x * kLanes + c) * VEC;
  const size_t slab_stride = (size_t)r * (size_t)n;
  const int cnt = UA ? min(VEC, n - j0) : VEC;     // channels of this thread that exist (if j0 < n)
  // VEC elements of an fp32 / moment / gradient array at element idx: one access, or the ragged end
  auto ld = [&](auto sb16, const APOLLO_GLOBAL void* base, size_t idx) -> vec_t {
    constexpr bool B = decltype(sb16)::value;
    if constexpr (UA) {
      if (cnt == VEC) return load_state<VEC, B, true>(base, idx);
      return load_state_part<B>(base, idx, cnt);
    } else {
      return load_state<VEC, B>(base, idx);
    }
  };
  auto st = [&](auto sb16, APOLLO_GLOBAL void* base, size_t idx, vec_t v) {
    constexpr bool B = decltype(sb16)::value;
    if constexpr (UA) {
      if (cnt == VEC) store_state<VEC, B, true>(base, idx, v);
      else store_state_part<B>(base, idx, v, cnt);
    } else {
      store_state<VEC, B>(base, idx, v);
    }
  };
  using f32_tag = std::integral_constant<bool, false>;
  using state_tag = std::integral_constant<bool, SB16>;
  using grad_tag = std::integral_constant<bool, RSRC == 2>;
  float a[VEC], b[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) a[e] = b[e] = 0.f;
  if (j0 < n) {
    // two rows per trip, all their loads issued before the arithmetic of either: six 16-byte
    // loads in flight per lane instead of three
    for (int kk = q; kk < r; kk += 2 * kRG) {
      const bool two = kk + kRG < r;
      const size_t idx0 = (size_t)kk * n + j0;
      const size_t idx1 = two ? idx0 + (size_t)kRG * n : idx0;
      vec_t Rv[2], mo[2], vo[2];
      if constexpr (RSRC == 0) {
        Rv[0] = ld(f32_tag{}, d.R, idx0);
        Rv[1] = ld(f32_tag{}, d.R, idx1);
      } else {
        Rv[0] = ld(grad_tag{}, d.g, idx0);
        Rv[1] = ld(grad_tag{}, d.g, idx1);
      }
      mo[0] = ld(state_tag{}, d.M, idx0);
      mo[1] = ld(state_tag{}, d.M, idx1);
      vo[0] = ld(state_tag{}, d.V, idx0);
      vo[1] = ld(state_tag{}, d.V, idx1);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        if (h == 1 && !two) break;
        const size_t idx = h ? idx1 : idx0;
        if (n_slabs > 1) {
          for (int sl = 1; sl < n_slabs; ++sl) Rv[h] += ld(f32_tag{}, d.R, sl * slab_stride + idx);
          st(f32_tag{}, d.R, idx, Rv[h]);
        }
        vec_t mn, vn;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float Re = Rv[h][e];
          float me, ve;
          const float rt = adam_element<SB16>(sp, Re, mo[h][e], vo[h][e], me, ve);
          a[e] = __builtin_fmaf(rt, rt, a[e]);
          b[e] = __builtin_fmaf(Re, Re, b[e]);
          mn[e] = me;
          vn[e] = ve;
        }
        st(state_tag{}, d.M, idx, mn);
        st(state_tag{}, d.V, idx, vn);
      }
    }
  }
  if (q > 0) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      red_a[q - 1][c * VEC + e] = a[e];
      red_b[q - 1][c * VEC + e] = b[e];
    }
  }
  __syncthreads();
  float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;
  if (q == 0 && j0 < n) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      if (UA && e >= cnt) break;
      const int j = j0 + e;
      float ae = a[e], be = b[e];
#pragma unroll
      for (int g = 0; g < kRG - 1; ++g) {      // fixed order
        ae += red_a[g][c * VEC + e];
        be += red_b[g][c * VEC + e];
      }
      float csq = RSRC == 0 ? d.colsq[j] : be;
      if (RSRC != 0) d.colsq[j] = be;
      if (n_slabs > 1) {
        for (int sl = 1; sl < n_slabs; ++sl) csq += d.colsq[(size_t)sl * n + j];
        d.colsq[j] = csq;
      }
      const float sj = (be > 0.f) ? __builtin_sqrtf(ae) / __builtin_sqrtf(be) : 0.f;
      d.s[j] = sj;                   // per-channel factor (Eq. 4); unused in tensor mode
      t0 += ae;
      t1 += be;
      t2 += csq;
      t3 += sj * sj * csq;
    }
  }
  if (q == 0) {
    blk[0][c] = t0;
    blk[1][c] = t1;
    blk[2][c] = t2;
    blk[3][c] = t3;
  }
  __syncthreads();
  // four waves: wave w reduces quantity w over the block's channel groups (fixed order: the lane's
  // strided values first, then the butterfly)
  {
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < kLanes / 64; ++i) v += blk[w][lane + 64 * i];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if (lane == 0) d.partials[(size_t)blockIdx.x * 4 + w] = v;
  }
}

// Blocks adam_norms_kernel needs for n channels (= entries of the per-block partial sums, times 4).
int adam_norms_blocks(int n) { return ((n + 3) / 4 + kLanes - 1) / kLanes; }

template <int RSRC>
static hipError_t launch_adam_norms_t(const TensorDesc* d_descs, int count, int n, bool state_bf16, const StepArgs& sa,
                                      hipStream_t st) {
  dim3 grid((unsigned)adam_norms_blocks(n), (unsigned)count, 1);
  if ((n & 3) == 0) {
    if (state_bf16) hipLaunchKernelGGL((adam_norms_kernel<4, true, RSRC>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev);
    else hipLaunchKernelGGL((adam_norms_kernel<4, false, RSRC>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev);
  } else {
    if (state_bf16) hipLaunchKernelGGL((adam_norms_kernel<4, true, RSRC, true>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev);
    else hipLaunchKernelGGL((adam_norms_kernel<4, false, RSRC, true>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev);
  }
  return hipGetLastError();
}

hipError_t launch_adam_norms(const TensorDesc* d_descs, int count, int n, bool state_bf16, const StepArgs& sa,
                             hipStream_t st) {
  return launch_adam_norms_t<0>(d_descs, count, n, state_bf16, sa, st);
}

// ---------------------------------------------------------------------------------------------
// No projection (Section 3.2, Eq. 2), channels = stored rows (a tensor with rows > cols): the
// moments have the gradient's own layout, one wave per channel walks its row of G, M and V with
// 16-byte accesses and reduces a_j = sum G~^2, b_j = sum G^2 over the lanes (butterfly, fixed
// order).  One block = four channels; it leaves the same four partial sums as adam_norms_kernel.
// ---------------------------------------------------------------------------------------------
template <bool GB16, bool SB16>
__global__ __launch_bounds__(256) void adam_identity_rows_kernel(const TensorDesc* __restrict__ descs, StepParams sp_arg, StepState* __restrict__ ss) {
  const StepParams sp = step_params(sp_arg, ss);
  __shared__ float blk[4][4];
  const TensorView d(descs[blockIdx.y]);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int m = d.m, n = d.n;
  const int j = blockIdx.x * 4 + w;
  float a = 0.f, b = 0.f;
  auto element = [&](float g, float mo, float vo, float& mn, float& vn) {
    float me, ve;
    const float rt = adam_element<SB16>(sp, g, mo, vo, me, ve);
    a = __builtin_fmaf(rt, rt, a);
    b = __builtin_fmaf(g, g, b);
    mn = me;
    vn = ve;
  };
  if (j < n) {
    const size_t base = (size_t)j * m;
    if ((m & 3) == 0) {
      typedef float vec_t __attribute__((ext_vector_type(4)));
      for (int i = lane * 4; i < m; i += 256) {
        const vec_t g = load_state<4, GB16>(d.g, base + i);
        const vec_t mo = load_state<4, SB16>(d.M, base + i);
        const vec_t vo = load_state<4, SB16>(d.V, base + i);
        vec_t mn, vn;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float me, ve;
          element(g[e], mo[e], vo[e], me, ve);
          mn[e] = me;
          vn[e] = ve;
        }
        store_state<4, SB16>(d.M, base + i, mn);
        store_state<4, SB16>(d.V, base + i, vn);
      }
    } else {
      typedef float vec_t __attribute__((ext_vector_type(1)));
      for (int i = lane; i < m; i += 64) {
        const vec_t g = load_state<1, GB16>(d.g, base + i);
        const vec_t mo = load_state<1, SB16>(d.M, base + i);
        const vec_t vo = load_state<1, SB16>(d.V, base + i);
        vec_t mn, vn;
        float me, ve;
        element(g[0], mo[0], vo[0], me, ve);
        mn[0] = me;
        vn[0] = ve;
        store_state<1, SB16>(d.M, base + i, mn);
        store_state<1, SB16>(d.V, base + i, vn);
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    a += __shfl_xor(a, off, 64);
    b += __shfl_xor(b, off, 64);
  }
  if (lane == 0) {
    float sj = 0.f;
    if (j < n) {
      sj = (b > 0.f) ? __builtin_sqrtf(a) / __builtin_sqrtf(b) : 0.f;
      d.s[j] = sj;
      d.colsq[j] = b;
    } else {
      a = b = 0.f;
    }
    blk[0][w] = a;
    blk[1][w] = b;
    blk[2][w] = b;
    blk[3][w] = sj * sj * b;
  }
  __syncthreads();
  if (threadIdx.x < 4) {
    const int q = threadIdx.x;
    d.partials[(size_t)blockIdx.x * 4 + q] = ((blk[q][0] + blk[q][1]) + blk[q][2]) + blk[q][3];
  }
}

hipError_t launch_adam_identity(const TensorDesc* d_descs, int count, int rows, int cols, bool left, bool g_bf16,
                                bool state_bf16, const StepArgs& sa, hipStream_t st) {
  if (left)
    return g_bf16 ? launch_adam_norms_t<2>(d_descs, count, cols, state_bf16, sa, st)
                  : launch_adam_norms_t<1>(d_descs, count, cols, state_bf16, sa, st);
  dim3 grid((unsigned)((rows + 3) / 4), (unsigned)count, 1);
  if (g_bf16) {
    if (state_bf16) hipLaunchKernelGGL((adam_identity_rows_kernel<true, true>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev);
    else hipLaunchKernelGGL((adam_identity_rows_kernel<true, false>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev);
  } else {
    if (state_bf16) hipLaunchKernelGGL((adam_identity_rows_kernel<false, true>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev);
    else hipLaunchKernelGGL((adam_identity_rows_kernel<false, false>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Per-tensor scalars: the tensor-wise factor (Section 4.2), the norm of the scaled gradient
// N = alpha sqrt(sum_j s_j^2 colsq_j) and the limiter (Eq. 3): if N > gamma N_prev the update is
// rescaled to norm gamma N_prev, which is also what is remembered (unless it is not finite).  One
// wave per tensor.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void finalize_kernel(const TensorDesc* __restrict__ descs, StepParams sp_arg, StepState* __restrict__ ss) {
  const StepParams sp = step_params(sp_arg, ss);
  const TensorView d(descs[blockIdx.x]);
  const int lane = threadIdx.x;
  float t[4] = {0.f, 0.f, 0.f, 0.f};
  for (int b = lane; b < d.k2_blocks; b += 64) {
    const f32x4_t p = reinterpret_cast<const APOLLO_GLOBAL f32x4_t*>(d.partials)[b];
    t[0] += p.x;
    t[1] += p.y;
    t[2] += p.z;
    t[3] += p.w;
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) t[k] += __shfl_xor(t[k], off, 64);
  }
  if (lane == 0) {
    float s_tensor = 0.f, sumsq;
    if (sp.tensor_mode) {
      s_tensor = (t[1] > 0.f) ? __builtin_sqrtf(t[0]) / __builtin_sqrtf(t[1]) : 0.f;
      sumsq = s_tensor * s_tensor * t[2];
    } else {
      sumsq = t[3];
    }
    float norm = sp.alpha * __builtin_sqrtf(sumsq);
    const float prev = *d.prev_norm;
    float c = 1.f;
    if (sp.gamma > 0.f && prev > 0.f && norm > sp.gamma * prev) {
      c = sp.gamma * prev / norm;
      norm = sp.gamma * prev;
    }
    // A non-finite gradient makes this step's norm non-finite; the stored norm then stays what it
    // was (a NaN there would switch the limiter off for good: every later comparison would be false).
    if (norm - norm == 0.f) *d.prev_norm = norm;
    d.scal[0] = sp.lr * sp.alpha * c * (sp.tensor_mode ? s_tensor : 1.f);
    d.scal[1] = c;
    d.scal[2] = norm;
    d.scal[3] = s_tensor;
    if (ss && blockIdx.x == 0) {        // this step's projection has run: the scratch holds this epoch's P
      ss->p_epoch = sp.epoch;
      ss->p_valid = 1;
    }
  }
}

hipError_t launch_finalize(const TensorDesc* d_descs, int count, const StepArgs& sa, hipStream_t st) {
  hipLaunchKernelGGL(finalize_kernel, dim3((unsigned)count), dim3(64), 0, st, d_descs, sa.host, sa.dev);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Update W <- W - coef * s_ch * G - lr*lambda * W with coef = lr * alpha * c (Algorithm 1, step 4).
// Pure streaming: G read once more (2 or 4 B), W read and written (8 B) per parameter.
//
// One thread = four consecutive elements of the flattened tensor: one 16-byte W load, one 8- or
// 16-byte G load, one 16-byte W store, so that every memory instruction of a wave covers one
// contiguous run; one block = 1024 consecutive elements, blocks in memory order.  W is streamed
// with non-temporal loads and stores (it is not touched again within the step).  Measured on
// MI355X this shape moves about 6.5 TB/s, against 5.0 TB/s for a row-tiled kernel with two
// 16-byte W accesses per lane.
// ---------------------------------------------------------------------------------------------
enum : int { kChanCol = 0, kChanRow = 1, kChanNone = 2 };


// Exact unsigned division by a run-time constant (Granlund & Montgomery, "Division by invariant
// integers using multiplication", 1994): q = (t + ((v - t) >> 1)) >> (l - 1), t = mulhi(m, v).
struct FastDiv {
  uint32_t mul, shift, one;   // one = 1 when the divisor is 1
};
static FastDiv make_fastdiv(uint32_t d) {
  FastDiv f{0, 0, 0};
  if (d == 1) { f.one = 1; return f; }
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;
  f.mul = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
  f.shift = l - 1;
  return f;
}
__device__ __forceinline__ uint32_t fastdiv(uint32_t v, const FastDiv& f) {
  if (f.one) return v;
  const uint32_t t = __umulhi(f.mul, v);
  return (t + ((v - t) >> 1)) >> f.shift;
}

// EPT consecutive elements (4 or 8) of a bf16 or fp32 array at element index e0 (a multiple of EPT;
// the group is naturally aligned), as floats, in 16-byte (8-byte for four bf16) accesses.
template <int EPT, bool IS_BF16, bool NT>
__device__ __forceinline__ void load_elems(const APOLLO_GLOBAL void* base, size_t e0, float (&out)[EPT]) {
  if constexpr (IS_BF16) {
    uint32_t h[EPT / 2];
    if constexpr (EPT == 8) {
      const APOLLO_GLOBAL u32x4_t* p = reinterpret_cast<const APOLLO_GLOBAL u32x4_t*>(reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(base) + e0);
      const u32x4_t v = NT ? __builtin_nontemporal_load(p) : *p;
      h[0] = v.x; h[1] = v.y; h[2] = v.z; h[3] = v.w;
    } else {
      const APOLLO_GLOBAL u32x2_t* p = reinterpret_cast<const APOLLO_GLOBAL u32x2_t*>(reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(base) + e0);
      const u32x2_t v = NT ? __builtin_nontemporal_load(p) : *p;
      h[0] = v.x; h[1] = v.y;
    }
#pragma unroll
    for (int i = 0; i < EPT / 2; ++i) {
      out[2 * i] = __uint_as_float(h[i] << 16);
      out[2 * i + 1] = __uint_as_float(h[i] & 0xFFFF0000u);
    }
  } else {
#pragma unroll
    for (int i = 0; i < EPT / 4; ++i) {
      const APOLLO_GLOBAL f32x4_t* p = reinterpret_cast<const APOLLO_GLOBAL f32x4_t*>(reinterpret_cast<const APOLLO_GLOBAL float*>(base) + e0) + i;
      const f32x4_t v = NT ? __builtin_nontemporal_load(p) : *p;
      out[4 * i] = v.x; out[4 * i + 1] = v.y; out[4 * i + 2] = v.z; out[4 * i + 3] = v.w;
    }
  }
}

// The counterpart store (non-temporal); bf16: one rounding to nearest even of each fp32 value.
template <int EPT, bool IS_BF16>
__device__ __forceinline__ void store_elems(APOLLO_GLOBAL void* base, size_t e0, const float (&v)[EPT]) {
  if constexpr (IS_BF16) {
    uint32_t h[EPT / 2];
#pragma unroll
    for (int i = 0; i < EPT / 2; ++i) h[i] = f32_to_bf16_bits(v[2 * i]) | (f32_to_bf16_bits(v[2 * i + 1]) << 16);
    if constexpr (EPT == 8)
      __builtin_nontemporal_store(mk_u4(h[0], h[1], h[2], h[3]),
                                  reinterpret_cast<APOLLO_GLOBAL u32x4_t*>(reinterpret_cast<APOLLO_GLOBAL uint16_t*>(base) + e0));
    else {
      u32x2_t w2 = {h[0], h[1]};
      __builtin_nontemporal_store(w2, reinterpret_cast<APOLLO_GLOBAL u32x2_t*>(reinterpret_cast<APOLLO_GLOBAL uint16_t*>(base) + e0));
    }
  } else {
#pragma unroll
    for (int i = 0; i < EPT / 4; ++i)
      __builtin_nontemporal_store(mk_f4(v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]),
                                  reinterpret_cast<APOLLO_GLOBAL f32x4_t*>(reinterpret_cast<APOLLO_GLOBAL float*>(base) + e0) + i);
  }
}

// One thread = EPT consecutive elements (4; 8 when both W and G are bfloat16, so that every access
// is still 16 bytes per lane).  ALIGNED: cols % EPT == 0, so a group never straddles a row and the
// tensor has no ragged tail.
template <bool BF16, int CHAN, bool ALIGNED, bool WB16, int EPT>
__device__ __forceinline__ void update_body(const TensorDesc& desc, const StepParams& sp, const FastDiv& div_cols, uint32_t block) {
  const TensorView d(desc);
  const uint32_t cols = (uint32_t)d.cols;
  const size_t total = (size_t)d.rows * (size_t)d.cols;
  const size_t e0 = ((size_t)block * 256u + threadIdx.x) * (size_t)EPT;
  if (e0 >= total) return;
  const float coef = d.scal[0];
  const float decay = sp.lr_decay;
  float k[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) k[e] = coef;
  if (CHAN != kChanNone) {
    uint32_t row = fastdiv((uint32_t)e0, div_cols);
    uint32_t col = (uint32_t)e0 - row * cols;
    if (ALIGNED) {
      if (CHAN == kChanCol) {
        float sv[EPT];
        load_elems<EPT, false, false>(d.s, col, sv);
#pragma unroll
        for (int e = 0; e < EPT; ++e) k[e] *= sv[e];
      } else {
        const float sr = d.s[row];
#pragma unroll
        for (int e = 0; e < EPT; ++e) k[e] *= sr;
      }
    } else if (col + EPT <= cols && e0 + EPT <= total) {
      // the thread's elements lie in one row (all but the threads at a row's end): their factors are
      // consecutive, one element-aligned vector load, or one factor for all
      if (CHAN == kChanCol) {
        typedef float f32x4_ua_t __attribute__((ext_vector_type(4), aligned(4)));
#pragma unroll
        for (int i = 0; i < EPT / 4; ++i) {
          const f32x4_ua_t sv = *reinterpret_cast<const APOLLO_GLOBAL f32x4_ua_t*>(d.s + col + 4 * i);
          k[4 * i] *= sv.x; k[4 * i + 1] *= sv.y; k[4 * i + 2] *= sv.z; k[4 * i + 3] *= sv.w;
        }
      } else {
        const float sr = d.s[row];
#pragma unroll
        for (int e = 0; e < EPT; ++e) k[e] *= sr;
      }
    } else {
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        if (e0 + e < total) k[e] *= d.s[CHAN == kChanCol ? col : row];
        if (++col == cols) { col = 0; ++row; }
      }
    }
  }
  if (ALIGNED || e0 + EPT <= total) {
    float g[EPT], w[EPT];
    load_elems<EPT, BF16, false>(d.g, e0, g);
    load_elems<EPT, WB16, true>(d.w, e0, w);
#pragma unroll
    for (int e = 0; e < EPT; ++e) w[e] = w[e] - __builtin_fmaf(k[e], g[e], decay * w[e]);
    store_elems<EPT, WB16>(d.w, e0, w);
  } else {
    for (int e = 0; e < EPT && e0 + e < total; ++e) {     // ragged tail of an unaligned tensor
      const float g = BF16 ? bf16_bits_to_f32(reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(d.g)[e0 + e])
                           : reinterpret_cast<const APOLLO_GLOBAL float*>(d.g)[e0 + e];
      if (WB16) {
        APOLLO_GLOBAL uint16_t* wp = reinterpret_cast<APOLLO_GLOBAL uint16_t*>(d.w) + e0 + e;
        const float w = bf16_bits_to_f32(*wp);
        *wp = (uint16_t)f32_to_bf16_bits(w - __builtin_fmaf(k[e], g, decay * w));
      } else {
        APOLLO_GLOBAL float* wp = reinterpret_cast<APOLLO_GLOBAL float*>(d.w) + e0 + e;
        const float w = *wp;
        *wp = w - __builtin_fmaf(k[e], g, decay * w);
      }
    }
  }
}

template <bool BF16, int CHAN, bool ALIGNED, bool WB16, int EPT>
__global__ __launch_bounds__(256) void update_kernel(const TensorDesc* __restrict__ descs, StepParams sp_arg, StepState* __restrict__ ss,
                                                     FastDiv div_cols) {
  const StepParams sp = step_params(sp_arg, ss);
  update_body<BF16, CHAN, ALIGNED, WB16, EPT>(descs[blockIdx.y], sp, div_cols, blockIdx.x);
}

// The same update for several shape groups in one launch (a small parameter set is bound by launch
// latency and by launches that do not fill the chip): the blocks of the groups follow each other in a
// one-dimensional grid, a block finds its group in the table, its tensor and its place in it.
constexpr int kMaxUpdateGroups = 8;
struct UpdateGroup {
  int first, count;               // descriptors descs[first .. first + count)
  uint32_t blocks_per_tensor;
  uint32_t blocks_end;            // one past the group's last block
  int chan, aligned;              // kChan*, cols % EPT == 0
  FastDiv div_cols;
};
struct UpdateGroups {
  UpdateGroup g[kMaxUpdateGroups];
  int n;
};

template <bool BF16, bool WB16, int EPT>
__global__ __launch_bounds__(256) void update_groups_kernel(const TensorDesc* __restrict__ descs, StepParams sp_arg,
                                                            StepState* __restrict__ ss, UpdateGroups tbl) {
  const StepParams sp = step_params(sp_arg, ss);
  const uint32_t b = blockIdx.x;
  UpdateGroup g = tbl.g[0];
  uint32_t begin = 0;
#pragma unroll
  for (int i = 1; i < kMaxUpdateGroups; ++i)
    if (i < tbl.n && b >= tbl.g[i - 1].blocks_end) {
      g = tbl.g[i];
      begin = tbl.g[i - 1].blocks_end;
    }
  const uint32_t local = b - begin;
  const uint32_t tensor = local / g.blocks_per_tensor, block = local - tensor * g.blocks_per_tensor;
  const TensorDesc& d = descs[g.first + tensor];
#define APOLLO_UPDATE_CASE(C, A) update_body<BF16, C, A, WB16, EPT>(d, sp, g.div_cols, block)
  if (g.chan == kChanCol) { if (g.aligned) APOLLO_UPDATE_CASE(kChanCol, true); else APOLLO_UPDATE_CASE(kChanCol, false); }
  else if (g.chan == kChanRow) { if (g.aligned) APOLLO_UPDATE_CASE(kChanRow, true); else APOLLO_UPDATE_CASE(kChanRow, false); }
  else { if (g.aligned) APOLLO_UPDATE_CASE(kChanNone, true); else APOLLO_UPDATE_CASE(kChanNone, false); }
#undef APOLLO_UPDATE_CASE
}

template <bool BF16, bool WB16>
static hipError_t launch_update_groups_t(const TensorDesc* d_descs, const UpdateGroupShape* groups, int n_groups,
                                         const StepArgs& sa, hipStream_t st) {
  // one element count per thread for the whole launch: 8 only if every group allows it
  int ept = (BF16 && WB16) ? 8 : 4;
  for (int i = 0; i < n_groups; ++i)
    if ((groups[i].cols & 7) != 0) ept = 4;
  for (int g0 = 0; g0 < n_groups; g0 += kMaxUpdateGroups) {
    UpdateGroups tbl{};
    tbl.n = std::min(kMaxUpdateGroups, n_groups - g0);
    uint64_t blocks = 0;
    for (int i = 0; i < tbl.n; ++i) {
      const UpdateGroupShape& g = groups[g0 + i];
      const size_t total = (size_t)g.rows * g.cols;
      const uint32_t bpt = (uint32_t)(((total + ept - 1) / ept + 255) / 256);
      blocks += (uint64_t)bpt * g.count;
      if (blocks >= (1ull << 31)) return hipErrorInvalidValue;
      tbl.g[i] = UpdateGroup{g.first, g.count, bpt, (uint32_t)blocks,
                             sa.host.tensor_mode ? kChanNone : (g.left ? kChanCol : kChanRow), (g.cols % ept) == 0 ? 1 : 0,
                             make_fastdiv((uint32_t)g.cols)};
    }
    if (ept == 8) {
      if constexpr (BF16 && WB16)
        hipLaunchKernelGGL((update_groups_kernel<BF16, WB16, 8>), dim3((unsigned)blocks), dim3(256), 0, st, d_descs, sa.host, sa.dev, tbl);
    } else {
      hipLaunchKernelGGL((update_groups_kernel<BF16, WB16, 4>), dim3((unsigned)blocks), dim3(256), 0, st, d_descs, sa.host, sa.dev, tbl);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_update_groups(const TensorDesc* d_descs, const UpdateGroupShape* groups, int n_groups, bool bf16, bool w_bf16,
                                const StepArgs& sa, hipStream_t st) {
  if (bf16) return w_bf16 ? launch_update_groups_t<true, true>(d_descs, groups, n_groups, sa, st)
                          : launch_update_groups_t<true, false>(d_descs, groups, n_groups, sa, st);
  return w_bf16 ? launch_update_groups_t<false, true>(d_descs, groups, n_groups, sa, st)
                : launch_update_groups_t<false, false>(d_descs, groups, n_groups, sa, st);
}

template <bool BF16, int CHAN, bool WB16>
static hipError_t launch_update_t(const TensorDesc* d_descs, int count, int rows, int cols, const StepArgs& sa,
                                  hipStream_t st) {
  const FastDiv fd = make_fastdiv((uint32_t)cols);
  const size_t total = (size_t)rows * cols;
  if constexpr (BF16 && WB16) {
    if ((cols & 7) == 0) {
      dim3 grid((unsigned)((total / 8 + 255) / 256), (unsigned)count, 1);
      hipLaunchKernelGGL((update_kernel<BF16, CHAN, true, WB16, 8>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev, fd);
      return hipGetLastError();
    }
  }
  const size_t quads = (total + 3) / 4;
  dim3 grid((unsigned)((quads + 255) / 256), (unsigned)count, 1);
  if ((cols & 3) == 0)
    hipLaunchKernelGGL((update_kernel<BF16, CHAN, true, WB16, 4>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev, fd);
  else
    hipLaunchKernelGGL((update_kernel<BF16, CHAN, false, WB16, 4>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev, fd);
  return hipGetLastError();
}

template <bool BF16, bool WB16>
static hipError_t launch_update_c(const TensorDesc* d_descs, int count, int rows, int cols, int chan,
                                  const StepArgs& sa, hipStream_t st) {
  if (chan == kChanCol) return launch_update_t<BF16, kChanCol, WB16>(d_descs, count, rows, cols, sa, st);
  if (chan == kChanRow) return launch_update_t<BF16, kChanRow, WB16>(d_descs, count, rows, cols, sa, st);
  return launch_update_t<BF16, kChanNone, WB16>(d_descs, count, rows, cols, sa, st);
}

hipError_t launch_update(const TensorDesc* d_descs, int count, int rows, int cols, bool left, bool bf16,
                         bool w_bf16, const StepArgs& sa, hipStream_t st) {
  const int chan = sa.host.tensor_mode ? kChanNone : (left ? kChanCol : kChanRow);
  if (bf16) {
    return w_bf16 ? launch_update_c<true, true>(d_descs, count, rows, cols, chan, sa, st)
                  : launch_update_c<true, false>(d_descs, count, rows, cols, chan, sa, st);
  }
  return w_bf16 ? launch_update_c<false, true>(d_descs, count, rows, cols, chan, sa, st)
                : launch_update_c<false, false>(d_descs, count, rows, cols, chan, sa, st);
}

// ---------------------------------------------------------------------------------------------
// Update of group-wise 8-bit weights (the format and the rounding stream are stated in
// include/apollo.h): de-quantise, W <- W - coef * s_ch * G - lr*lambda * W in fp32, quantise every
// group of 128 elements again from its new range.  One thread = 8 consecutive elements (8 bytes
// of codes, 16 bytes of a bf16 gradient), so a group is 16 consecutive lanes: its minimum and
// maximum come from four butterfly steps within those lanes, and one Philox call per thread
// yields the eight 16-bit rounding offsets.  cols is a multiple of 128: a group never straddles a
// row, and a 16-lane group is either whole or absent at the end of the tensor.
// ---------------------------------------------------------------------------------------------
// min (MAX = false) or max over each aligned run of 16 lanes, in every lane of the run, by DPP lane
// permutations: swap within pairs, swap the pairs of a quad, mirror each half of the row, mirror the
// row.  A lane whose partner is inactive keeps its own value.
template <bool MAX>
__device__ __forceinline__ float row16_reduce(float v) {
#define APOLLO_ROW_STEP(ctrl)                                                                              \
  {                                                                                                        \
    const int self = __builtin_bit_cast(int, v);                                                           \
    const float o = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(self, self, ctrl, 0xF, 0xF, false)); \
    v = MAX ? fmaxf(v, o) : fminf(v, o);                                                                   \
  }
  APOLLO_ROW_STEP(0xB1)    // quad_perm [1,0,3,2]
  APOLLO_ROW_STEP(0x4E)    // quad_perm [2,3,0,1]
  APOLLO_ROW_STEP(0x141)   // row_half_mirror
  APOLLO_ROW_STEP(0x140)   // row_mirror
#undef APOLLO_ROW_STEP
  return v;
}

template <bool BF16, int CHAN>
__global__ __launch_bounds__(256) void update_q8_kernel(const TensorDesc* __restrict__ descs, StepParams sp_arg, StepState* __restrict__ ss,
                                                        FastDiv div_cols) {
  const StepParams sp = step_params(sp_arg, ss);
  const TensorView d(descs[blockIdx.y]);
  const uint32_t cols = (uint32_t)d.cols;
  const size_t total = (size_t)d.rows * (size_t)d.cols;
  const size_t oct = (size_t)blockIdx.x * 256u + threadIdx.x;
  const size_t e0 = oct * 8u;
  if (e0 >= total) return;
  const float coef = d.scal[0];
  const float decay = sp.lr_decay;
  float k[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) k[e] = coef;
  if (CHAN != kChanNone) {
    const uint32_t row = fastdiv((uint32_t)e0, div_cols);
    const uint32_t col = (uint32_t)e0 - row * cols;
    if (CHAN == kChanCol) {
      float sv[8];
      load_elems<8, false, false>(d.s, col, sv);
#pragma unroll
      for (int e = 0; e < 8; ++e) k[e] *= sv[e];
    } else {
      const float sr = d.s[row];
#pragma unroll
      for (int e = 0; e < 8; ++e) k[e] *= sr;
    }
  }
  float g[8];
  load_elems<8, BF16, false>(d.g, e0, g);
  const u32x2_t codes = __builtin_nontemporal_load(reinterpret_cast<const APOLLO_GLOBAL u32x2_t*>(d.w) + oct);
  const size_t group = e0 >> 7;
  // w' = w (1 - lr lambda) - k g with w = zero + scale q: the decay goes into the group's pair once
  const float keep = 1.f - decay;
  const float scale = d.w_meta[2 * group] * keep, zero = d.w_meta[2 * group + 1] * keep;
  float w[8];
  float lo = 3.4e38f, hi = -3.4e38f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t q = ((e < 4 ? codes.x : codes.y) >> (8 * (e & 3))) & 0xFFu;
    w[e] = __builtin_fmaf(-k[e], g[e], __builtin_fmaf(scale, (float)q, zero));
    lo = fminf(lo, w[e]);
    hi = fmaxf(hi, w[e]);
  }
  // a group is the 16 lanes of one DPP row: butterfly by lane permutations within the row (pairs,
  // quads, mirrored halves, mirrored row); every lane ends with the group's min and max
  lo = row16_reduce<false>(lo);
  hi = row16_reduce<true>(hi);
  const float range = hi - lo;
  const float inv = range > 0.f ? 255.f * __builtin_amdgcn_rcpf(range) : 0.f;
  float u[8];
  if (sp.q8_stochastic) {
    uint32_t c[4] = {(uint32_t)oct, sp.step_lo, 0x80000000u | (uint32_t)d.tensor_id, (uint32_t)(oct >> 32)};
    philox4x32_10(c, sp.ks);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      u[2 * kk] = (float)(c[kk] & 0xFFFFu) * (1.f / 65536.f);
      u[2 * kk + 1] = (float)(c[kk] >> 16) * (1.f / 65536.f);
    }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) u[e] = 0.5f;
  }
  uint32_t out[2] = {0u, 0u};
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    // floor(x + u), then the conversion that saturates to 0..255 and places the byte (its own
    // rounding, to nearest, has nothing left to round)
    const float y = __builtin_floorf(__builtin_fmaf(w[e] - lo, inv, u[e]));
    out[e >> 2] = __builtin_amdgcn_cvt_pk_u8_f32(y, e & 3, out[e >> 2]);
  }
  u32x2_t packed = {out[0], out[1]};
  __builtin_nontemporal_store(packed, reinterpret_cast<APOLLO_GLOBAL u32x2_t*>(d.w) + oct);
  if ((threadIdx.x & 15) == 0) {
    d.w_meta[2 * group] = range * (1.f / 255.f);
    d.w_meta[2 * group + 1] = lo;
  }
}

template <bool BF16>
static hipError_t launch_update_q8_t(const TensorDesc* d_descs, int count, int rows, int cols, int chan,
                                     const StepArgs& sa, hipStream_t st) {
  const FastDiv fd = make_fastdiv((uint32_t)cols);
  const size_t octs = (size_t)rows * cols / 8;
  dim3 grid((unsigned)((octs + 255) / 256), (unsigned)count, 1);
  if (chan == kChanCol) hipLaunchKernelGGL((update_q8_kernel<BF16, kChanCol>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev, fd);
  else if (chan == kChanRow) hipLaunchKernelGGL((update_q8_kernel<BF16, kChanRow>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev, fd);
  else hipLaunchKernelGGL((update_q8_kernel<BF16, kChanNone>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev, fd);
  return hipGetLastError();
}

// cols must be a multiple of 128 (checked when the handle is created).
hipError_t launch_update_q8(const TensorDesc* d_descs, int count, int rows, int cols, bool left, bool bf16,
                            const StepArgs& sa, hipStream_t st) {
  const int chan = sa.host.tensor_mode ? kChanNone : (left ? kChanCol : kChanRow);
  return bf16 ? launch_update_q8_t<true>(d_descs, count, rows, cols, chan, sa, st)
              : launch_update_q8_t<false>(d_descs, count, rows, cols, chan, sa, st);
}

}  // namespace apollo
