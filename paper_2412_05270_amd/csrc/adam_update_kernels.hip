// Low-rank Adam moments + scaling factors (Algorithm 1, steps 2-3; Section 4.1, Eq. 4; Section
// 4.2), the per-tensor norm-growth limiter (Section 3.2, Eq. 3) and the scaled weight update
// (Algorithm 1, step 4).
#include "apollo_internal.h"

namespace apollo {

// ---------------------------------------------------------------------------------------------
// Moments and norms.  Block = 64 channels x 4 rank lanes: thread (c, q) walks rows q, q+4, ...
// of column j of R, M^R, V^R (coalesced along j), accumulating a_j = sum R~^2 and b_j = sum R^2
// in registers; the four lanes are combined through LDS in a fixed order, then the 64 channels
// of the block are reduced to four block partials.  No atomics: results are run-to-run
// identical.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void adam_norms_kernel(const TensorDesc* __restrict__ descs, StepParams sp) {
  __shared__ float red_a[3][64], red_b[3][64];
  __shared__ float blk[4][64];
  const TensorDesc& d = descs[blockIdx.y];
  const int r = sp.r, n = d.n, n_slabs = d.n_slabs;
  const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + c;
  const size_t slab_stride = (size_t)r * (size_t)n;
  float a = 0.f, b = 0.f;
  if (j < n) {
    for (int kk = q; kk < r; kk += 4) {
      const size_t idx = (size_t)kk * n + j;
      float Rv = d.R[idx];
      if (n_slabs > 1) {
        for (int sl = 1; sl < n_slabs; ++sl) Rv += d.R[sl * slab_stride + idx];
        d.R[idx] = Rv;
      }
      const float mo = d.M[idx], vo = d.V[idx];
      const float mn = __builtin_fmaf(sp.beta1, mo, sp.omb1 * Rv);
      const float vn = __builtin_fmaf(sp.beta2, vo, sp.omb2 * (Rv * Rv));
      d.M[idx] = mn;
      d.V[idx] = vn;
      const float rt = (mn * sp.inv_bc1) / (__builtin_sqrtf(vn * sp.inv_bc2) + sp.eps);
      a = __builtin_fmaf(rt, rt, a);
      b = __builtin_fmaf(Rv, Rv, b);
    }
  }
  if (q > 0) {
    red_a[q - 1][c] = a;
    red_b[q - 1][c] = b;
  }
  __syncthreads();
  float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;
  if (q == 0 && j < n) {
    a = ((a + red_a[0][c]) + red_a[1][c]) + red_a[2][c];
    b = ((b + red_b[0][c]) + red_b[1][c]) + red_b[2][c];
    float csq = d.colsq[j];
    if (n_slabs > 1) {
      for (int sl = 1; sl < n_slabs; ++sl) csq += d.colsq[(size_t)sl * n + j];
      d.colsq[j] = csq;
    }
    const float sj = (b > 0.f) ? __builtin_sqrtf(a) / __builtin_sqrtf(b) : 0.f;
    d.s[j] = sj;                     // per-channel factor (Eq. 4); unused in tensor mode
    t0 = a;
    t1 = b;
    t2 = csq;
    t3 = sj * sj * csq;
  }
  if (q == 0) {
    blk[0][c] = t0;
    blk[1][c] = t1;
    blk[2][c] = t2;
    blk[3][c] = t3;
  }
  __syncthreads();
  // four waves: wave w reduces quantity w over the 64 channels (fixed butterfly order)
  {
    float v = blk[q][c];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if (c == 0) d.partials[(size_t)blockIdx.x * 4 + q] = v;
  }
}

hipError_t launch_adam_norms(const TensorDesc* d_descs, int count, int n, const StepParams& sp, hipStream_t st) {
  dim3 grid((unsigned)((n + 63) / 64), (unsigned)count, 1);
  hipLaunchKernelGGL(adam_norms_kernel, grid, dim3(256), 0, st, d_descs, sp);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Per-tensor scalars: the tensor-wise factor (Section 4.2), the norm of the scaled gradient
// N = alpha sqrt(sum_j s_j^2 colsq_j) and the limiter (Eq. 3): if N > gamma N_prev the update is
// rescaled to norm gamma N_prev, which is also what is remembered.  One wave per tensor.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void finalize_kernel(const TensorDesc* __restrict__ descs, StepParams sp) {
  const TensorDesc& d = descs[blockIdx.x];
  const int lane = threadIdx.x;
  float t[4] = {0.f, 0.f, 0.f, 0.f};
  for (int b = lane; b < d.k2_blocks; b += 64) {
    const float4 p = reinterpret_cast<const float4*>(d.partials)[b];
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
    *d.prev_norm = norm;
    d.scal[0] = sp.lr * sp.alpha * c * (sp.tensor_mode ? s_tensor : 1.f);
    d.scal[1] = c;
    d.scal[2] = norm;
    d.scal[3] = s_tensor;
  }
}

hipError_t launch_finalize(const TensorDesc* d_descs, int count, const StepParams& sp, hipStream_t st) {
  hipLaunchKernelGGL(finalize_kernel, dim3((unsigned)count), dim3(64), 0, st, d_descs, sp);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Update W <- W - coef * s_ch * G - lr*lambda * W with coef = lr * alpha * c (Algorithm 1, step 4).
// Pure streaming: G read once more (2 or 4 B), W read and written (8 B) per parameter.
// ---------------------------------------------------------------------------------------------
enum : int { kChanCol = 0, kChanRow = 1, kChanNone = 2 };

__device__ __forceinline__ void unpack8u(const uint4& v, float f[8]) {
  f[0] = __uint_as_float(v.x << 16);
  f[1] = __uint_as_float(v.x & 0xFFFF0000u);
  f[2] = __uint_as_float(v.y << 16);
  f[3] = __uint_as_float(v.y & 0xFFFF0000u);
  f[4] = __uint_as_float(v.z << 16);
  f[5] = __uint_as_float(v.z & 0xFFFF0000u);
  f[6] = __uint_as_float(v.w << 16);
  f[7] = __uint_as_float(v.w & 0xFFFF0000u);
}

// Tiled path (cols % 8 == 0): block = 64 column octets x 4 row lanes over a 512-column x
// kUpdRows-row tile; a thread keeps the factors of its eight columns in registers.
constexpr int kUpdRows = 32;

template <bool BF16, int CHAN>
__global__ __launch_bounds__(256) void update_tiled_kernel(const TensorDesc* __restrict__ descs, StepParams sp) {
  const TensorDesc& d = descs[blockIdx.z];
  const int rows = d.rows, cols = d.cols;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int cv = blockIdx.x * 64 + tx;
  if (cv * 8 >= cols) return;
  const float coef = d.scal[0];
  const float decay = sp.lr_decay;
  float cs[8];
  if (CHAN == kChanCol) {
    const float4 s0 = reinterpret_cast<const float4*>(d.s)[2 * cv];
    const float4 s1 = reinterpret_cast<const float4*>(d.s)[2 * cv + 1];
    cs[0] = coef * s0.x; cs[1] = coef * s0.y; cs[2] = coef * s0.z; cs[3] = coef * s0.w;
    cs[4] = coef * s1.x; cs[5] = coef * s1.y; cs[6] = coef * s1.z; cs[7] = coef * s1.w;
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) cs[e] = coef;
  }
  const int row0 = blockIdx.y * kUpdRows + ty;
  const size_t nv = (size_t)(cols >> 3);
#pragma unroll
  for (int it = 0; it < kUpdRows / 4; it += 4) {
    float g[4][8];
    float4 wa[4], wb[4];
    float rs[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int row = row0 + 4 * (it + u);
      if (row < rows) {
        const size_t vi = (size_t)row * nv + cv;
        if (BF16) {
          const uint4 gv = reinterpret_cast<const uint4*>(d.g)[vi];
          unpack8u(gv, g[u]);
        } else {
          const float4 g0 = reinterpret_cast<const float4*>(d.g)[2 * vi];
          const float4 g1 = reinterpret_cast<const float4*>(d.g)[2 * vi + 1];
          g[u][0] = g0.x; g[u][1] = g0.y; g[u][2] = g0.z; g[u][3] = g0.w;
          g[u][4] = g1.x; g[u][5] = g1.y; g[u][6] = g1.z; g[u][7] = g1.w;
        }
        wa[u] = reinterpret_cast<const float4*>(d.w)[2 * vi];
        wb[u] = reinterpret_cast<const float4*>(d.w)[2 * vi + 1];
        rs[u] = (CHAN == kChanRow) ? d.s[row] : 1.f;
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int row = row0 + 4 * (it + u);
      if (row < rows) {
        const size_t vi = (size_t)row * nv + cv;
        float w[8] = {wa[u].x, wa[u].y, wa[u].z, wa[u].w, wb[u].x, wb[u].y, wb[u].z, wb[u].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float k = (CHAN == kChanRow) ? cs[e] * rs[u] : cs[e];
          w[e] = w[e] - __builtin_fmaf(k, g[u][e], decay * w[e]);
        }
        reinterpret_cast<float4*>(d.w)[2 * vi] = make_float4(w[0], w[1], w[2], w[3]);
        reinterpret_cast<float4*>(d.w)[2 * vi + 1] = make_float4(w[4], w[5], w[6], w[7]);
      }
    }
  }
}

// General path (any cols): one thread per element.
template <bool BF16, int CHAN>
__global__ __launch_bounds__(256) void update_flat_kernel(const TensorDesc* __restrict__ descs, StepParams sp) {
  const TensorDesc& d = descs[blockIdx.y];
  const size_t total = (size_t)d.rows * (size_t)d.cols;
  const float coef = d.scal[0];
  const float decay = sp.lr_decay;
  for (size_t e = (size_t)blockIdx.x * 256u + threadIdx.x; e < total; e += (size_t)gridDim.x * 256u) {
    float k = coef;
    if (CHAN == kChanCol) k *= d.s[e % (size_t)d.cols];
    if (CHAN == kChanRow) k *= d.s[e / (size_t)d.cols];
    const float g = BF16 ? bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(d.g)[e])
                         : reinterpret_cast<const float*>(d.g)[e];
    const float w = d.w[e];
    d.w[e] = w - __builtin_fmaf(k, g, decay * w);
  }
}

template <bool BF16, int CHAN>
static hipError_t launch_update_t(const TensorDesc* d_descs, int count, int rows, int cols, const StepParams& sp,
                                  hipStream_t st) {
  if ((cols & 7) == 0) {
    dim3 grid((unsigned)((cols / 8 + 63) / 64), (unsigned)((rows + kUpdRows - 1) / kUpdRows), (unsigned)count);
    hipLaunchKernelGGL((update_tiled_kernel<BF16, CHAN>), grid, dim3(256), 0, st, d_descs, sp);
  } else {
    size_t blocks = ((size_t)rows * cols + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL((update_flat_kernel<BF16, CHAN>), dim3((unsigned)blocks, (unsigned)count), dim3(256), 0, st,
                       d_descs, sp);
  }
  return hipGetLastError();
}

hipError_t launch_update(const TensorDesc* d_descs, int count, int rows, int cols, bool left, bool bf16,
                         const StepParams& sp, hipStream_t st) {
  const int chan = sp.tensor_mode ? kChanNone : (left ? kChanCol : kChanRow);
  if (bf16) {
    if (chan == kChanCol) return launch_update_t<true, kChanCol>(d_descs, count, rows, cols, sp, st);
    if (chan == kChanRow) return launch_update_t<true, kChanRow>(d_descs, count, rows, cols, sp, st);
    return launch_update_t<true, kChanNone>(d_descs, count, rows, cols, sp, st);
  }
  if (chan == kChanCol) return launch_update_t<false, kChanCol>(d_descs, count, rows, cols, sp, st);
  if (chan == kChanRow) return launch_update_t<false, kChanRow>(d_descs, count, rows, cols, sp, st);
  return launch_update_t<false, kChanNone>(d_descs, count, rows, cols, sp, st);
}

}  // namespace apollo
