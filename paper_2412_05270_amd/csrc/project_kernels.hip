// Projection kernels R = P G (Algorithm 1, step 1) with the by-product colsq_j = sum_i G[i,j]^2
// (needed by the norm-growth limiter, Section 3.2): a general fp32-FMA kernel for any rank,
// dtype and orientation, and a streaming kernel for rank 1 (APOLLO-Mini, Section 4.2) that
// generates its row of P on the fly.
#include "apollo_internal.h"

namespace apollo {

__device__ __forceinline__ float load_g(const APOLLO_GLOBAL void* g, size_t idx, bool bf16) {
  if (bf16) return bf16_bits_to_f32(reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(g)[idx]);
  return reinterpret_cast<const APOLLO_GLOBAL float*>(g)[idx];
}

// ---------------------------------------------------------------------------------------------
// General projection: block = 64 channels x 32 rows of R, looping over the reduced dimension in
// steps of 32 through LDS.  P comes from the scratch copy written by fill_projection_kernel.
// Gm(i, j) is G[i][j] when the rows are projected (left) and G[j][i] otherwise.
// ---------------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void project_generic_kernel(const TensorDesc* __restrict__ descs, StepParams sp_arg, StepState* __restrict__ ss) {
  const StepParams sp = step_params(sp_arg, ss);
  __shared__ float Gs[32][65];
  __shared__ float Ps[32][33];
  const TensorView d(descs[blockIdx.z]);
  const int r = sp.r, m = d.m, n = d.n, cols = d.cols;
  const int tid = threadIdx.x;
  const int j0 = blockIdx.x * 64, kk0 = blockIdx.y * 32;
  const int tx = tid & 15, ty = tid >> 4;
  float acc[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  float sq = 0.f;
  for (int i0 = 0; i0 < m; i0 += 32) {
    if (d.left) {
      const int jj = tid & 63;
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const int ii = (tid >> 6) + 4 * p;
        const int i = i0 + ii, j = j0 + jj;
        Gs[ii][jj] = (i < m && j < n) ? load_g(d.g, (size_t)i * cols + j, BF16) : 0.f;
      }
    } else {
      const int ii = tid & 31;
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const int jj = (tid >> 5) + 8 * p;
        const int i = i0 + ii, j = j0 + jj;
        Gs[ii][jj] = (i < m && j < n) ? load_g(d.g, (size_t)j * cols + i, BF16) : 0.f;
      }
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int e = tid + 256 * p;
      const int i8 = e & 7, kk = (e >> 3) & 31, io = e >> 8;
      const int ii = io * 8 + i8;
      const int i = i0 + ii, k = kk0 + kk;
      float v = 0.f;
      if (k < r && i < d.m8) {
        const size_t idx = p_index(k, i, r);
        v = BF16 ? bf16_bits_to_f32(reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(d.P)[idx])
                 : reinterpret_cast<const APOLLO_GLOBAL float*>(d.P)[idx];
      }
      Ps[kk][ii] = v;
    }
    __syncthreads();
#pragma unroll 8
    for (int ii = 0; ii < 32; ++ii) {
      const float p0 = Ps[2 * ty][ii], p1 = Ps[2 * ty + 1][ii];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float gv = Gs[ii][4 * tx + c];
        acc[0][c] = __builtin_fmaf(p0, gv, acc[0][c]);
        acc[1][c] = __builtin_fmaf(p1, gv, acc[1][c]);
      }
    }
    if (blockIdx.y == 0 && tid < 64) {
#pragma unroll 8
      for (int ii = 0; ii < 32; ++ii) sq = __builtin_fmaf(Gs[ii][tid], Gs[ii][tid], sq);
    }
    __syncthreads();
  }
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const int k = kk0 + 2 * ty + a;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int j = j0 + 4 * tx + c;
      if (k < r && j < n) d.R[(size_t)k * n + j] = acc[a][c] * sp.rsqrt_r;
    }
  }
  if (blockIdx.y == 0 && tid < 64 && j0 + tid < n) d.colsq[j0 + tid] = sq;
}

hipError_t launch_project_generic(const TensorDesc* d_descs, int count, int n, bool bf16, const StepArgs& sa,
                                  hipStream_t st) {
  dim3 grid((unsigned)((n + 63) / 64), (unsigned)((sa.host.r + 31) / 32), (unsigned)count);
  if (bf16)
    hipLaunchKernelGGL(project_generic_kernel<true>, grid, dim3(256), 0, st, d_descs, sa.host, sa.dev);
  else
    hipLaunchKernelGGL(project_generic_kernel<false>, grid, dim3(256), 0, st, d_descs, sa.host, sa.dev);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Rank 1 (APOLLO-Mini): R[j] = sum_i z[i] Gm[i, j] is a matrix-vector product, bound by the one
// pass over G.  z is generated into LDS by the block that needs it; G is read with 16-byte
// loads (eight bf16, or two loads of four fp32); a row length that is not a multiple of 8 takes the
// same loads unaligned and the ragged last octet of a row element by element.
// ---------------------------------------------------------------------------------------------

// unpack eight bf16 (one 16-byte load) to floats
__device__ __forceinline__ void unpack8(const u32x4_t& v, float f[8]) {
  f[0] = __uint_as_float(v.x << 16);
  f[1] = __uint_as_float(v.x & 0xFFFF0000u);
  f[2] = __uint_as_float(v.y << 16);
  f[3] = __uint_as_float(v.y & 0xFFFF0000u);
  f[4] = __uint_as_float(v.z << 16);
  f[5] = __uint_as_float(v.z & 0xFFFF0000u);
  f[6] = __uint_as_float(v.w << 16);
  f[7] = __uint_as_float(v.w & 0xFFFF0000u);
}

// Eight consecutive gradient elements starting at element index `elem` of a row-major array, as
// floats, streamed: one 16-byte load of bf16, or two of fp32.  elem is a multiple of 8 (the loads are
// naturally aligned) unless UA: then it is any element index, and the loads are declared aligned to
// the element type only (global memory takes unaligned vector accesses).
template <bool BF16, bool UA>
__device__ __forceinline__ void load_octet(const APOLLO_GLOBAL void* g, size_t elem, float f[8]) {
  typedef uint32_t u32x4_ua_t __attribute__((ext_vector_type(4), aligned(2)));
  typedef float f32x4_ua_t __attribute__((ext_vector_type(4), aligned(4)));
  if constexpr (BF16) {
    const APOLLO_GLOBAL uint16_t* p = reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(g) + elem;
    if constexpr (UA) {
      const u32x4_ua_t t = __builtin_nontemporal_load(reinterpret_cast<const APOLLO_GLOBAL u32x4_ua_t*>(p));
      u32x4_t v;
      v.x = t.x; v.y = t.y; v.z = t.z; v.w = t.w;
      unpack8(v, f);
    } else {
      unpack8(__builtin_nontemporal_load(reinterpret_cast<const APOLLO_GLOBAL u32x4_t*>(p)), f);
    }
  } else {
    const APOLLO_GLOBAL float* p = reinterpret_cast<const APOLLO_GLOBAL float*>(g) + elem;
    if constexpr (UA) {
      const f32x4_ua_t lo = __builtin_nontemporal_load(reinterpret_cast<const APOLLO_GLOBAL f32x4_ua_t*>(p));
      const f32x4_ua_t hi = __builtin_nontemporal_load(reinterpret_cast<const APOLLO_GLOBAL f32x4_ua_t*>(p) + 1);
      f[0] = lo.x; f[1] = lo.y; f[2] = lo.z; f[3] = lo.w;
      f[4] = hi.x; f[5] = hi.y; f[6] = hi.z; f[7] = hi.w;
    } else {
      const f32x4_t lo = __builtin_nontemporal_load(reinterpret_cast<const APOLLO_GLOBAL f32x4_t*>(p));
      const f32x4_t hi = __builtin_nontemporal_load(reinterpret_cast<const APOLLO_GLOBAL f32x4_t*>(p) + 1);
      f[0] = lo.x; f[1] = lo.y; f[2] = lo.z; f[3] = lo.w;
      f[4] = hi.x; f[5] = hi.y; f[6] = hi.z; f[7] = hi.w;
    }
  }
}

// The first cnt (1..7) of eight consecutive elements, one at a time (the ragged end of a row whose
// length is not a multiple of 8); the rest read as 0.
template <bool BF16>
__device__ __forceinline__ void load_octet_part(const APOLLO_GLOBAL void* g, size_t elem, int cnt, float f[8]) {
#pragma unroll
  for (int e = 0; e < 8; ++e) f[e] = 0.f;
#pragma unroll
  for (int e = 0; e < 7; ++e)
    if (e < cnt) f[e] = load_g(g, elem + e, BF16);
}

// Generates z[i0 .. i0+count) (count % 4 == 0 or the tail beyond m ignored) into zs[0 .. count).
__device__ __forceinline__ void gen_z_to_lds(float* zs, int i0, int count, int m, const StepParams& sp,
                                             uint32_t tensor_id, bool round_bf16) {
  const int q0 = i0 >> 2;                      // i0 is a multiple of 4
  const int nq = (count + 3) >> 2;
  for (int q = threadIdx.x; q < nq; q += blockDim.x) {
    float z[4];
    projection_quad(sp.ks, sp.epoch, tensor_id, (uint64_t)(q0 + q), z);   // row kk = 0
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int li = 4 * q + e;
      if (li < count) {
        float v = (i0 + li < m) ? z[e] : 0.f;
        if (round_bf16) v = bf16_bits_to_f32(f32_to_bf16_bits(v));
        zs[li] = v;
      }
    }
  }
}

// LEFT (rows projected): block = 512 columns x one slab of rows; thread (tx = column octet,
// ty = row lane) accumulates eight column dot products over its rows; the four row lanes are
// combined through LDS.  Output: partial R and colsq of this slab.
constexpr int kMiniSlabRowsMax = 1024;

template <bool BF16, bool UA>
__global__ __launch_bounds__(256) void project_rank1_left_kernel(const TensorDesc* __restrict__ descs, StepParams sp_arg, StepState* __restrict__ ss,
                                                                 int slab_rows) {
  const StepParams sp = step_params(sp_arg, ss);
  __shared__ float zs[kMiniSlabRowsMax];
  __shared__ float red[2][3][64][9];
  const TensorView d(descs[blockIdx.z]);
  const int rows = d.rows, cols = d.cols;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int i0 = blockIdx.y * slab_rows;
  const int i1 = min(rows, i0 + slab_rows);
  gen_z_to_lds(zs, i0, i1 - i0, rows, sp, (uint32_t)d.tensor_id, BF16);
  __syncthreads();
  const int cv = blockIdx.x * 64 + tx;          // column octet
  const bool active = cv * 8 < cols;
  // UA (a row length that is not a multiple of 8): rows start at any element, and the last octet
  // of a row has only cnt columns
  const int cnt = min(8, cols - cv * 8);
  float acc[8], sq[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = sq[e] = 0.f;
  if (active) {
    auto ld = [&](int row, float f[8]) {
      const size_t elem = (size_t)row * (size_t)cols + (size_t)cv * 8;
      if (!UA || cnt == 8) load_octet<BF16, UA>(d.g, elem, f);
      else load_octet_part<BF16>(d.g, elem, cnt, f);
    };
    int i = i0 + ty;
    for (; i + 12 < i1; i += 16) {
      float f[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) ld(i + 4 * u, f[u]);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float z = zs[i + 4 * u - i0];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          acc[e] = __builtin_fmaf(z, f[u][e], acc[e]);
          sq[e] = __builtin_fmaf(f[u][e], f[u][e], sq[e]);
        }
      }
    }
    for (; i < i1; i += 4) {
      float f[8];
      ld(i, f);
      const float z = zs[i - i0];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        acc[e] = __builtin_fmaf(z, f[e], acc[e]);
        sq[e] = __builtin_fmaf(f[e], f[e], sq[e]);
      }
    }
  }
  if (ty > 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      red[0][ty - 1][tx][e] = acc[e];
      red[1][ty - 1][tx][e] = sq[e];
    }
  }
  __syncthreads();
  if (ty == 0 && active) {
    APOLLO_GLOBAL float* Rp = d.R + (size_t)blockIdx.y * d.n + (size_t)cv * 8;
    APOLLO_GLOBAL float* Cp = d.colsq + (size_t)blockIdx.y * d.n + (size_t)cv * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float a = ((acc[e] + red[0][0][tx][e]) + red[0][1][tx][e]) + red[0][2][tx][e];
      const float b = ((sq[e] + red[1][0][tx][e]) + red[1][1][tx][e]) + red[1][2][tx][e];
      if (!UA || e < cnt) {
        Rp[e] = a;          // r = 1: 1/sqrt(r) = 1
        Cp[e] = b;
      }
    }
  }
}

// RIGHT (columns projected): R[i] = sum_j z[j] G[i][j]; a wave owns whole rows, four at a time,
// lanes stride the row in 16-byte pieces, then a wave reduction.  z for the whole row (m <= 16384)
// sits in LDS.
constexpr int kMiniRightMaxM = 16384;
constexpr int kMiniRightRowsPerBlock = 128;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

template <bool BF16, bool UA>
__global__ __launch_bounds__(256) void project_rank1_right_kernel(const TensorDesc* __restrict__ descs,
                                                                  StepParams sp_arg, StepState* __restrict__ ss) {
  const StepParams sp = step_params(sp_arg, ss);
  extern __shared__ float zs[];
  const TensorView d(descs[blockIdx.z]);
  const int rows = d.rows, cols = d.cols;
  gen_z_to_lds(zs, 0, (cols + 7) & ~7, cols, sp, (uint32_t)d.tensor_id, BF16);   // (zeros behind a ragged end)
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nv = (cols + 7) >> 3;          // octets per row; with UA the last one may have only cols % 8 elements
  const int row_begin = blockIdx.x * kMiniRightRowsPerBlock + wave * (kMiniRightRowsPerBlock / 4);
  const int row_end = min(rows, row_begin + kMiniRightRowsPerBlock / 4);
  for (int i = row_begin; i < row_end; i += 4) {
    float acc[4] = {0.f, 0.f, 0.f, 0.f}, sq[4] = {0.f, 0.f, 0.f, 0.f};
    for (int v0 = lane; v0 < nv; v0 += 64) {
      float fv[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int ii = min(i + u, rows - 1);
        const size_t elem = (size_t)ii * (size_t)cols + (size_t)v0 * 8;
        if (!UA || v0 * 8 + 8 <= cols) load_octet<BF16, UA>(d.g, elem, fv[u]);
        else load_octet_part<BF16>(d.g, elem, cols - v0 * 8, fv[u]);
      }
      const f32x4_t za = reinterpret_cast<const f32x4_t*>(zs)[2 * v0];
      const f32x4_t zb = reinterpret_cast<const f32x4_t*>(zs)[2 * v0 + 1];
      const float z[8] = {za.x, za.y, za.z, za.w, zb.x, zb.y, zb.z, zb.w};
#pragma unroll
      for (int u = 0; u < 4; ++u) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          acc[u] = __builtin_fmaf(z[e], fv[u][e], acc[u]);
          sq[u] = __builtin_fmaf(fv[u][e], fv[u][e], sq[u]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float a = wave_sum(acc[u]);
      const float b = wave_sum(sq[u]);
      if (lane == 0 && i + u < row_end) {
        d.R[i + u] = a;
        d.colsq[i + u] = b;
      }
    }
  }
}

bool project_rank1_supported(int rows, int cols, bool left, bool bf16) {
  (void)bf16;
  if (!left && cols > kMiniRightMaxM) return false;
  (void)rows;
  return true;
}

hipError_t launch_project_rank1(const TensorDesc* d_descs, int count, int rows, int cols, bool left, bool bf16,
                                int n_slabs, const StepArgs& sa, hipStream_t st) {
  const bool ua = (cols & 7) != 0;     // rows of the gradient do not start on 16-byte boundaries
  if (left) {
    const int slab_rows = (((rows + n_slabs - 1) / n_slabs) + 3) & ~3;   // multiple of 4: slabs start on a quad
    dim3 grid((unsigned)(((cols + 7) / 8 + 63) / 64), (unsigned)n_slabs, (unsigned)count);
    if (bf16 && !ua) hipLaunchKernelGGL((project_rank1_left_kernel<true, false>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev, slab_rows);
    else if (bf16) hipLaunchKernelGGL((project_rank1_left_kernel<true, true>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev, slab_rows);
    else if (!ua) hipLaunchKernelGGL((project_rank1_left_kernel<false, false>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev, slab_rows);
    else hipLaunchKernelGGL((project_rank1_left_kernel<false, true>), grid, dim3(256), 0, st, d_descs, sa.host, sa.dev, slab_rows);
  } else {
    dim3 grid((unsigned)((rows + kMiniRightRowsPerBlock - 1) / kMiniRightRowsPerBlock), 1, (unsigned)count);
    const size_t lds = (size_t)((cols + 7) & ~7) * sizeof(float);
    if (bf16 && !ua) hipLaunchKernelGGL((project_rank1_right_kernel<true, false>), grid, dim3(256), lds, st, d_descs, sa.host, sa.dev);
    else if (bf16) hipLaunchKernelGGL((project_rank1_right_kernel<true, true>), grid, dim3(256), lds, st, d_descs, sa.host, sa.dev);
    else if (!ua) hipLaunchKernelGGL((project_rank1_right_kernel<false, false>), grid, dim3(256), lds, st, d_descs, sa.host, sa.dev);
    else hipLaunchKernelGGL((project_rank1_right_kernel<false, true>), grid, dim3(256), lds, st, d_descs, sa.host, sa.dev);
  }
  return hipGetLastError();
}

}  // namespace apollo
