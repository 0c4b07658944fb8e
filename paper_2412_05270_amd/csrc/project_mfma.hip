// Matrix-core projection R = P G for bf16 gradients (Algorithm 1, step 1), with the per-channel
// squared norms of G as a by-product (needed by the limiter of Section 3.2).
//
// D[kk][j] = sum_i z[kk][i] Gm[i][j] with v_mfma_f32_32x32x16_bf16: z (the unit-variance P, read
// from the per-step scratch in fragment-major order) is the A operand, G the B operand, fp32
// accumulation, 1/sqrt(r) applied in the epilogue.  A block of 256 threads (four waves) owns an
// RT x 256 tile of R (RT = 32, 64, 128 or 256 rows) and walks the reduced dimension in stages of
// 64 through a double-buffered LDS tile; G is read from HBM exactly once per r-tile with 16-byte
// loads.  Both operands of the matrix core want eight consecutive reduction indices per lane:
//   - columns projected (G stored channel-major, reduction index contiguous): a 16-byte load is
//     already a fragment;
//   - rows projected (reduction index strided): each thread loads an 8 x 8 block (eight rows,
//     16 bytes each), transposes it in registers with byte permutes and stores eight fragments.
//     Fragment slot c*32 + b holds channel 8*b + c, which makes the LDS stores and loads
//     conflict-free; the epilogue undoes the permutation.
#include "apollo_internal.h"

namespace apollo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kNT = 256;          // channels per block
constexpr int kKT = 64;           // reduction indices per stage
constexpr int kBKO = 4096 + 32;   // bytes between k-octets of the B tile in LDS (padding: see stores)

template <int MT, int WM>
struct MfmaCfg {
  static constexpr int RT = 32 * MT * WM;
  static constexpr int WN = 4 / WM;
  static constexpr int NTW = 8 / WN;
  static constexpr int A_BYTES = 8 * RT * 16;
  static constexpr int B_BYTES = 8 * kBKO;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int A_CHUNKS = (8 * RT) / 256;   // 16-byte chunks per thread per stage
};

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ __forceinline__ void sq_accum8(const u32x4_t& v, float sq[8]) {
  float f;
  f = bf_lo(v.x); sq[0] = __builtin_fmaf(f, f, sq[0]);
  f = bf_hi(v.x); sq[1] = __builtin_fmaf(f, f, sq[1]);
  f = bf_lo(v.y); sq[2] = __builtin_fmaf(f, f, sq[2]);
  f = bf_hi(v.y); sq[3] = __builtin_fmaf(f, f, sq[3]);
  f = bf_lo(v.z); sq[4] = __builtin_fmaf(f, f, sq[4]);
  f = bf_hi(v.z); sq[5] = __builtin_fmaf(f, f, sq[5]);
  f = bf_lo(v.w); sq[6] = __builtin_fmaf(f, f, sq[6]);
  f = bf_hi(v.w); sq[7] = __builtin_fmaf(f, f, sq[7]);
}

template <int MT, int WM, bool LEFT>
__global__ __launch_bounds__(256) void project_mfma_kernel(const TensorDesc* __restrict__ descs, StepParams sp) {
  using C = MfmaCfg<MT, WM>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const TensorView d(descs[blockIdx.z]);
  const int r = sp.r, m = d.m, n = d.n;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int n0 = blockIdx.x * kNT;
  const int rbase = blockIdx.y * C::RT;
  const bool do_sq = blockIdx.y == 0;
  const APOLLO_GLOBAL u32x4_t* __restrict__ Pg = reinterpret_cast<const APOLLO_GLOBAL u32x4_t*>(d.P);     // one u32x4_t = (octet, row)
  const APOLLO_GLOBAL uint16_t* __restrict__ G = reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(d.g);

  f32x16_t acc[MT][C::NTW];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < C::NTW; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
  float sq[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  u32x4_t areg[C::A_CHUNKS];
  u32x4_t breg[8];
  // loader coordinates
  const int br = tid >> 5, bc = tid & 31;           // LEFT: k-octet of the stage, channel octet
  const int ko_r = tid & 7, jl_r = tid >> 3;        // RIGHT: k-octet, channel (plus 32 u)
  const u32x4_t zero4 = mk_u4(0, 0, 0, 0);

  auto load_stage = [&](int s) {
#pragma unroll
    for (int u = 0; u < C::A_CHUNKS; ++u) {
      const int q = tid + 256 * u;
      const int ko = q / C::RT, row = q % C::RT;
      areg[u] = Pg[(size_t)(8 * s + ko) * r + rbase + row];
    }
    if (LEFT) {
      const int col = n0 + 8 * bc;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int row = kKT * s + 8 * br + u;
        breg[u] = (col < n) ? *reinterpret_cast<const APOLLO_GLOBAL u32x4_t*>(G + (size_t)row * n + col) : zero4;
      }
    } else {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int j = n0 + jl_r + 32 * u;
        breg[u] = (j < n) ? *reinterpret_cast<const APOLLO_GLOBAL u32x4_t*>(G + (size_t)j * m + kKT * s + 8 * ko_r) : zero4;
      }
    }
  };

  auto store_stage = [&](int buf) {
    unsigned char* A = lds + buf * C::STAGE_BYTES;
    unsigned char* B = A + C::A_BYTES;
#pragma unroll
    for (int u = 0; u < C::A_CHUNKS; ++u) *reinterpret_cast<u32x4_t*>(A + (size_t)(tid + 256 * u) * 16) = areg[u];
    if (LEFT) {
      if (do_sq) {
#pragma unroll
        for (int u = 0; u < 8; ++u) sq_accum8(breg[u], sq);
      }
      // transpose the 8 x 8 block: fragment c = column c of the block, eight k values
      const uint32_t in[8][4] = {{breg[0].x, breg[0].y, breg[0].z, breg[0].w}, {breg[1].x, breg[1].y, breg[1].z, breg[1].w},
                                 {breg[2].x, breg[2].y, breg[2].z, breg[2].w}, {breg[3].x, breg[3].y, breg[3].z, breg[3].w},
                                 {breg[4].x, breg[4].y, breg[4].z, breg[4].w}, {breg[5].x, breg[5].y, breg[5].z, breg[5].w},
                                 {breg[6].x, breg[6].y, breg[6].z, breg[6].w}, {breg[7].x, breg[7].y, breg[7].z, breg[7].w}};
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
        u32x4_t o;
        o.x = __builtin_amdgcn_perm(in[1][c >> 1], in[0][c >> 1], sel);
        o.y = __builtin_amdgcn_perm(in[3][c >> 1], in[2][c >> 1], sel);
        o.z = __builtin_amdgcn_perm(in[5][c >> 1], in[4][c >> 1], sel);
        o.w = __builtin_amdgcn_perm(in[7][c >> 1], in[6][c >> 1], sel);
        *reinterpret_cast<u32x4_t*>(B + br * kBKO + (c * 32 + bc) * 16) = o;
      }
    } else {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (do_sq) {
          float t[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          sq_accum8(breg[u], t);
          sq[u] += ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
        }
        *reinterpret_cast<u32x4_t*>(B + ko_r * kBKO + (jl_r + 32 * u) * 16) = breg[u];
      }
    }
  };

  const int stages = m / kKT;
  load_stage(0);
  store_stage(0);
  __syncthreads();
  for (int s = 0; s < stages; ++s) {
    const int buf = s & 1;
    if (s + 1 < stages) load_stage(s + 1);
    const unsigned char* A = lds + buf * C::STAGE_BYTES;
    const unsigned char* B = A + C::A_BYTES;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int oct = 2 * ks + (lane >> 5);
      bf16x8_t af[MT], bfr[C::NTW];
#pragma unroll
      for (int a = 0; a < MT; ++a)
        af[a] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(
                                                 A + (size_t)(oct * C::RT + wm * 32 * MT + a * 32 + (lane & 31)) * 16));
#pragma unroll
      for (int b = 0; b < C::NTW; ++b)
        bfr[b] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(
                                                  B + oct * kBKO + ((wn * C::NTW + b) * 32 + (lane & 31)) * 16));
#pragma unroll
      for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < C::NTW; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
    }
    if (s + 1 < stages) store_stage(buf ^ 1);
    __syncthreads();
  }

  // epilogue: R = acc / sqrt(r)
  const float scale = sp.rsqrt_r;
#pragma unroll
  for (int a = 0; a < MT; ++a) {
#pragma unroll
    for (int b = 0; b < C::NTW; ++b) {
      const int c = wn * C::NTW + b;
      const int j = LEFT ? n0 + 8 * (lane & 31) + c : n0 + 32 * c + (lane & 31);
      if (j < n) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = rbase + wm * 32 * MT + a * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
          d.R[(size_t)i * n + j] = acc[a][b][v] * scale;
        }
      }
    }
  }

  if (do_sq) {
    float* red = reinterpret_cast<float*>(lds);       // all tiles are consumed: reuse the LDS
    if (LEFT) {
      // thread (br, bc) holds partial sums of channels 8 bc .. 8 bc + 7 over its rows: add the 8 br
#pragma unroll
      for (int c = 0; c < 8; ++c) red[br * 264 + 8 * bc + c] = sq[c];
      __syncthreads();
      const int j = n0 + tid;
      if (j < n) {
        float t = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) t += red[k * 264 + tid];
        d.colsq[j] = t;
      }
    } else {
      // thread (ko, jl) holds channel jl + 32 u over its k-octets: add the 8 ko (adjacent lanes)
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        float t = sq[u];
        t += __shfl_xor(t, 1, 64);
        t += __shfl_xor(t, 2, 64);
        t += __shfl_xor(t, 4, 64);
        const int j = n0 + jl_r + 32 * u;
        if (ko_r == 0 && j < n) d.colsq[j] = t;
      }
    }
  }
}

bool project_mfma_supported(int rows, int cols, bool left, bool bf16, int r) {
  if (!bf16 || (r & 31) != 0) return false;
  const int m = left ? rows : cols;
  if ((m % kKT) != 0) return false;
  if ((cols & 7) != 0) return false;       // 16-byte gradient loads
  return true;
}

template <int MT, int WM, bool LEFT>
static hipError_t launch_cfg(const TensorDesc* d_descs, int count, int n, const StepParams& sp, hipStream_t st) {
  using C = MfmaCfg<MT, WM>;
  const int lds_bytes = 2 * C::STAGE_BYTES;
  static bool attr_done = false;
  if (!attr_done) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&project_mfma_kernel<MT, WM, LEFT>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  dim3 grid((unsigned)((n + kNT - 1) / kNT), (unsigned)(sp.r / C::RT), (unsigned)count);
  hipLaunchKernelGGL((project_mfma_kernel<MT, WM, LEFT>), grid, dim3(256), lds_bytes, st, d_descs, sp);
  return hipGetLastError();
}

template <bool LEFT>
static hipError_t launch_side(const TensorDesc* d_descs, int count, int n, const StepParams& sp, hipStream_t st) {
  const int r = sp.r;
  if (r % 256 == 0) return launch_cfg<4, 2, LEFT>(d_descs, count, n, sp, st);
  if (r % 128 == 0) return launch_cfg<4, 1, LEFT>(d_descs, count, n, sp, st);
  if (r % 64 == 0) return launch_cfg<2, 1, LEFT>(d_descs, count, n, sp, st);
  return launch_cfg<1, 1, LEFT>(d_descs, count, n, sp, st);
}

hipError_t launch_project_mfma(const TensorDesc* d_descs, int count, int rows, int cols, bool left,
                               const StepParams& sp, hipStream_t st) {
  const int n = left ? cols : rows;
  return left ? launch_side<true>(d_descs, count, n, sp, st) : launch_side<false>(d_descs, count, n, sp, st);
}

}  // namespace apollo
