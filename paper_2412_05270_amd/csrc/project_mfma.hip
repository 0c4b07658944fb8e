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
//
// Software pipeline of one stage s (LDS buffer s & 1 is being multiplied), per wave:
//   start   : P(s+1) from L2 straight into the other LDS buffer (direct-to-LDS loads), global loads
//             of G(s+2) into registers (G two stages ahead: HBM latency)
//   k-step 0: fragments of k-step 1 <- LDS | 16 MFMA
//   k-step 1: fragments of k-step 2 <- LDS | 16 MFMA | G(s+1) registers -> transpose -> other LDS buffer
//   k-step 2: fragments of k-step 3 <- LDS | 16 MFMA | squared norms of G(s+1)
//   k-step 3:                              | 16 MFMA
//   barrier, fragments of k-step 0 of stage s+1 <- LDS
// so that LDS reads, the transpose and the norm arithmetic issue in the shadow of the MFMAs.
//
// Blocks are numbered so that all tiles of one tensor run on the same XCD (workgroups are dealt
// to the eight XCDs round-robin): the 2 MB of P of a tensor then stay in that XCD's L2 instead
// of being fetched from HBM once per XCD.
#include "apollo_internal.h"

namespace apollo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kNT = 256;          // channels per block
constexpr int kKT = 64;           // reduction indices per stage
constexpr int kBKO = 4096 + 32;   // bytes between k-octets of the B tile in LDS (padding: see stores)
constexpr int kXcds = 8;
#define APOLLO_LDS __attribute__((address_space(3)))

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

__device__ __forceinline__ void sq_accum8(const u32x4_t& v, float (&sq)[8]) {
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

__device__ __forceinline__ float sq_sum8(const u32x4_t& v) {
  float t0 = bf_lo(v.x) * bf_lo(v.x), t1 = bf_hi(v.x) * bf_hi(v.x);
  t0 = __builtin_fmaf(bf_lo(v.y), bf_lo(v.y), t0);
  t1 = __builtin_fmaf(bf_hi(v.y), bf_hi(v.y), t1);
  t0 = __builtin_fmaf(bf_lo(v.z), bf_lo(v.z), t0);
  t1 = __builtin_fmaf(bf_hi(v.z), bf_hi(v.z), t1);
  t0 = __builtin_fmaf(bf_lo(v.w), bf_lo(v.w), t0);
  t1 = __builtin_fmaf(bf_hi(v.w), bf_hi(v.w), t1);
  return t0 + t1;
}

// Per-thread coordinates and base pointers of the kernel, bundled so the pipeline pieces can be
// small force-inlined functions working on register arrays passed by reference.
template <int MT, int WM, bool LEFT>
struct MfmaCtx {
  using C = MfmaCfg<MT, WM>;
  const APOLLO_GLOBAL u32x4_t* Pg;   // scratch P: one 16-byte word per (octet, row)
  const APOLLO_GLOBAL uint16_t* G;
  unsigned char* lds;
  int r, m, n, n0, rbase, tid, lane, wm, wn;
  int br, bc;        // LEFT loader: k-octet of the stage, channel octet
  int ko_r, jl_r;    // RIGHT loader: k-octet, channel (plus 32 u)
  int last_stage;
  bool do_sq;

  // P tile of stage s -> LDS A buffer `buf` with direct-to-LDS loads (global_load_lds_dwordx4):
  // lane i of a wave lands at (wave-uniform LDS address in M0) + 16 i, which is the fragment
  // order already, so P never passes through registers.  Written as inline assembly because the
  // compiler would otherwise wait for each such load before issuing the next; it therefore does
  // not count them in its own vmcnt bookkeeping (which only makes its waits longer, never
  // shorter: they are issued BEFORE the G loads of the same stage, see wait_dma()).
  __device__ __forceinline__ void dma_a(int s, int buf) const {
    s = min(s, last_stage);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(APOLLO_LDS unsigned char*)(lds + buf * C::STAGE_BYTES);
#pragma unroll
    for (int u = 0; u < C::A_CHUNKS; ++u) {
      const int q = tid + 256 * u;
      const APOLLO_GLOBAL u32x4_t* src = Pg + (size_t)(8 * s + q / C::RT) * r + rbase + (q % C::RT);
      const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_base + (uint32_t)((tid & ~63) + 256 * u) * 16u);
      uint32_t saved_m0;   // M0 is restored: the compiler may hold a value of its own there
      asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                   : "=&s"(saved_m0)
                   : "s"(dst), "v"(src)
                   : "memory");
    }
  }
  // Waits until at most `newer` vector-memory operations issued after the last dma_a() are
  // outstanding, i.e. until the P tile is in LDS (vmcnt retires in issue order).
  template <int NEWER>
  __device__ __forceinline__ void wait_dma() const {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(NEWER) : "memory");
  }
  // No bounds checks: a ragged last tile is shifted left to end at channel n (see the kernel), so
  // every address is valid and the stage body stays free of branches.
  __device__ __forceinline__ void load_b(int s, u32x4_t (&bq)[8]) const {
    s = min(s, last_stage);
    if (LEFT) {
      const APOLLO_GLOBAL uint16_t* p = G + (size_t)(kKT * s + 8 * br) * n + (n0 + 8 * bc);
#pragma unroll
      for (int u = 0; u < 8; ++u) bq[u] = *reinterpret_cast<const APOLLO_GLOBAL u32x4_t*>(p + (size_t)u * n);
    } else {
      const APOLLO_GLOBAL uint16_t* p = G + (size_t)(n0 + jl_r) * m + (kKT * s + 8 * ko_r);
#pragma unroll
      for (int u = 0; u < 8; ++u) bq[u] = *reinterpret_cast<const APOLLO_GLOBAL u32x4_t*>(p + (size_t)(32 * u) * m);
    }
  }
  // registers -> fragments in LDS buffer `buf` (transposing when rows are projected)
  __device__ __forceinline__ void store_b(int buf, const u32x4_t (&bq)[8]) const {
    unsigned char* B = lds + buf * C::STAGE_BYTES + C::A_BYTES;
    if (LEFT) {
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
        u32x4_t o;
        o.x = __builtin_amdgcn_perm(bq[1][c >> 1], bq[0][c >> 1], sel);
        o.y = __builtin_amdgcn_perm(bq[3][c >> 1], bq[2][c >> 1], sel);
        o.z = __builtin_amdgcn_perm(bq[5][c >> 1], bq[4][c >> 1], sel);
        o.w = __builtin_amdgcn_perm(bq[7][c >> 1], bq[6][c >> 1], sel);
        *reinterpret_cast<u32x4_t*>(B + br * kBKO + (c * 32 + bc) * 16) = o;
      }
    } else {
#pragma unroll
      for (int u = 0; u < 8; ++u) *reinterpret_cast<u32x4_t*>(B + ko_r * kBKO + (jl_r + 32 * u) * 16) = bq[u];
    }
  }
  // every r-tile block sums the squares (branch-free stage body); only the first writes them
  __device__ __forceinline__ void accum_sq(const u32x4_t (&bq)[8], float (&sq)[8]) const {
    if (LEFT) {
#pragma unroll
      for (int u = 0; u < 8; ++u) sq_accum8(bq[u], sq);
    } else {
#pragma unroll
      for (int u = 0; u < 8; ++u) sq[u] += sq_sum8(bq[u]);
    }
  }
  __device__ __forceinline__ void read_frags(int buf, int ks, bf16x8_t (&af)[MT], bf16x8_t (&bf)[C::NTW]) const {
    const unsigned char* A = lds + buf * C::STAGE_BYTES;
    const unsigned char* B = A + C::A_BYTES;
    const int oct = 2 * ks + (lane >> 5);
#pragma unroll
    for (int a = 0; a < MT; ++a)
      af[a] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(
                                               A + (size_t)(oct * C::RT + wm * 32 * MT + a * 32 + (lane & 31)) * 16));
#pragma unroll
    for (int b = 0; b < C::NTW; ++b)
      bf[b] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(
                                               B + oct * kBKO + ((wn * C::NTW + b) * 32 + (lane & 31)) * 16));
  }
};

template <int MT, int NTW>
__device__ __forceinline__ void mfma_block(f32x16_t (&acc)[MT][NTW], const bf16x8_t (&af)[MT], const bf16x8_t (&bf)[NTW]) {
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < NTW; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
}

// Scheduling hints for one k-step region (the compiler otherwise sinks the LDS reads of the next
// k-step below the MFMAs and bunches the side work): first the fragment reads, then the MFMAs
// with the side work (VALU, LDS writes) spread between them.
//   masks of sched_group_barrier: 0x2 VALU, 0x8 MFMA, 0x100 LDS read, 0x200 LDS write
template <int READS, int MFMAS>
__device__ __forceinline__ void sched_reads_then_mfma() {
  if (READS > 0) __builtin_amdgcn_sched_group_barrier(0x100, READS, 0);
  __builtin_amdgcn_sched_group_barrier(0x008, MFMAS, 0);
}
template <int READS, int MFMAS, int VALU_PER, int WRITES_PER, int GROUPS>
__device__ __forceinline__ void sched_reads_then_mix() {
  if (READS > 0) __builtin_amdgcn_sched_group_barrier(0x100, READS, 0);
#pragma unroll
  for (int g = 0; g < GROUPS; ++g) {
    __builtin_amdgcn_sched_group_barrier(0x008, MFMAS / GROUPS, 0);
    if (VALU_PER > 0) __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, 0);
    if (WRITES_PER > 0) __builtin_amdgcn_sched_group_barrier(0x200, WRITES_PER, 0);
  }
}

template <int MT, int WM, bool LEFT>
__global__ __launch_bounds__(256) void project_mfma_kernel(const TensorDesc* __restrict__ descs, StepParams sp,
                                                           int tiles, int count) {
  using C = MfmaCfg<MT, WM>;
  using Ctx = MfmaCtx<MT, WM, LEFT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  // XCD-aware numbering: block w runs on XCD w % 8; XCD x works through tensors x, x+8, ...
  const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
  const int tensor = xcd + kXcds * (slot / tiles);
  if (tensor >= count) return;
  const TensorView d(descs[tensor]);
  Ctx cx;
  cx.Pg = reinterpret_cast<const APOLLO_GLOBAL u32x4_t*>(d.P);
  cx.G = reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(d.g);
  cx.lds = lds;
  cx.r = sp.r; cx.m = d.m; cx.n = d.n;
  cx.n0 = min((slot % tiles) * kNT, d.n - kNT);   // ragged last tile: overlap its neighbour instead of
                                                  // masking (both blocks then write identical values)
  cx.rbase = blockIdx.y * C::RT;
  cx.tid = threadIdx.x; cx.lane = cx.tid & 63;
  const int wave = cx.tid >> 6;
  cx.wm = wave / C::WN; cx.wn = wave % C::WN;
  cx.br = cx.tid >> 5; cx.bc = cx.tid & 31;
  cx.ko_r = cx.tid & 7; cx.jl_r = cx.tid >> 3;
  cx.do_sq = blockIdx.y == 0;
  const int stages = cx.m / kKT;
  cx.last_stage = stages - 1;
  const int n = cx.n;

  f32x16_t acc[MT][C::NTW];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < C::NTW; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
  float sq[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  u32x4_t bq0[8], bq1[8];            // G staging: one holds G(s+1), the other receives G(s+2)
  bf16x8_t af0[MT], bf0[C::NTW], af1[MT], bf1[C::NTW];

  // prologue: stage 0 into LDS buffer 0, G(1) on its way into bq1
  cx.dma_a(0, 0);
  cx.load_b(0, bq0);
  cx.load_b(1, bq1);
  cx.accum_sq(bq0, sq);
  cx.store_b(0, bq0);
  cx.template wait_dma<0>();
  __syncthreads();
  cx.read_frags(0, 0, af0, bf0);

  // One stage that has a successor, as straight-line code.  CUR: LDS buffer being multiplied;
  // BQ_NEXT holds G(s+1) (requested one stage ago), BQ_FAR receives G(s+2).
#define APOLLO_STAGE(CUR, S, BQ_NEXT, BQ_FAR)            \
  {                                                       \
    cx.dma_a((S) + 1, (CUR) ^ 1);                         \
    cx.load_b((S) + 2, BQ_FAR);                           \
    __builtin_amdgcn_sched_barrier(0);                    \
    cx.read_frags(CUR, 1, af1, bf1);                      \
    mfma_block<MT, C::NTW>(acc, af0, bf0);                \
    sched_reads_then_mfma<MT + C::NTW, MT * C::NTW>();    \
    __builtin_amdgcn_sched_barrier(0);                    \
    cx.read_frags(CUR, 2, af0, bf0);                      \
    mfma_block<MT, C::NTW>(acc, af1, bf1);                \
    cx.store_b((CUR) ^ 1, BQ_NEXT);                       \
    sched_reads_then_mix<MT + C::NTW, MT * C::NTW, LEFT ? 4 : 0, 1, 8>();  \
    __builtin_amdgcn_sched_barrier(0);                    \
    cx.read_frags(CUR, 3, af1, bf1);                      \
    mfma_block<MT, C::NTW>(acc, af0, bf0);                \
    cx.accum_sq(BQ_NEXT, sq);                             \
    sched_reads_then_mix<MT + C::NTW, MT * C::NTW, 128 / (MT * C::NTW), 0, MT * C::NTW>(); \
    __builtin_amdgcn_sched_barrier(0);                    \
    mfma_block<MT, C::NTW>(acc, af1, bf1);                \
    __builtin_amdgcn_sched_barrier(0);                    \
    cx.template wait_dma<8>();                            \
    __syncthreads();                                      \
    cx.read_frags((CUR) ^ 1, 0, af0, bf0);                \
  }

  int s = 0;
  for (; s + 2 < stages; s += 2) {      // two stages per trip: the staging registers swap roles
    APOLLO_STAGE(0, s, bq1, bq0)
    APOLLO_STAGE(1, s + 1, bq0, bq1)
  }
  if (s + 1 < stages) {                 // s is even: one more stage with a successor
    APOLLO_STAGE(0, s, bq1, bq0)
  }
#undef APOLLO_STAGE
  // last stage (no successor): fragments of its k-step 0 are already in af0 / bf0
  {
    const int cur = (stages - 1) & 1;
    cx.read_frags(cur, 1, af1, bf1);
    mfma_block<MT, C::NTW>(acc, af0, bf0);
    cx.read_frags(cur, 2, af0, bf0);
    mfma_block<MT, C::NTW>(acc, af1, bf1);
    cx.read_frags(cur, 3, af1, bf1);
    mfma_block<MT, C::NTW>(acc, af0, bf0);
    mfma_block<MT, C::NTW>(acc, af1, bf1);
  }

  // epilogue: R = acc / sqrt(r)
  const float scale = sp.rsqrt_r;
  const int lane = cx.lane, n0 = cx.n0;
  if constexpr (LEFT && C::NTW == 4) {
    // n-tile c of this wave holds channel 8 l + c: the four tiles of a lane are four consecutive
    // channels -> one 16-byte store per row
    const int j = n0 + 8 * (lane & 31) + 4 * cx.wn;
    if (j < n) {
#pragma unroll
      for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = cx.rbase + cx.wm * 32 * MT + a * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
          const f32x4_t o = mk_f4(acc[a][0][v] * scale, acc[a][1][v] * scale, acc[a][2][v] * scale,
                                  acc[a][3][v] * scale);
          *reinterpret_cast<APOLLO_GLOBAL f32x4_t*>(d.R + (size_t)i * n + j) = o;
        }
    }
  } else {
#pragma unroll
    for (int a = 0; a < MT; ++a) {
#pragma unroll
      for (int b = 0; b < C::NTW; ++b) {
        const int c = cx.wn * C::NTW + b;
        const int j = LEFT ? n0 + 8 * (lane & 31) + c : n0 + 32 * c + (lane & 31);
        if (j < n) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int i = cx.rbase + cx.wm * 32 * MT + a * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
            d.R[(size_t)i * n + j] = acc[a][b][v] * scale;
          }
        }
      }
    }
  }

  if (cx.do_sq) {
    float* red = reinterpret_cast<float*>(lds);       // all tiles are consumed: reuse the LDS
    __syncthreads();
    if (LEFT) {
      // thread (br, bc) holds partial sums of channels 8 bc .. 8 bc + 7 over its rows: add the 8 br
#pragma unroll
      for (int c = 0; c < 8; ++c) red[cx.br * 264 + 8 * cx.bc + c] = sq[c];
      __syncthreads();
      const int j = n0 + cx.tid;
      if (j < n) {
        float t = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) t += red[k * 264 + cx.tid];
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
        const int j = n0 + cx.jl_r + 32 * u;
        if (cx.ko_r == 0 && j < n) d.colsq[j] = t;
      }
    }
  }
}

bool project_mfma_supported(int rows, int cols, bool left, bool bf16, int r) {
  if (!bf16 || (r & 31) != 0) return false;
  const int m = left ? rows : cols;
  if ((m % kKT) != 0) return false;
  if ((cols & 7) != 0) return false;       // 16-byte gradient loads
  const int n = left ? cols : rows;
  if (n < kNT) return false;               // a block needs a full tile of channels
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
  const int tiles = (n + kNT - 1) / kNT;
  const int per_xcd = (count + kXcds - 1) / kXcds;
  dim3 grid((unsigned)(kXcds * per_xcd * tiles), (unsigned)(sp.r / C::RT), 1);
  hipLaunchKernelGGL((project_mfma_kernel<MT, WM, LEFT>), grid, dim3(256), lds_bytes, st, d_descs, sp, tiles, count);
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
