// Matrix-core projection R = P G for bf16 gradients (Algorithm 1, step 1), variant in which BOTH
// operands reach LDS by direct-to-LDS loads (global_load_lds_dwordx4) and never pass through
// registers; per-channel squared norms of G (limiter, Section 3.2) come from the fragments.
//
// Block = 512 threads (eight waves, two per SIMD) = an RT x 256 tile of R, RT = 32 MT WM; a wave
// owns a (32 MT) x (32 WM) sub-tile.  A wave issues at most one instruction every four cycles, so
// with a single wave per SIMD every address, wait and load instruction is time the matrix core
// idles; with two, one wave's bookkeeping hides behind the other's MFMAs.  The reduced dimension
// is walked in stages of 32 through a ring of kRing LDS buffers; the loads of stage s+3 are in
// flight while stage s is multiplied.  A direct-to-LDS load puts lane i's 16 bytes at (uniform
// base) + 16 i, so the LDS image of a wave's load is fixed to "64 consecutive 16-byte slots";
// which global 16 bytes a lane fetches is free, and that freedom is used to swizzle (the LDS has
// 64 banks of 4 bytes; a b128 read is served 16 lanes at a time, a b64 read 32 lanes at a time):
//   A (P from the scratch, fragment-major): slot (octet, row), already fragment order.
//   B, columns projected (G channel-major, reduction index contiguous): slot (channel j, p) holds
//     octet p ^ ((j >> 2) & 3) of channel j; a fragment is one ds_read_b128, conflict-free.
//   B, rows projected (reduction index strided): the tile is stored as it is in memory, row k =
//     32 chunks of 8 channels, slot (k, p) holding chunk p ^ (4 (k & 3)); fragments are read with
//     the LDS transpose read ds_read_b64_tr_b16 (within 16 lanes, result lane i, element e =
//     element i % 4 of the 8 bytes addressed by lane 4 e + i / 4), two reads per fragment.
// All vector-memory operations of the main loop are inline assembly (the compiler would wait
// for each direct-to-LDS load separately); vmcnt is therefore managed by hand: every stage
// issues the same number of loads per wave, and "stage s+1 has landed" is vmcnt(loads of one
// stage) because the only younger loads are those of stage s+2.
#include <atomic>

#include "apollo_internal.h"

namespace apollo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
#define APOLLO_LDS __attribute__((address_space(3)))

namespace {

constexpr int kNT = 256;     // channels per block
constexpr int kKT = 32;      // reduction indices per stage (two MFMA k-steps)
constexpr int kRing = 4;     // LDS buffers; kRing - 1 stages of loads in flight
constexpr int kXcds = 8;
constexpr int kBBytes = kKT * kNT * 2;   // 16 KB

constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;

template <int MT, int WM>
struct Cfg {
  static constexpr int RT = 32 * MT * WM;
  static constexpr int WN = kWaves / WM;
  static constexpr int NTW = 8 / WN;                          // = WM
  static constexpr int A_BYTES = (kKT / 8) * RT * 16;
  static constexpr int STAGE_BYTES = A_BYTES + kBBytes;
  static constexpr int A_SLOTS = A_BYTES / 16;
  static constexpr int A_CHUNKS = A_SLOTS / kThreads;         // loads per thread per stage (0 if RT < 128)
  static constexpr int A_LOADS = A_CHUNKS > 0 ? A_CHUNKS : 1;
  static constexpr int B_LOADS = kBBytes / 16 / kThreads;     // 2
  static constexpr int LOADS = A_LOADS + B_LOADS;             // per wave and stage
};

// One direct-to-LDS load: lane i fetches the 16 bytes at (uniform base) + (its own 32-bit byte
// offset) and they land at LDS address (uniform dst) + 16 i.  Base and destination live in scalar
// registers, so a stage's loads cost scalar arithmetic only; the per-lane offsets are loop
// invariants.
__device__ __forceinline__ void dma16(const APOLLO_GLOBAL void* base_uniform, uint32_t lane_off, uint32_t lds_dst_uniform) {
  uint32_t saved_m0;   // M0 is restored: the compiler may hold a value of its own there
  // (one wait state between the write of M0 and the load that reads it: the compiler's hazard
  // handling does not look inside inline assembly)
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
               : "=&s"(saved_m0)
               : "s"(lds_dst_uniform), "v"(lane_off), "s"(base_uniform)
               : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// acc + sum of the squares of a fragment's eight bf16 values: four packed dot products
// (v_dot2c_f32_bf16: acc += a.lo b.lo + a.hi b.hi), no unpacking.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float sq_accum8(const bf16x8_t& f, float acc) {
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(f, f, 0, 1), __builtin_shufflevector(f, f, 0, 1), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(f, f, 2, 3), __builtin_shufflevector(f, f, 2, 3), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(f, f, 4, 5), __builtin_shufflevector(f, f, 4, 5), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(f, f, 6, 7), __builtin_shufflevector(f, f, 6, 7), acc, false);
  return acc;
}

template <int MT, int WM, bool LEFT>
struct Ctx {
  using C = Cfg<MT, WM>;
  const APOLLO_GLOBAL u32x4_t* Pg;
  const APOLLO_GLOBAL uint16_t* G;
  unsigned char* lds;
  uint32_t lds_base;     // LDS byte address of `lds`
  int r, m, n, ldg, n0, rbase, tid, lane, wave, wm, wn, last_stage;   // ldg: row pitch of G in elements
  uint32_t a_off[C::A_LOADS], b_off[C::B_LOADS];   // per-lane byte offsets of the loads (loop invariants)

  // Split every load address into a wave-uniform base (one per operand and stage) and a per-lane
  // offset that also carries the position of the load within the stage.
  //   P slot q = tid + 512 u of a stage holds word ((4 s + q / RT) r + rbase + q % RT) of the
  //     scratch (tiles of fewer than 512 slots: the first waves load, the rest repeat the last one's
  //     load, same data to the same place, so that every wave issues the same number of loads).
  //   G, rows projected: wave-load u covers rows k = 4 wave + 2 u + (lane >> 5), lane fetching chunk
  //     (lane & 31) ^ (4 (k & 3)), and k & 3 = (2 u + (lane >> 5)) & 3.
  //   G, columns projected: wave-load u covers channels j = 32 wave + 16 u + (lane >> 2), lane
  //     fetching octet (lane & 3) ^ ((j >> 2) & 3), and (j >> 2) & 3 = (lane >> 4) & 3.
  __device__ __forceinline__ void setup_loads() {
    if (C::A_CHUNKS > 0) {
#pragma unroll
      for (int u = 0; u < C::A_LOADS; ++u) {
        const int q = tid + kThreads * u;
        a_off[u] = (uint32_t)((q / C::RT) * r + q % C::RT) * 16u;
      }
    } else {
      const int q = min(wave, C::A_SLOTS / 64 - 1) * 64 + lane;
      a_off[0] = (uint32_t)((q / C::RT) * r + q % C::RT) * 16u;
    }
#pragma unroll
    for (int u = 0; u < C::B_LOADS; ++u) {
      if (LEFT) {
        const int chunk = (lane & 31) ^ (4 * ((2 * u + (lane >> 5)) & 3));
        b_off[u] = (uint32_t)((2 * u + (lane >> 5)) * ldg + 8 * chunk) * 2u;
      } else {
        const int oct = (lane & 3) ^ ((lane >> 4) & 3);
        b_off[u] = (uint32_t)((16 * u + (lane >> 2)) * m + 8 * oct) * 2u;
      }
    }
  }

  // all loads of stage s (clamped) into ring buffer `buf`: P tile first, then the G tile
  __device__ __forceinline__ void issue(int s, int buf) const {
    s = min(s, last_stage);
    const uint32_t a_base = lds_base + (uint32_t)(buf * C::STAGE_BYTES);
    const uint32_t b_base = a_base + (uint32_t)C::A_BYTES;
    const APOLLO_GLOBAL u32x4_t* a_src = Pg + (size_t)((kKT / 8) * s) * r + rbase;
    if (C::A_CHUNKS > 0) {
#pragma unroll
      for (int u = 0; u < C::A_LOADS; ++u) dma16(a_src, a_off[u], a_base + (uint32_t)(wave * 64 + kThreads * u) * 16u);
    } else {
      dma16(a_src, a_off[0], a_base + (uint32_t)(min(wave, C::A_SLOTS / 64 - 1) * 64) * 16u);
    }
    if (LEFT) {
      const APOLLO_GLOBAL uint16_t* b_src = G + (size_t)(kKT * s + 4 * wave) * ldg + n0;
#pragma unroll
      for (int u = 0; u < C::B_LOADS; ++u) dma16(b_src, b_off[u], b_base + (uint32_t)(4 * wave + 2 * u) * 512u);
    } else {
      const APOLLO_GLOBAL uint16_t* b_src = G + (size_t)(n0 + 32 * wave) * m + kKT * s;
#pragma unroll
      for (int u = 0; u < C::B_LOADS; ++u) dma16(b_src, b_off[u], b_base + (uint32_t)(2 * wave + u) * 1024u);
    }
  }

  // n-tile (32 channels) of the block that this wave's fragment b covers.  The order is rotated
  // by wm so that fragment 0 is a different tile in each of the WM waves sharing the same
  // channels: every wave then sums the norms of its fragment 0 only, and together they cover all.
  __device__ __forceinline__ int tile_of(int b) const { return wn * C::NTW + (b ^ wm); }

  __device__ __forceinline__ void read_frags(int buf, int ks, bf16x8_t (&af)[MT], bf16x8_t (&bf)[C::NTW]) const {
    const unsigned char* A = lds + buf * C::STAGE_BYTES;
    const unsigned char* B = A + C::A_BYTES;
    const int oct = 2 * ks + (lane >> 5);
#pragma unroll
    for (int a = 0; a < MT; ++a)
      af[a] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(
                                               A + (size_t)(oct * C::RT + wm * 32 * MT + a * 32 + (lane & 31)) * 16));
    if (LEFT) {
      const int q = lane >> 4, s16 = lane & 15;
      const int e_s = s16 >> 2, g_s = s16 & 3;
#pragma unroll
      for (int b = 0; b < C::NTW; ++b) {
        const int col0 = 32 * tile_of(b) + 16 * (q & 1) + 4 * g_s;
        s16x4_t h[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const int k = 16 * ks + 8 * (q >> 1) + 4 * t + e_s;
          const unsigned char* p = B + k * 512 + (((col0 >> 3) ^ (4 * (k & 3))) * 16) + ((col0 >> 2) & 1) * 8;
          h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((APOLLO_LDS s16x4_t*)(p));
        }
        typedef short s16x8_t __attribute__((ext_vector_type(8)));
        const s16x8_t both = __builtin_shufflevector(h[0], h[1], 0, 1, 2, 3, 4, 5, 6, 7);
        bf[b] = __builtin_bit_cast(bf16x8_t, both);
      }
    } else {
#pragma unroll
      for (int b = 0; b < C::NTW; ++b) {
        const int j = 32 * tile_of(b) + (lane & 31);
        bf[b] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(B + j * 64 + ((oct ^ ((j >> 2) & 3)) * 16)));
      }
    }
  }
};

template <int MT, int NTW>
__device__ __forceinline__ void mfma_block(f32x16_t (&acc)[MT][NTW], const bf16x8_t (&af)[MT], const bf16x8_t (&bf)[NTW]) {
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < NTW; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
}

// Scheduling hint for one k-step region: the LDS fragment reads of the next k-step are spread over
// the first MFMAs, one group of reads behind each, and the norm arithmetic over all of them.  A
// wave issues in order and its LDS reads take tens of cycles each to issue: bunched at the head of
// the k-step they would leave the matrix core idle; placed behind an MFMA they issue while it runs,
// and the last of them still has half a k-step to land.
//   masks of sched_group_barrier: 0x2 VALU, 0x8 MFMA, 0x100 LDS read
template <int READS, int MFMAS, int VALU_PER, int G = 0>
__device__ __forceinline__ void sched_kstep() {
  if constexpr (G < MFMAS) {
    constexpr int kSpread = MFMAS > 1 ? (MFMAS + 1) / 2 : 1;   // MFMAs that carry reads
    constexpr int nr = G < kSpread ? (G + 1) * READS / kSpread - G * READS / kSpread : 0;
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if constexpr (nr > 0) __builtin_amdgcn_sched_group_barrier(0x100, nr, 0);
    if constexpr (VALU_PER > 0) __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, 0);
    sched_kstep<READS, MFMAS, VALU_PER, G + 1>();
  }
}

template <int MT, int WM, bool LEFT>
__global__ __launch_bounds__(kThreads) void project_mfma_kernel(const TensorDesc* __restrict__ descs, StepParams sp,
                                                                    int tiles, int count, int padded) {
  using C = Cfg<MT, WM>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  // XCD-aware numbering: block w runs on XCD w % 8; XCD x works through tensors x, x+8, ...
  // Within a tensor the row tiles of one channel tile are neighbours on their XCD: they read the
  // same tile of G at about the same time, so all but the first find it in that XCD's L2.
  const int row_tiles = sp.r / C::RT;
  const int xcd = blockIdx.x % kXcds, slot = (blockIdx.x / kXcds) / row_tiles;
  const int row_tile = (blockIdx.x / kXcds) % row_tiles;
  const int tensor = xcd + kXcds * (slot / tiles);
  if (tensor >= count) return;
  const TensorView d(descs[tensor]);
  Ctx<MT, WM, LEFT> cx;
  cx.Pg = reinterpret_cast<const APOLLO_GLOBAL u32x4_t*>(d.P);
  cx.G = reinterpret_cast<const APOLLO_GLOBAL uint16_t*>(padded ? (const APOLLO_GLOBAL void*)d.gpad : d.g);
  cx.lds = lds;
  cx.lds_base = (uint32_t)(uintptr_t)(APOLLO_LDS unsigned char*)lds;
  cx.r = sp.r; cx.m = d.m; cx.n = d.n; cx.ldg = d.ldg;
  // the ragged last tile overlaps its neighbour.  With rows projected its start stays a multiple
  // of 8 channels (16-byte loads), so with padded rows it may reach up to 7 channels past n: those
  // read the zero padding and are not stored.  With columns projected a channel is a stored row
  // and the tile ends exactly at n.
  cx.n0 = min((slot % tiles) * kNT, LEFT ? (d.n - kNT + 7) & ~7 : d.n - kNT);
  cx.rbase = row_tile * C::RT;
  cx.tid = threadIdx.x; cx.lane = cx.tid & 63; cx.wave = __builtin_amdgcn_readfirstlane(cx.tid >> 6);
  cx.wm = cx.wave / C::WN; cx.wn = cx.wave % C::WN;
  const int stages = cx.m / kKT;
  cx.last_stage = stages - 1;
  cx.setup_loads();

  f32x16_t acc[MT][C::NTW];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < C::NTW; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
  float sq = 0.f;    // squared norm of this wave's fragment-0 channels (see tile_of)
  bf16x8_t af0[MT], bf0[C::NTW], af1[MT], bf1[C::NTW];

  // prologue: three stages requested, wait for the first
#pragma unroll
  for (int p = 0; p < kRing - 1; ++p) cx.issue(p, p);
  wait_vmcnt<(kRing - 2) * C::LOADS>();
  __syncthreads();
  cx.read_frags(0, 0, af0, bf0);

  for (int s = 0; s < stages; ++s) {
    const int cur = s % kRing;
    // k-step 0 of stage s, fragments of k-step 1 on their way
    cx.read_frags(cur, 1, af1, bf1);
    mfma_block<MT, C::NTW>(acc, af0, bf0);
    sq = sq_accum8(bf0[0], sq);
    sched_kstep<MT + (LEFT ? 2 : 1) * C::NTW, MT * C::NTW, (4 + MT * C::NTW - 1) / (MT * C::NTW)>();
    __builtin_amdgcn_sched_barrier(0);
    // stage s+1 has landed once only the loads of stage s+2 are outstanding; after the barrier
    // every wave is past stage s-1, whose buffer then receives stage s+3
    wait_vmcnt<(kRing - 3) * C::LOADS>();
    __syncthreads();
    cx.issue(s + kRing - 1, (s + kRing - 1) % kRing);
    __builtin_amdgcn_sched_barrier(0);
    // k-step 1 of stage s, fragments of k-step 0 of stage s+1 on their way
    cx.read_frags((s + 1) % kRing, 0, af0, bf0);
    mfma_block<MT, C::NTW>(acc, af1, bf1);
    sq = sq_accum8(bf1[0], sq);
    sched_kstep<MT + (LEFT ? 2 : 1) * C::NTW, MT * C::NTW, (4 + MT * C::NTW - 1) / (MT * C::NTW)>();
    __builtin_amdgcn_sched_barrier(0);
  }
  wait_vmcnt<0>();      // drain the (clamped, redundant) loads still in flight before LDS is reused

  // epilogue: R = acc / sqrt(r); n-tile c of the block covers channels n0 + 32 c .. + 31
  const float scale = sp.rsqrt_r;
  const int lane = cx.lane, n = cx.n;
#pragma unroll
  for (int a = 0; a < MT; ++a) {
#pragma unroll
    for (int b = 0; b < C::NTW; ++b) {
      const int j = cx.n0 + 32 * cx.tile_of(b) + (lane & 31);
      if (j < n) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = cx.rbase + cx.wm * 32 * MT + a * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
          d.R[(size_t)i * n + j] = acc[a][b][v] * scale;
        }
      }
    }
  }
  if (row_tile == 0) {
    // lanes l and l + 32 hold the two k-halves of channel (tile, l % 32)
    const float t = sq + __shfl_xor(sq, 32, 64);
    const int j = cx.n0 + 32 * cx.tile_of(0) + lane;
    if (lane < 32 && j < n) d.colsq[j] = t;
  }
}

template <int MT, int WM, bool LEFT>
hipError_t launch_cfg(const TensorDesc* d_descs, int count, int n, bool padded, const StepParams& sp, hipStream_t st) {
  using C = Cfg<MT, WM>;
  const int lds_bytes = kRing * C::STAGE_BYTES;
  static std::atomic<bool> attr_done{false};   // (two threads arriving together both set the attribute: harmless)
  if (!attr_done.load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&project_mfma_kernel<MT, WM, LEFT>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_done.store(true, std::memory_order_release);
  }
  const int tiles = (n + kNT - 1) / kNT;
  const int per_xcd = (count + kXcds - 1) / kXcds;
  dim3 grid((unsigned)(kXcds * per_xcd * tiles * (sp.r / C::RT)), 1, 1);
  hipLaunchKernelGGL((project_mfma_kernel<MT, WM, LEFT>), grid, dim3(kThreads), lds_bytes, st, d_descs, sp, tiles, count,
                     padded ? 1 : 0);
  return hipGetLastError();
}

template <bool LEFT>
hipError_t launch_side(const TensorDesc* d_descs, int count, int n, bool padded, const StepParams& sp, hipStream_t st) {
  const int r = sp.r;
  if (r % 256 == 0) return launch_cfg<4, 2, LEFT>(d_descs, count, n, padded, sp, st);
  if (r % 128 == 0) return launch_cfg<2, 2, LEFT>(d_descs, count, n, padded, sp, st);
  if (r % 64 == 0) return launch_cfg<1, 2, LEFT>(d_descs, count, n, padded, sp, st);
  return launch_cfg<1, 1, LEFT>(d_descs, count, n, padded, sp, st);
}

}  // namespace

bool project_mfma_supported(int rows, int cols, bool left, bool bf16, int r) {
  if (!bf16 || (r & 31) != 0) return false;
  const int m = left ? rows : cols;
  if ((m % 64) != 0) return false;          // whole stages, and P's octets full
  const int n = left ? cols : rows;
  if (n < kNT) return false;                // a block needs a full tile of channels
  return true;
}

// Rows of the stored gradient must start on 16-byte boundaries.  With columns projected the row
// length is m (a multiple of 64); with rows projected it is n, and a row length that is not a
// multiple of 8 elements needs the padded scratch copy (launch_pad_gradient).
bool project_mfma_needs_padding(int rows, int cols, bool left) {
  (void)rows;
  return left && (cols & 7) != 0;
}

hipError_t launch_project_mfma(const TensorDesc* d_descs, int count, int rows, int cols, bool left, bool padded,
                               const StepParams& sp, hipStream_t st) {
  const int n = left ? cols : rows;
  return left ? launch_side<true>(d_descs, count, n, padded, sp, st) : launch_side<false>(d_descs, count, n, padded, sp, st);
}

}  // namespace apollo
