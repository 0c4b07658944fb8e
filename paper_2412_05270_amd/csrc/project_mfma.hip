// Matrix-core projection R = P G for bf16 gradients (Algorithm 1, step 1), variant in which BOTH
// operands reach LDS by direct-to-LDS loads (global_load_lds_dwordx4) and never pass through
// registers; per-channel squared norms of G (limiter, Section 3.2) come from the fragments.
//
// Block = 512 threads (eight waves, two per SIMD) = an RT x 256 tile of R, RT = 32 MT WM; a wave
// owns a (32 MT) x (32 WM) sub-tile.  A wave issues at most one instruction every four cycles, so
// with a single wave per SIMD every address, wait and load instruction is time the matrix core
// idles; with two, one wave's bookkeeping hides behind the other's MFMAs.  The reduced dimension
// is walked in stages of 32 through a ring of kRing LDS buffers; the loads of stages s+1 .. s+3
// are in flight or landed while stage s is multiplied, and stage s's buffer is refilled (with stage s+4) as soon as
// its second half has gone to registers.  A direct-to-LDS load puts lane i's 16 bytes at (uniform
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
#include <algorithm>
#include <atomic>

#include "apollo_internal.h"
#include "state_io.hpp"

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

  // load u (0 .. LOADS-1) of stage s (clamped) into ring buffer `buf`: the P tile's loads first, then the G tile's
  __device__ __forceinline__ void issue_one(int s, int buf, int u) const {
    s = min(s, last_stage);
    const uint32_t a_base = lds_base + (uint32_t)(buf * C::STAGE_BYTES);
    const uint32_t b_base = a_base + (uint32_t)C::A_BYTES;
    if (u < C::A_LOADS) {
      const APOLLO_GLOBAL u32x4_t* a_src = Pg + (size_t)((kKT / 8) * s) * r + rbase;
      if (C::A_CHUNKS > 0) dma16(a_src, a_off[u], a_base + (uint32_t)(wave * 64 + kThreads * u) * 16u);
      else dma16(a_src, a_off[0], a_base + (uint32_t)(min(wave, C::A_SLOTS / 64 - 1) * 64) * 16u);
    } else if (LEFT) {
      const int ub = u - C::A_LOADS;
      const APOLLO_GLOBAL uint16_t* b_src = G + (size_t)(kKT * s + 4 * wave) * ldg + n0;
      dma16(b_src, b_off[ub], b_base + (uint32_t)(4 * wave + 2 * ub) * 512u);
    } else {
      const int ub = u - C::A_LOADS;
      const APOLLO_GLOBAL uint16_t* b_src = G + (size_t)(n0 + 32 * wave) * m + kKT * s;
      dma16(b_src, b_off[ub], b_base + (uint32_t)(2 * wave + ub) * 1024u);
    }
  }
  __device__ __forceinline__ void issue(int s, int buf) const {
#pragma unroll
    for (int u = 0; u < C::LOADS; ++u) issue_one(s, buf, u);
  }

  // n-tile (32 channels) of the block that this wave's fragment b covers.  The order is rotated
  // by wm so that fragment 0 is a different tile in each of the WM waves sharing the same
  // channels: every wave then sums the norms of its fragment 0 only, and together they cover all.
  __device__ __forceinline__ int tile_of(int b) const { return wn * C::NTW + (b ^ wm); }

  // fragment a (32 rows of P x 16 reduction indices of k-step ks) of the stage in ring buffer `buf`
  __device__ __forceinline__ bf16x8_t read_a(int buf, int ks, int a) const {
    const unsigned char* A = lds + buf * C::STAGE_BYTES;
    const int oct = 2 * ks + (lane >> 5);
    return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(
                                            A + (size_t)(oct * C::RT + wm * 32 * MT + a * 32 + (lane & 31)) * 16));
  }
  // fragment b (16 reduction indices x 32 channels)
  __device__ __forceinline__ bf16x8_t read_b(int buf, int ks, int b) const {
    const unsigned char* B = lds + buf * C::STAGE_BYTES + C::A_BYTES;
    if (LEFT) {
      const int q = lane >> 4, s16 = lane & 15;
      const int e_s = s16 >> 2, g_s = s16 & 3;
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
      return __builtin_bit_cast(bf16x8_t, both);
    } else {
      const int oct = 2 * ks + (lane >> 5);
      const int j = 32 * tile_of(b) + (lane & 31);
      return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(B + j * 64 + ((oct ^ ((j >> 2) & 3)) * 16)));
    }
  }
  __device__ __forceinline__ void read_frags(int buf, int ks, bf16x8_t (&af)[MT], bf16x8_t (&bf)[C::NTW]) const {
#pragma unroll
    for (int a = 0; a < MT; ++a) af[a] = read_a(buf, ks, a);
#pragma unroll
    for (int b = 0; b < C::NTW; ++b) bf[b] = read_b(buf, ks, b);
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

// FUSED (the step's kernel): the epilogue does not store R but carries on with Algorithm 1, steps 2-3,
// on the accumulators: the low-rank Adam update of M^R, V^R for the block's RT rows (read, updated,
// written back: the only pass over the state in the step), and a_j = sum_k R~[k,j]^2, b_j = sum_k
// R[k,j]^2 over those rows (the tile passes through LDS so that the state is accessed in whole rows; a
// lane sums its rows of four channels, the eight waves are combined through LDS in a fixed order).  When the block holds all r rows (r = RT: rank
// 32, 64, 128, 256) it goes on to the channel factor s_j (Eq. 4) and the four block sums the limiter
// kernel consumes; with several row tiles per channel tile (rank 96, 192, 512, ...) it leaves a_j, b_j
// per row tile in the scratch and channel_factors_kernel adds them up.  SB16: the state is bfloat16.
// Not FUSED: R itself is stored, to r_override (the debug view: no R is kept by a step).
// `block` is the block's number within its shape group (see project_mfma_kernel).
template <int MT, int WM, bool LEFT, bool FUSED, bool SB16>
__device__ __forceinline__ void project_body(const TensorDesc* __restrict__ descs, const StepParams& sp, int tiles,
                                             int count, int padded, float* __restrict__ r_override, int block,
                                             unsigned char* lds) {
  using C = Cfg<MT, WM>;
  // XCD-aware numbering: block w runs on XCD w % 8; XCD x works through tensors x, x+8, ...
  // Within a tensor the row tiles of one channel tile are neighbours on their XCD: they read the
  // same tile of G at about the same time, so all but the first find it in that XCD's L2.
  const int row_tiles = sp.r / C::RT;
  const int xcd = block % kXcds, slot = (block / kXcds) / row_tiles;
  const int row_tile = (block / kXcds) % row_tiles;
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

  // prologue: every buffer of the ring requested, wait for the first
#pragma unroll
  for (int p = 0; p < kRing; ++p) cx.issue(p, p);
  wait_vmcnt<(kRing - 1) * C::LOADS>();
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
    // stage s+1 has landed once only the loads of the stages behind it are outstanding.  After the
    // barrier no wave reads stage s's buffer again (its second half went to registers at the top of
    // this iteration, and every wave has waited for those reads), so it receives stage s + kRing
    wait_vmcnt<(kRing - 2) * C::LOADS>();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's fragment reads of stage s have returned
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    // k-step 1 of stage s, with the fragments of k-step 0 of stage s+1 and the loads of stage s + kRing spread
    // between its MFMAs: the texture path takes a wave's 1 KB load every few tens of cycles only, and a
    // wave that waits to issue one issues nothing else.  Issued in one burst behind the barrier, the
    // eight waves' loads queue up and the matrix cores idle meanwhile; issued one at a time behind an
    // MFMA each, a load waits while that MFMA (and the other wave's) run.
    {
      constexpr int NM = MT * C::NTW, NR = MT + C::NTW, NS = NM > NR ? NM : NR;
      const int nb = (s + 1) % kRing, lb = s % kRing;
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        if (i < MT) af0[i] = cx.read_a(nb, 0, i);
        else if (i < NR) bf0[i - MT] = cx.read_b(nb, 0, i - MT);
        if (i < NM) {
          acc[i / C::NTW][i % C::NTW] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af1[i / C::NTW], bf1[i % C::NTW], acc[i / C::NTW][i % C::NTW], 0, 0, 0);
#pragma unroll
          for (int u = 0; u < C::LOADS; ++u)
            if ((u * NM) / C::LOADS == i) cx.issue_one(s + kRing, lb, u);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      sq = sq_accum8(bf1[0], sq);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  wait_vmcnt<0>();      // drain the (clamped, redundant) loads still in flight before LDS is reused

  // epilogue: R = acc / sqrt(r); n-tile c of the block covers channels n0 + 32 c .. + 31
  const float scale = sp.rsqrt_r;
  const int lane = cx.lane, n = cx.n;
  if constexpr (!FUSED) {
    APOLLO_GLOBAL float* Rout = gptr(r_override);
#pragma unroll
    for (int a = 0; a < MT; ++a) {
#pragma unroll
      for (int b = 0; b < C::NTW; ++b) {
        const int j = cx.n0 + 32 * cx.tile_of(b) + (lane & 31);
        if (j < n) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int i = cx.rbase + cx.wm * 32 * MT + a * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
            Rout[(size_t)i * n + j] = acc[a][b][v] * scale;
          }
        }
      }
    }
  } else {
    __syncthreads();                    // every wave is past its last fragment read: the ring is free
    // Two ways to the state, chosen by the row pitch n of M^R and V^R:
    //  * n a multiple of 32: straight from the accumulators' own layout, a half-wave access = 32
    //    consecutive channels of one row = one whole 128-byte line; no barrier, every wave on its own
    //    (measured faster than the row pass below when the pieces are line-aligned: LLaMA-7B shapes
    //    4.2 against 4.5 ms);
    //  * otherwise (LLaMA-1B's 5461 channels): 128-byte pieces would straddle lines, and partially
    //    written lines cost read-modify-write traffic (3.0 against 2.1 ms on those shapes), so the
    //    accumulators go through LDS and M^R, V^R are accessed row by row: the R tile is laid out
    //    row-major in LDS, one chunk of CH rows (the rows of one wave row) at a time, and every wave
    //    walks whole rows of the chunk, a lane owning four consecutive channels -- one wave access =
    //    256 consecutive channels = 1 KB of a row.
    // Either way every wave ends with sums of a_j, b_j over the rows it handled, in red_a / red_b.
    const bool direct = (n & 31) == 0;
    float* red_a = reinterpret_cast<float*>(lds);        // [kWaves][kNT]: every wave's sums over its rows
    float* red_b = red_a + kWaves * kNT;                 // [kWaves][kNT]
    float* csq = red_b + kWaves * kNT;                   // [kNT]
    float* wsum = csq + kNT;                             // [4 waves][4]
    // the shifted last tile overlaps its neighbour: channels below jmin are that tile's
    const int jmin = (slot % tiles) * kNT;
    // lanes l and l + 32 hold the two k-halves of channel (fragment-0 tile, l % 32)
    const float csq_own = sq + __shfl_xor(sq, 32, 64);
    if (direct) {
      // a wave holds sums for its own 32 NTW channels only: the rest of its row of red_a / red_b is zero
      for (int i = cx.tid; i < 2 * kWaves * kNT; i += kThreads) red_a[i] = 0.f;
      __syncthreads();
#pragma unroll
      for (int b = 0; b < C::NTW; ++b) {
        const int jl = 32 * cx.tile_of(b) + (lane & 31);
        const int j = cx.n0 + jl;
        const bool valid = j >= jmin && j < n;
        float a_sum = 0.f, b_sum = 0.f;
#pragma unroll
        for (int a = 0; a < MT; ++a) {
          const size_t idx0 = (size_t)(cx.rbase + cx.wm * 32 * MT + a * 32 + (lane >> 5) * 4) * (size_t)n + (size_t)j;
          typedef float one_t __attribute__((ext_vector_type(1)));
          float mo[16], vo[16];
          if (valid) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const size_t idx = idx0 + (size_t)((v >> 2) * 8 + (v & 3)) * (size_t)n;
              mo[v] = load_state<1, SB16>(d.M, idx)[0];
              vo[v] = load_state<1, SB16>(d.V, idx)[0];
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const size_t idx = idx0 + (size_t)((v >> 2) * 8 + (v & 3)) * (size_t)n;
              const float Re = acc[a][b][v] * scale;
              float me, ve;
              const float rt = adam_element<SB16>(sp, Re, mo[v], vo[v], me, ve);
              a_sum = __builtin_fmaf(rt, rt, a_sum);
              b_sum = __builtin_fmaf(Re, Re, b_sum);
              one_t m1 = {me}, v1 = {ve};
              store_state<1, SB16>(d.M, idx, m1);
              store_state<1, SB16>(d.V, idx, v1);
            }
          }
        }
        a_sum += __shfl_xor(a_sum, 32, 64);
        b_sum += __shfl_xor(b_sum, 32, 64);
        if (lane < 32) {
          red_a[cx.wave * kNT + jl] = a_sum;
          red_b[cx.wave * kNT + jl] = b_sum;
        }
      }
    } else {
      constexpr int CH = 32 * MT;
      static_assert(CH * kNT * (int)sizeof(float) <= kRing * C::STAGE_BYTES, "a chunk of the R tile fits the ring");
      float* tileR = reinterpret_cast<float*>(lds);        // [CH][kNT]
      const int jl0 = 4 * lane, j0 = cx.n0 + jl0;          // this lane's four channels in the row pass
      const int e_lo = max(0, jmin - j0), e_hi = min(4, n - j0);      // those of them that exist and are this tile's
      const bool all4 = e_lo == 0 && e_hi == 4;
      const bool quads_aligned = (n & 3) == 0;             // then every (row, j0) is a multiple of 4 elements
      float a4[4] = {0.f, 0.f, 0.f, 0.f}, b4[4] = {0.f, 0.f, 0.f, 0.f};
      auto load4 = [&](const APOLLO_GLOBAL void* base, size_t idx) -> f32x4_t {
        if (all4) return quads_aligned ? load_state<4, SB16>(base, idx) : load_state<4, SB16, true>(base, idx);
        f32x4_t v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (e >= e_lo && e < e_hi) v[e] = load_state<1, SB16>(base, idx + e)[0];
        return v;
      };
      auto store4 = [&](APOLLO_GLOBAL void* base, size_t idx, f32x4_t v) {
        if (all4) {
          if (quads_aligned) store_state<4, SB16>(base, idx, v);
          else store_state<4, SB16, true>(base, idx, v);
          return;
        }
        typedef float one_t __attribute__((ext_vector_type(1)));
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (e >= e_lo && e < e_hi) {
            one_t o = {v[e]};
            store_state<1, SB16>(base, idx + e, o);
          }
      };
#pragma unroll
      for (int c = 0; c < WM; ++c) {
        if (c > 0) __syncthreads();       // the previous chunk has been consumed
        if (cx.wm == c) {
#pragma unroll
          for (int a = 0; a < MT; ++a)
#pragma unroll
            for (int b = 0; b < C::NTW; ++b) {
              float* col = tileR + (a * 32 + (lane >> 5) * 4) * kNT + 32 * cx.tile_of(b) + (lane & 31);
#pragma unroll
              for (int v = 0; v < 16; ++v) col[((v >> 2) * 8 + (v & 3)) * kNT] = acc[a][b][v] * scale;
            }
        }
        __syncthreads();
        if (e_lo < e_hi) {
          const size_t row0 = (size_t)(cx.rbase + c * CH);
          // wave w takes rows w, w + 8, ... of the chunk, four rows per trip (all loads of a trip first)
          for (int rl = cx.wave; rl < CH; rl += 4 * kWaves) {
            f32x4_t Rv[4], mo[4], vo[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const int row = rl + kWaves * u;
              const size_t idx = (row0 + row) * (size_t)n + (size_t)j0;
              Rv[u] = *reinterpret_cast<const f32x4_t*>(tileR + row * kNT + jl0);
              mo[u] = load4(d.M, idx);
              vo[u] = load4(d.V, idx);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const size_t idx = (row0 + rl + kWaves * u) * (size_t)n + (size_t)j0;
              f32x4_t mn, vn;
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const float Re = Rv[u][e];
                float me, ve;
                const float rt = adam_element<SB16>(sp, Re, mo[u][e], vo[u][e], me, ve);
                a4[e] = __builtin_fmaf(rt, rt, a4[e]);     // (channels that are not this tile's are dropped below)
                b4[e] = __builtin_fmaf(Re, Re, b4[e]);
                mn[e] = me;
                vn[e] = ve;
              }
              store4(d.M, idx, mn);
              store4(d.V, idx, vn);
            }
          }
        }
      }
      __syncthreads();                  // the tile is consumed: its LDS now takes the sums
      *reinterpret_cast<f32x4_t*>(red_a + cx.wave * kNT + jl0) = mk_f4(a4[0], a4[1], a4[2], a4[3]);
      *reinterpret_cast<f32x4_t*>(red_b + cx.wave * kNT + jl0) = mk_f4(b4[0], b4[1], b4[2], b4[3]);
    }
    if (lane < 32) csq[32 * cx.tile_of(0) + lane] = csq_own;
    __syncthreads();
    if (row_tiles > 1) {
      // several row tiles share these channels: leave this tile's sums for channel_factors_kernel
      if (cx.tid < kNT) {
        const int jl = cx.tid, j = cx.n0 + jl;
        if (j >= jmin && j < n) {
          float ae = red_a[jl], be = red_b[jl];
#pragma unroll
          for (int w = 1; w < kWaves; ++w) {     // fixed order
            ae += red_a[w * kNT + jl];
            be += red_b[w * kNT + jl];
          }
          d.R[(size_t)(2 * row_tile) * n + j] = ae;
          d.R[(size_t)(2 * row_tile + 1) * n + j] = be;
          if (row_tile == 0) d.colsq[j] = csq[jl];
        }
      }
      return;
    }
    // one thread per channel of the tile: factor, and the four sums over the block's own channels
    if (cx.tid < kNT) {
      const int jl = cx.tid, j = cx.n0 + jl;
      float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;
      if (j >= jmin && j < n) {
        float ae = red_a[jl], be = red_b[jl];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) {       // fixed order
          ae += red_a[w * kNT + jl];
          be += red_b[w * kNT + jl];
        }
        const float c2 = csq[jl];
        const float sj = (be > 0.f) ? __builtin_sqrtf(ae) / __builtin_sqrtf(be) : 0.f;
        d.s[j] = sj;
        d.colsq[j] = c2;
        t0 = ae;
        t1 = be;
        t2 = c2;
        t3 = sj * sj * c2;
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        t0 += __shfl_xor(t0, off, 64);
        t1 += __shfl_xor(t1, off, 64);
        t2 += __shfl_xor(t2, off, 64);
        t3 += __shfl_xor(t3, off, 64);
      }
      if (lane == 0) {
        wsum[cx.wave * 4 + 0] = t0;
        wsum[cx.wave * 4 + 1] = t1;
        wsum[cx.wave * 4 + 2] = t2;
        wsum[cx.wave * 4 + 3] = t3;
      }
    }
    __syncthreads();
    if (cx.tid < 4)
      d.partials[(size_t)(slot % tiles) * 4 + cx.tid] =
          ((wsum[cx.tid] + wsum[4 + cx.tid]) + wsum[8 + cx.tid]) + wsum[12 + cx.tid];
  }
}

// One launch serves up to kMaxGroups shape groups (tensors of one shape and orientation each): the
// blocks of the groups follow each other in the grid, every group's count a multiple of the XCD
// count, so that block w still runs on XCD w % 8.  A set of a few small tensors then fills the chip
// with one launch, and a large set has one tail of partly idle compute units instead of one per group.
constexpr int kMaxGroups = 8;
struct MfmaGroup {
  int first, count;     // its descriptors: descs[first .. first + count)
  int tiles;            // channel tiles per tensor
  int blocks_end;       // one past its last block in the grid
  int left, padded;     // rows projected; the gradient is read from the row-padded copy
};
struct MfmaGroups {
  MfmaGroup g[kMaxGroups];
  int n;
};

template <int MT, int WM, bool FUSED, bool SB16>
__global__ __launch_bounds__(kThreads) void project_mfma_kernel(const TensorDesc* __restrict__ descs, StepParams sp_arg,
                                                                    StepState* __restrict__ ss, MfmaGroups tbl,
                                                                    float* __restrict__ r_override) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const StepParams sp = step_params(sp_arg, ss);
  const int b = blockIdx.x;
  int first = 0, count = 0, tiles = 1, left = 0, padded = 0, begin = 0;
#pragma unroll
  for (int i = 0; i < kMaxGroups; ++i) {
    const int lo = i ? tbl.g[i - 1].blocks_end : 0;
    if (i < tbl.n && b >= lo && b < tbl.g[i].blocks_end) {
      first = tbl.g[i].first; count = tbl.g[i].count; tiles = tbl.g[i].tiles;
      left = tbl.g[i].left; padded = tbl.g[i].padded; begin = lo;
    }
  }
  if (left) project_body<MT, WM, true, FUSED, SB16>(descs + first, sp, tiles, count, padded, r_override, b - begin, lds);
  else project_body<MT, WM, false, FUSED, SB16>(descs + first, sp, tiles, count, padded, r_override, b - begin, lds);
}

// Channel factors for ranks with several row tiles per channel tile: adds the row tiles' a_j, b_j (fixed
// order), forms s_j (Eq. 4) and leaves the four block sums of 256 channels, as the fused epilogue does
// when one block holds all rows.
__global__ __launch_bounds__(kNT) void channel_factors_kernel(const TensorDesc* __restrict__ descs, int row_tiles) {
  __shared__ float wsum[4][4];
  const TensorView d(descs[blockIdx.y]);
  const int n = d.n, j = blockIdx.x * kNT + threadIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;
  if (j < n) {
    float ae = 0.f, be = 0.f;
    for (int rt = 0; rt < row_tiles; ++rt) {
      ae += d.R[(size_t)(2 * rt) * n + j];
      be += d.R[(size_t)(2 * rt + 1) * n + j];
    }
    const float c2 = d.colsq[j];
    const float sj = (be > 0.f) ? __builtin_sqrtf(ae) / __builtin_sqrtf(be) : 0.f;
    d.s[j] = sj;
    t0 = ae;
    t1 = be;
    t2 = c2;
    t3 = sj * sj * c2;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    t0 += __shfl_xor(t0, off, 64);
    t1 += __shfl_xor(t1, off, 64);
    t2 += __shfl_xor(t2, off, 64);
    t3 += __shfl_xor(t3, off, 64);
  }
  if (lane == 0) {
    wsum[wave][0] = t0;
    wsum[wave][1] = t1;
    wsum[wave][2] = t2;
    wsum[wave][3] = t3;
  }
  __syncthreads();
  if (threadIdx.x < 4)
    d.partials[(size_t)blockIdx.x * 4 + threadIdx.x] =
        ((wsum[0][threadIdx.x] + wsum[1][threadIdx.x]) + wsum[2][threadIdx.x]) + wsum[3][threadIdx.x];
}

template <int MT, int WM, bool FUSED, bool SB16>
hipError_t launch_cfg(const TensorDesc* d_descs, const MfmaGroups& tbl, float* r_override, const StepArgs& sa, hipStream_t st) {
  using C = Cfg<MT, WM>;
  const int lds_bytes = kRing * C::STAGE_BYTES;
  static_assert(!FUSED || kRing * C::STAGE_BYTES >= (int)((2 * kWaves + 1) * kNT + 16) * (int)sizeof(float), "epilogue sums fit the ring");
  static std::atomic<bool> attr_done{false};   // (two threads arriving together both set the attribute: harmless)
  if (!attr_done.load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&project_mfma_kernel<MT, WM, FUSED, SB16>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_done.store(true, std::memory_order_release);
  }
  dim3 grid((unsigned)tbl.g[tbl.n - 1].blocks_end, 1, 1);
  hipLaunchKernelGGL((project_mfma_kernel<MT, WM, FUSED, SB16>), grid, dim3(kThreads), lds_bytes, st, d_descs, sa.host, sa.dev, tbl, r_override);
  return hipGetLastError();
}

template <int MT, int WM>
hipError_t launch_variant(const TensorDesc* d_descs, const MfmaGroups& tbl, bool fused, bool state_bf16, float* r_override,
                          const StepArgs& sa, hipStream_t st) {
  if (!fused) return launch_cfg<MT, WM, false, false>(d_descs, tbl, r_override, sa, st);
  if (state_bf16) return launch_cfg<MT, WM, true, true>(d_descs, tbl, nullptr, sa, st);
  return launch_cfg<MT, WM, true, false>(d_descs, tbl, nullptr, sa, st);
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

// Row tiles per channel tile at rank r (the launcher picks the largest row tile that divides r).
int project_mfma_row_tiles(int r) { return r % 256 == 0 ? r / 256 : r % 128 == 0 ? r / 128 : r % 64 == 0 ? r / 64 : r / 32; }

// Channel tiles per tensor (= block sums left per tensor).
int project_mfma_tiles(int n) { return (n + kNT - 1) / kNT; }

hipError_t launch_project_mfma_groups(const TensorDesc* d_descs, const MfmaGroupShape* groups, int n_groups, bool fused,
                                      bool state_bf16, float* r_override, const StepArgs& sa, hipStream_t st) {
  if (n_groups < 1 || fused == (r_override != nullptr) || (r_override && (n_groups != 1 || groups[0].count != 1)))
    return hipErrorInvalidValue;
  const int r = sa.host.r;
  const int row_tiles = project_mfma_row_tiles(r);
  for (int g0 = 0; g0 < n_groups; g0 += kMaxGroups) {
    MfmaGroups tbl{};
    tbl.n = std::min(kMaxGroups, n_groups - g0);
    int blocks = 0;
    for (int i = 0; i < tbl.n; ++i) {
      const MfmaGroupShape& g = groups[g0 + i];
      const int n = g.left ? g.cols : g.rows;
      const int tiles = project_mfma_tiles(n);
      const int per_xcd = (g.count + kXcds - 1) / kXcds;
      blocks += kXcds * per_xcd * tiles * row_tiles;
      tbl.g[i] = MfmaGroup{g.first, g.count, tiles, blocks, g.left ? 1 : 0, g.padded ? 1 : 0};
    }
    hipError_t e;
    if (r % 256 == 0) e = launch_variant<4, 2>(d_descs, tbl, fused, state_bf16, r_override, sa, st);
    else if (r % 128 == 0) e = launch_variant<2, 2>(d_descs, tbl, fused, state_bf16, r_override, sa, st);
    else if (r % 64 == 0) e = launch_variant<1, 2>(d_descs, tbl, fused, state_bf16, r_override, sa, st);
    else e = launch_variant<1, 1>(d_descs, tbl, fused, state_bf16, r_override, sa, st);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_project_mfma(const TensorDesc* d_descs, int count, int rows, int cols, bool left, bool padded,
                               bool fused, bool state_bf16, float* r_override, const StepArgs& sa, hipStream_t st) {
  const MfmaGroupShape g{0, count, rows, cols, left, padded};
  return launch_project_mfma_groups(d_descs, &g, 1, fused, state_bf16, r_override, sa, st);
}

hipError_t launch_channel_factors(const TensorDesc* d_descs, int count, int n, int row_tiles, hipStream_t st) {
  hipLaunchKernelGGL(channel_factors_kernel, dim3((unsigned)project_mfma_tiles(n), (unsigned)count), dim3(kNT), 0, st, d_descs,
                     row_tiles);
  return hipGetLastError();
}

}  // namespace apollo
