// Host/device shared declarations of the APOLLO step library (internal; the public interface
// is include/apollo.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "philox_gauss.hpp"

namespace apollo {

// One weight matrix as the kernels see it.  Resident in the workspace; only w and g change
// between steps.  m = projected (reduced) dimension, n = channel dimension (Algorithm 1 has
// W in R^{m x n}, m <= n; `left` says whether m runs along the stored rows).
struct TensorDesc {
  void* w;             // rows x cols, fp32, bf16 or 8-bit codes, updated in place
  float* w_meta;       // 8-bit weights: (scale, zero) per group of 128 elements, else unused
  const void* g;       // rows x cols, bf16 or fp32
  void* M;             // state: M^R, r x n, fp32 or bf16
  void* V;             // state: V^R, r x n
  float* prev_norm;    // state: stored norm of the scaled gradient (limiter), 1 float
  void* P;             // scratch: unit-variance projection z, fragment-major (see p_index)
  void* gpad;          // scratch: copy of g with rows padded to ldg elements (16-byte aligned rows), or null
  float* R;            // scratch: n_slabs partial copies of R, each r x n (slab 0 ends canonical); matrix-core path:
                       // no R, but with several row tiles per channel tile their sums a_j, b_j (2 n floats per row tile)
  float* colsq;        // scratch: n_slabs partial copies of sum_i G[i,j]^2, each n
  float* s;            // scratch: channel factors s_j, n floats
  float* partials;     // scratch: 4 floats per block of the moment kernel (sums of a_j, b_j, colsq_j, s_j^2 colsq_j)
  float* scal;         // scratch: [0] lr*alpha*c(*s for tensor mode) [1] c [2] norm [3] s (tensor mode)
  int32_t rows, cols;
  int32_t m, n;
  int32_t m8;          // m rounded up to a multiple of 8 (row length of P in the scratch)
  int32_t left;        // 1: m = rows (R = P G), 0: m = cols (R = G P^T)
  int32_t tensor_id;   // index in the caller's list: part of the generator's counter
  int32_t n_slabs;     // number of partial sums the projection kernel leaves along m
  int32_t k2_blocks;   // blocks of the moment kernel (256 channels each)
  int32_t ldg;         // row pitch, in elements, of the gradient the matrix-core projection reads (gpad or g)
};

// Per-step scalars handed to the kernels by value.
struct StepParams {
  PhiloxKeySchedule ks;
  uint32_t epoch;      // (step-1) / T
  int32_t r;           // rank
  int32_t tensor_mode; // 1 = one factor per tensor (APOLLO-Mini), 0 = per channel
  float rsqrt_r;       // 1/sqrt(r): the variance 1/r of P applied to the product
  float beta1, beta2, omb1, omb2, eps;
  float inv_bc1, inv_bc2;  // 1/(1-beta^t) or 1
  float alpha, gamma;
  float lr, lr_decay;  // lr, lr * lambda
  uint32_t step_lo;    // step mod 2^32 (counter word of the weight-rounding stream)
  int32_t q8_stochastic;
};

// A step's scalars and the bookkeeping of the projection scratch in DEVICE memory (in the workspace),
// for steps that are replayed from a HIP graph: a replayed launch cannot carry new kernel arguments,
// so its kernels read the scalars from here, where apollo_step_prepare wrote them.
struct StepState {
  StepParams sp;
  uint32_t p_epoch;    // refresh epoch of the P the scratch holds (written by the limiter kernel of every step)
  int32_t p_valid;     // 0: the scratch holds no P yet
  int32_t regen;       // this step has to write the scratch copy of P first (set by apollo_step_prepare)
  int32_t pad;
};

// How the launches of a step get their scalars: by value (dev == nullptr: the ordinary step), or from
// device memory (a step that may be captured and replayed).  `host` is always filled: the launchers
// take what shapes the launch (rank, mode) from it, and those do not change from step to step.
struct StepArgs {
  StepParams host;
  StepState* dev;
};
// The scalars as a kernel sees them.  The device copy is read as constant memory (scalar loads: the
// values stay wave-uniform in scalar registers, as kernel arguments are); no kernel writes the
// scalars while a step's kernels run (apollo_step_prepare's kernel precedes them in stream order).
__device__ __forceinline__ StepParams step_params(const StepParams& by_value, const StepState* ss) {
  static_assert(sizeof(StepParams) % 4 == 0, "copied word by word");
  typedef const __attribute__((address_space(4))) uint32_t* constant_words_t;
  if (!ss) return by_value;
  StepParams out;
  constant_words_t src = (constant_words_t)(uintptr_t)(&ss->sp);
  uint32_t* dst = reinterpret_cast<uint32_t*>(&out);
#pragma unroll
  for (int i = 0; i < (int)(sizeof(StepParams) / 4); ++i) dst[i] = src[i];
  return out;
}

// Pointers read from a TensorDesc are generic to the compiler; every buffer they name is device
// global memory.  Saying so turns flat_load / flat_store into global_load / global_store, which
// do not tie up the LDS counter (a flat access makes every later LDS wait also wait for it).
#define APOLLO_GLOBAL __attribute__((address_space(1)))
// Clang vector types (usable in any address space, unlike the HIP uint4 / float4 classes).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__host__ __device__ __forceinline__ u32x4_t mk_u4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  u32x4_t v = {a, b, c, d};
  return v;
}
__host__ __device__ __forceinline__ f32x4_t mk_f4(float a, float b, float c, float d) {
  f32x4_t v = {a, b, c, d};
  return v;
}
template <class T>
__device__ __forceinline__ APOLLO_GLOBAL T* gptr(T* p) {
  return (APOLLO_GLOBAL T*)p;
}

// A TensorDesc with its pointers typed as global memory; kernels build one from the table entry.
struct TensorView {
  APOLLO_GLOBAL void* w;
  APOLLO_GLOBAL float* w_meta;
  APOLLO_GLOBAL const void* g;
  APOLLO_GLOBAL void* M;
  APOLLO_GLOBAL void* V;
  APOLLO_GLOBAL float* prev_norm;
  APOLLO_GLOBAL void* P;
  APOLLO_GLOBAL void* gpad;
  APOLLO_GLOBAL float* R;
  APOLLO_GLOBAL float* colsq;
  APOLLO_GLOBAL float* s;
  APOLLO_GLOBAL float* partials;
  APOLLO_GLOBAL float* scal;
  int32_t rows, cols, m, n, m8, left, tensor_id, n_slabs, k2_blocks, ldg;
  __device__ __forceinline__ explicit TensorView(const TensorDesc& d)
      : w(gptr(d.w)), w_meta(gptr(d.w_meta)), g(gptr(d.g)), M(gptr(d.M)), V(gptr(d.V)), prev_norm(gptr(d.prev_norm)), P(gptr(d.P)), gpad(gptr(d.gpad)),
        R(gptr(d.R)), colsq(gptr(d.colsq)), s(gptr(d.s)), partials(gptr(d.partials)), scal(gptr(d.scal)),
        rows(d.rows), cols(d.cols), m(d.m), n(d.n), m8(d.m8), left(d.left), tensor_id(d.tensor_id),
        n_slabs(d.n_slabs), k2_blocks(d.k2_blocks), ldg(d.ldg) {}
};

// One element of the low-rank Adam update (Algorithm 1, step 2; Section 4.1): new moments from the
// old ones and the projected gradient Re, and the Adam-normalised value R~ = M^ / (sqrt(V^) + eps).
// With a bfloat16 state (SB16) the moments are rounded to nearest even first and R~ is formed from
// what is stored.  Hardware square root and reciprocal (1 ulp each) instead of the correctly rounded
// sequences: 3 instead of ~50 instructions per element of kernels that otherwise only stream; the
// error (~3e-7 relative) is far below the binary32 rounding of the sums R~ enters.
template <bool SB16>
__device__ __forceinline__ float adam_element(const StepParams& sp, float Re, float mo, float vo, float& me, float& ve) {
  me = __builtin_fmaf(sp.beta1, mo, sp.omb1 * Re);
  ve = __builtin_fmaf(sp.beta2, vo, sp.omb2 * (Re * Re));
  if (SB16) {
    me = bf16_bits_to_f32(f32_to_bf16_bits(me));
    ve = bf16_bits_to_f32(f32_to_bf16_bits(ve));
  }
  return (me * sp.inv_bc1) * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(ve * sp.inv_bc2) + sp.eps);
}

// Element (kk, i) of the scratch projection: eight consecutive i of one row are contiguous, the
// r rows of such an octet follow each other, octets follow along i.  A matrix-core A fragment
// (32 or 16 rows x 8 i per lane) is then one contiguous, coalesced 16-byte load per lane.
__host__ __device__ inline size_t p_index(int kk, int i, int r) {
  return ((size_t)(i >> 3) * (size_t)r + (size_t)kk) * 8u + (size_t)(i & 7);
}

// One flat parameter tensor of the element-wise AdamW path (Section 3.1, Eq. 1).
struct AdamwDesc {
  void* w;               // numel, fp32 or bf16 (store16), updated in place
  const void* g;         // numel, bf16 or fp32
  void* m;               // state: first moment, fp32 or bf16 (store16)
  void* v;               // state: second moment
  uint64_t numel;
  uint32_t first_block;  // index of the tensor's first block in the launch
  uint16_t bf16;         // gradient is bf16
  uint16_t store16;      // W, M, V are bf16
};

struct AdamwParams {
  float beta1, beta2, omb1, omb2, eps;
  float inv_bc1, inv_bc2;   // 1/(1-beta^t) or 1
  float lr, lr_decay;       // lr, lr * lambda
};

constexpr int kAdamwBlockElems = 1024;   // 256 threads x 4 consecutive elements

hipError_t launch_adamw(const AdamwDesc* d_descs, const uint32_t* d_block_tensor, uint32_t n_blocks,
                        const AdamwParams& p, hipStream_t st);

// ---- launchers (defined in the .hip files); all enqueue on `st` and return the launch status
hipError_t launch_fill_projection(const TensorDesc* d_descs, int count, int r, int m8, bool bf16,
                                  const StepArgs& sa, hipStream_t st);
hipError_t launch_fill_projection_rowmajor(void* out, bool out_bf16, int r, int m, uint32_t tensor_id,
                                           const StepParams& sp, hipStream_t st);
hipError_t launch_project_generic(const TensorDesc* d_descs, int count, int n, bool bf16,
                                  const StepArgs& sa, hipStream_t st);
hipError_t launch_project_rank1(const TensorDesc* d_descs, int count, int rows, int cols, bool left,
                                bool bf16, int n_slabs, const StepArgs& sa, hipStream_t st);
bool project_rank1_supported(int rows, int cols, bool left, bool bf16);
// fused (the step): the kernel also performs the moment update and the channel sums, and the factors
// when one block holds all rows of its channels (project_mfma_row_tiles(r) == 1; otherwise
// launch_channel_factors follows).  Not fused (count must be 1): R is stored to r_override (debug view).
hipError_t launch_project_mfma(const TensorDesc* d_descs, int count, int rows, int cols, bool left, bool padded,
                               bool fused, bool state_bf16, float* r_override, const StepArgs& sa, hipStream_t st);
// The same for several shape groups in one launch (their blocks follow each other in the grid); `first`
// is the group's first descriptor relative to d_descs.
struct MfmaGroupShape {
  int first, count, rows, cols;
  bool left, padded;
};
hipError_t launch_project_mfma_groups(const TensorDesc* d_descs, const MfmaGroupShape* groups, int n_groups, bool fused,
                                      bool state_bf16, float* r_override, const StepArgs& sa, hipStream_t st);
hipError_t launch_channel_factors(const TensorDesc* d_descs, int count, int n, int row_tiles, hipStream_t st);
int project_mfma_row_tiles(int r);
int project_mfma_tiles(int n);
bool project_mfma_needs_padding(int rows, int cols, bool left);
hipError_t launch_pad_gradient(const TensorDesc* d_descs, int count, int rows, int cols, int ldg, hipStream_t st);
bool project_mfma_supported(int rows, int cols, bool left, bool bf16, int r);
hipError_t launch_adam_norms(const TensorDesc* d_descs, int count, int n, bool state_bf16, const StepArgs& sa,
                             hipStream_t st);
hipError_t launch_finalize(const TensorDesc* d_descs, int count, const StepArgs& sa, hipStream_t st);
hipError_t launch_update(const TensorDesc* d_descs, int count, int rows, int cols, bool left, bool bf16,
                         bool w_bf16, const StepArgs& sa, hipStream_t st);
// The same for several shape groups of one gradient type in one launch (small parameter sets).
struct UpdateGroupShape {
  int first, count, rows, cols;
  bool left;
};
hipError_t launch_update_groups(const TensorDesc* d_descs, const UpdateGroupShape* groups, int n_groups, bool bf16, bool w_bf16,
                                const StepArgs& sa, hipStream_t st);
int adam_norms_blocks(int n);
hipError_t launch_adam_identity(const TensorDesc* d_descs, int count, int rows, int cols, bool left, bool g_bf16,
                                bool state_bf16, const StepArgs& sa, hipStream_t st);
hipError_t launch_update_q8(const TensorDesc* d_descs, int count, int rows, int cols, bool left, bool bf16,
                            const StepArgs& sa, hipStream_t st);
hipError_t launch_bf16_to_f32(float* dst, const void* src, size_t count, hipStream_t st);
hipError_t launch_philox_words(const uint32_t* ctr, uint32_t k0, uint32_t k1, uint32_t* out,
                               int64_t count, hipStream_t st);
hipError_t launch_gauss_parts(uint32_t first, int64_t count, float* radius, float* cosv, float* sinv,
                              hipStream_t st);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st);
// Writes a step's scalars into device memory and decides whether that step has to write P first:
// force_regen, or the scratch holds none, or one of another refresh epoch.  reset: mark the scratch empty.
hipError_t launch_set_step(StepState* d_state, const StepParams& sp, bool force_regen, bool reset, hipStream_t st);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t st);

}  // namespace apollo
