/*
 * apollo.h -- C ABI of the MI355X (gfx950) APOLLO / APOLLO-Mini optimizer-step library.
 *
 * The library performs, for every weight matrix W (rows x cols, row-major, fp32) with
 * gradient G (same shape, bf16 or fp32), the step of Algorithm 1 of "APOLLO: SGD-like
 * Memory, AdamW-level Performance" (arXiv 2412.05270):
 *
 *   1. P  <- seeded Gaussian random projection, r x m, variance 1/r, generated from a
 *            counter-based generator whenever it is needed and never kept as optimizer state
 *            (Algorithm 1 "P_t <- N_seed(0,1/r)"; Section 4.1 "Generating random projection
 *            matrix"); a new P is drawn every T steps.
 *   2. R  <- P G                                   (Algorithm 1, step 1; r x n)
 *   3. M^R, V^R <- Adam moments of R; R~ <- M^R / (sqrt(V^R) + eps)   (Section 4.1)
 *   4. s_j <- ||R~[:,j]|| / ||R[:,j]||  per channel (APOLLO, Eq. 4), or
 *      s   <- ||R~|| / ||R||            per tensor  (APOLLO-Mini, Section 4.2)
 *   5. norm-growth limiter on ||alpha G diag(s)||_F with threshold gamma  (Section 3.2, Eq. 3)
 *   6. W  <- W - lr * alpha * G diag(s) - lr * lambda * W              (Algorithm 1, step 4)
 *
 * m = min(rows, cols) is the projected dimension, n = max(rows, cols) the channel dimension
 * (Algorithm 1 assumes m <= n; a tensor with rows > cols is treated as its transpose without
 * being moved).  All of it runs in hand-written HIP kernels on the stream the caller passes.
 *
 * Conventions
 *   - Every pointer argument is a HOST pointer unless its comment says DEVICE.
 *   - The library allocates no device memory; it creates at most one stream of its own per handle
 *     (see APOLLO_SCHEDULE_OVERLAP).  The caller owns W, G,
 *     the state buffer and the workspace (all DEVICE memory) and keeps them alive while the
 *     handle uses them.  The library owns only the host-side handle.
 *   - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and return without synchronising the stream.  Nothing is read back to the host.
 *     (One wait can occur: apollo_step copies the tensor pointers to the device through one of four
 *     pinned staging slots when they differ from the previous call's; a call that changes them waits
 *     for the copy made four such calls earlier, which has normally long finished.)
 *   - Functions returning apollo_status_t return APOLLO_OK (0) or a negative code; argument
 *     errors are detected before anything is launched.  apollo_last_error() gives the text.
 *   - `g` is the ordinary gradient (d loss / d W); the step subtracts.
 *   - Threads: different handles may be used from different host threads at the same time.  The
 *     calls on one handle must not overlap (the handle keeps the descriptor table, the profiling
 *     events and the error text), and two steps of one handle on different streams are ordered by
 *     the caller (they share the state and the workspace).
 */
#ifndef APOLLO_H_
#define APOLLO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct apollo_handle apollo_handle_t; /* opaque, host-side */

typedef int32_t apollo_status_t;
enum {
  APOLLO_OK = 0,
  APOLLO_EINVAL = -1,       /* null pointer, rank < 1, rank > min(rows, cols), T < 1, bad enum,
                               tensor count mismatch, step < 1, misaligned W/G pointer          */
  APOLLO_ENOMEM = -2,       /* host allocation failed                                           */
  APOLLO_ESTATE = -3,       /* state or workspace buffer too small or not 256-byte aligned      */
  APOLLO_EHIP = -4,         /* a HIP call failed (text in apollo_last_error)                    */
  APOLLO_EUNSUPPORTED = -5  /* gradient dtype other than fp32 / bf16; a dimension above 2^20 or
                               2^31 or more elements in one tensor                             */
};

/* element types: of the gradient (per tensor), of W and of M^R, V^R (per configuration);
   all factors and the stored norm are fp32 */
enum { APOLLO_F32 = 0, APOLLO_BF16 = 1, APOLLO_Q8 = 2 /* weights only: see apollo_config_t */ };
/* rounding of the 8-bit weight codes */
enum { APOLLO_ROUND_NEAREST = 0, APOLLO_ROUND_STOCHASTIC = 1 };
/* launch schedule of a step */
enum { APOLLO_SCHEDULE_SERIAL = 0, APOLLO_SCHEDULE_OVERLAP = 1, APOLLO_SCHEDULE_CHUNKED = 2 };
/* granularity of the scaling factor: APOLLO (Eq. 4) or APOLLO-Mini (Section 4.2) */
enum { APOLLO_CHANNEL = 0, APOLLO_TENSOR = 1 };
/* which dimension is projected away: AUTO = the smaller one (Algorithm 1's m <= n);
   LEFT = rows (R = P G, channels are columns); RIGHT = columns (R = G P^T, channels are rows) */
enum { APOLLO_SIDE_AUTO = 0, APOLLO_SIDE_LEFT = 1, APOLLO_SIDE_RIGHT = 2 };
/* where the moments live: in the random low-rank space of Algorithm 1, or (Section 3.2) in the
   full space */
enum { APOLLO_PROJ_RANDOM = 0, APOLLO_PROJ_IDENTITY = 1 };
/* selectors of apollo_debug_get */
enum {
  APOLLO_DBG_M = 0,     /* M^R, r x n, channel index contiguous; always delivered as fp32      */
  APOLLO_DBG_V = 1,     /* V^R, r x n fp32                                                    */
  APOLLO_DBG_S = 2,     /* scaling factor of the last step: n fp32 (channel) or 1 fp32 (tensor) */
  APOLLO_DBG_NORM = 3,  /* stored norm ||alpha G diag(s)||_F after limiting, 1 fp32            */
  APOLLO_DBG_C = 4,     /* limiter factor c in (0, 1] of the last step, 1 fp32                 */
  APOLLO_DBG_R = 5,     /* R = P G of the last step, r x n fp32.  For a tensor on
                           APOLLO_PATH_MATRIX_CORE no R is kept: it is computed again into `out`
                           from the gradient buffer passed to the last step, which must still
                           hold that step's gradient                                            */
  APOLLO_DBG_COLSQ = 6  /* ||G[:,j]||^2 per channel of the last step, n fp32                   */
};

typedef struct {
  int64_t rows, cols;   /* W and G are rows x cols, row-major, leading dimension = cols        */
  int32_t grad_dtype;   /* APOLLO_F32 or APOLLO_BF16                                           */
  int32_t reserved;     /* set to 0                                                            */
} apollo_shape_t;

/* Hyper-parameters (Algorithm 1's input list; gamma from Section 3.2). */
typedef struct {
  int32_t rank;             /* r >= 1 and r <= min(rows, cols) of every tensor                 */
  int32_t mode;             /* APOLLO_CHANNEL or APOLLO_TENSOR                                 */
  uint64_t seed;            /* key of the counter-based generator                              */
  float beta1, beta2, eps;  /* Adam on R                                                       */
  float scale;              /* alpha: 1 for APOLLO, sqrt(128) for APOLLO-Mini (Sections 4.1/4.2) */
  float weight_decay;       /* lambda (decoupled), 0 = none                                    */
  float nl_gamma;           /* gamma of the norm-growth limiter, 1.01 in the paper; 0 = off    */
  int32_t refresh_interval; /* T >= 1: a new P is drawn when (step-1) % T == 0                 */
  int32_t bias_correction;  /* 1 = Adam's bias correction (default), 0 = literal Section 4.1   */
  int32_t side;             /* APOLLO_SIDE_*                                                   */
  int32_t weight_dtype;     /* APOLLO_F32 (0, default), APOLLO_BF16 or APOLLO_Q8: storage of every W */
  int32_t state_dtype;      /* APOLLO_F32 (0, default) or APOLLO_BF16: element type of M^R, V^R */
  int32_t projection;       /* APOLLO_PROJ_RANDOM (0, default) or APOLLO_PROJ_IDENTITY          */
  int32_t weight_rounding;  /* APOLLO_ROUND_* of the codes when weight_dtype is APOLLO_Q8       */
  int32_t schedule;         /* APOLLO_SCHEDULE_SERIAL (0, default), _OVERLAP or _CHUNKED          */
} apollo_config_t;

/* APOLLO_SCHEDULE_OVERLAP: when some projection runs on the matrix cores (bf16 gradients, rank a
 * multiple of 32) and the tensors form more than one shape group, apollo_step runs the groups as
 * chains on two streams -- the caller's and one the library creates in apollo_init (default
 * priority, destroyed by apollo_destroy) -- so that one group's projection overlaps another group's
 * memory-bound kernels.  The second stream is forked from and joined back into `hip_stream` within
 * the call: the caller sees ordinary in-order work on its stream.  Results are bit-identical to
 * APOLLO_SCHEDULE_SERIAL (the groups touch disjoint data); the gain measured on MI355X is small
 * (about 3 % of a rank-256 step: the projection and the streaming kernels contend for the same
 * load path), which is why it is not the default.  Steps recorded by apollo_profile_enable use the
 * serial schedule, which is the one that has phases to time. */

/* APOLLO_SCHEDULE_CHUNKED: P is not kept from step to step.  For rank > 1 the default schedules hold
 * every tensor's P in the workspace for a whole refresh interval (Algorithm 1 holds P_t until it is
 * re-sampled), r x m elements per tensor -- 0.47 GB for the LLaMA-7B matrices at rank 256.  With this
 * schedule a step works through each shape group in chunks of tensors whose P together fit 128 MiB:
 * generate the chunk's P from the seed, project the chunk (the moment update included where the
 * projection runs on the matrix cores), go on to the next chunk over the same scratch; limiter and
 * update follow as usual.  apollo_workspace_bytes shrinks accordingly (7B, rank 256: 0.13 GB); every
 * step pays the generation (about 2 % of such a step) and a few more launches.  Results are
 * bit-identical to APOLLO_SCHEDULE_SERIAL.  apollo_step_launch (the replayable step) is not offered
 * with it (APOLLO_EUNSUPPORTED); apollo_step_noalloc ignores the schedule. */

/* APOLLO_Q8: group-wise 8-bit weights (Section 5.4 / Table 6 combine APOLLO with 8-bit integer
 * weights quantised in groups of 128, and say no more; the reading taken is the usual asymmetric
 * min/max group quantiser with optional stochastic rounding).  W is held as unsigned 8-bit codes
 * q (rows x cols, row-major, cols a multiple of 128) and, per group of 128 consecutive elements,
 * an fp32 pair (scale, zero) in apollo_tensor_t.w_meta:  w = zero + scale * q.  A step de-quantises,
 * applies the update of Algorithm 1 (step 4) in fp32 and quantises every group again from its own
 * new range: zero' = min w', scale' = (max w' - min w') / 255, q' = min(255, floor((w' - zero') /
 * scale' + u)), u = 1/2 (nearest) or, stochastic, a 16-bit uniform from Philox4x32-10 under `seed`
 * with counter (o mod 2^32, step mod 2^32, 2^31 + tensor index, o div 2^32), o = e div 8 for
 * flattened element index e; output word k gives element 8 o + 2 k its low and element
 * 8 o + 2 k + 1 its high 16 bits, u = bits / 65536. */

/* APOLLO_PROJ_IDENTITY: no projection at all -- the structured channel-wise rule of Section 3.2
 * (Eq. 2) itself, with full-rank Adam moments of G: G~ = M^ / (sqrt(V^) + eps), s_j = ||G~[:,j]|| /
 * ||G[:,j]|| (or one factor per tensor with APOLLO_TENSOR), limiter and update as in Algorithm 1.
 * It is the reference the low-rank factors approximate (Theorem 4.1's ratio sqrt(r/n) is measured
 * against it).  `rank` is ignored (r = m, P = I, no 1/sqrt(r)); the moments have the tensor's own
 * rows x cols row-major layout, which is also what apollo_debug_get delivers for M and V;
 * APOLLO_DBG_R is not available.  State: 2 rows cols elements + 1 norm per tensor. */

/* Storage in bfloat16 (the paper trains in the bfloat16 format and sizes the state at 2 bytes per
 * element, Table 3, without giving a rounding rule): arithmetic is fp32; a quantity kept in
 * bfloat16 is rounded to nearest, ties to even, when it is stored, and whatever is computed after
 * that uses the stored value (R~ is formed from the rounded moments), so the state alone
 * determines the rest of the step.  An update smaller than half a unit in the last place of a
 * bfloat16 weight is lost; that is a property of the format, not of this library. */

typedef struct {
  void* w;        /* DEVICE, weight_dtype (fp32 by default), rows x cols, 16-byte aligned,
                     updated in place                                                          */
  const void* g;  /* DEVICE, grad_dtype, rows x cols, 16-byte aligned, read only               */
  void* w_meta;   /* DEVICE, only with APOLLO_Q8 weights (else ignored, may be NULL): rows * cols /
                     128 pairs (scale, zero) fp32, 8-byte aligned, updated in place              */
} apollo_tensor_t;

/* Bytes of optimizer state for the tensor list (Table 1: 2nr + 2 scalars per tensor, here
 * 2nr moments + 1 norm, the seed being in the config), 0 on invalid arguments.
 * Layout, stable and meant for checkpointing: per tensor, in list order, each block starting
 * on a 256-byte boundary: M^R[r][n], V^R[r][n] (state_dtype: fp32 or bf16), prev_norm fp32. */
size_t apollo_state_bytes(const apollo_config_t* cfg, const apollo_shape_t* shapes, int32_t n_tensors);

/* Byte offsets of one tensor's M^R, V^R and prev_norm inside the state buffer.  Any of the
 * output pointers may be NULL.  Pure host arithmetic. */
apollo_status_t apollo_state_offsets(const apollo_config_t* cfg, const apollo_shape_t* shapes,
                                     int32_t n_tensors, int32_t tensor, size_t* m_offset,
                                     size_t* v_offset, size_t* norm_offset);

/* Bytes of scratch (the generated P, R (except on APOLLO_PATH_MATRIX_CORE), per-channel sums, factors, per-tensor scalars, the device
 * descriptor table and, for a bf16 tensor whose rows are projected and whose row length is not a
 * multiple of 8, a copy of its gradient with rows padded to 16 bytes).  The library keeps P there
 * from one step to the next within a refresh interval (Algorithm 1 holds P_t until it is re-sampled)
 * and re-generates it whenever the step's interval differs from the one it holds: P is never
 * optimizer state, nothing in the workspace has to be saved.  The caller must not write to the
 * workspace while the handle lives.  0 on invalid arguments. */
size_t apollo_workspace_bytes(const apollo_config_t* cfg, const apollo_shape_t* shapes, int32_t n_tensors);

/* Creates a handle for a fixed tensor list.  `state` (DEVICE, >= apollo_state_bytes, 256-byte
 * aligned) is zero-filled on `hip_stream` (M^R_0 = V^R_0 = 0, Section 4.1; stored norm 0 =
 * "unset") unless `zero_state` is 0 (resume from a checkpointed buffer).  `workspace` (DEVICE,
 * >= apollo_workspace_bytes, 256-byte aligned).  On failure *out is NULL. */
apollo_status_t apollo_init(apollo_handle_t** out, const apollo_config_t* cfg,
                            const apollo_shape_t* shapes, int32_t n_tensors, void* state,
                            size_t state_bytes, void* workspace, size_t workspace_bytes,
                            int32_t zero_state, void* hip_stream);

/* One optimizer step (Algorithm 1) on every tensor of the list.  `tensors[i]` carries the
 * DEVICE pointers of the i-th shape given to apollo_init; n_tensors must match.  `step` is
 * 1-based; the projection epoch is (step-1) / T and the bias-correction exponent is `step`,
 * so steps need not be consecutive, but M^R, V^R and the stored norm are what the previous
 * call left.  Calls on one handle must be ordered on one stream (or otherwise serialised). */
apollo_status_t apollo_step(apollo_handle_t* h, const apollo_tensor_t* tensors, int32_t n_tensors,
                            int64_t step, float lr, void* hip_stream);

/* The step in two parts, for callers that replay it from a HIP graph (a replayed launch cannot carry
 * a new step number or learning rate in its kernel arguments):
 *   apollo_step_prepare  writes the scalars of step `step` (bias corrections, refresh epoch, lr, ...) into
 *                        the workspace with one small kernel and decides there whether that step has to
 *                        write the scratch copy of P first (the scratch holds none, or another epoch's);
 *   apollo_step_launch   enqueues the kernels of one step, which read those scalars from device memory:
 *                        the same kernels, launch shapes and results as apollo_step (serial schedule).
 * apollo_step_prepare(h, t, lr, s) followed by apollo_step_launch(h, tensors, n, s) equals apollo_step(h,
 * tensors, n, t, lr, s) bit for bit.  Capture apollo_step_launch alone (it then only launches kernels:
 * no copy, no memset, no event), after one ordinary call with the same tensor pointers -- a call whose
 * pointers differ from the previous call's first copies them to the device, which does not belong into
 * a graph -- and per iteration call apollo_step_prepare on the stream and launch the graph after it.
 * The weights, gradients, state and workspace must be the buffers the graph was captured with.  The kernel
 * that writes P is part of every replay and returns at once when the scratch is current. */
apollo_status_t apollo_step_prepare(apollo_handle_t* h, int64_t step, float lr, void* hip_stream);
apollo_status_t apollo_step_launch(apollo_handle_t* h, const apollo_tensor_t* tensors, int32_t n_tensors,
                                   void* hip_stream);

/* For callers that cannot allocate device memory or call anything that does (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): one step of Algorithm 1 on a short
 * tensor list, the same kernels and results as apollo_init(..., zero_state, ...) followed by
 * apollo_step on a fresh handle, but with no handle and no workspace argument.  The scratch lives
 * in a static device array of APOLLO_NOALLOC_SCRATCH_BYTES inside the library (one copy per GPU,
 * held until the process ends); the tensor descriptors reach the device as kernel arguments.  The
 * call makes no hipMalloc, hipFree, hipHostMalloc, event or stream creation and no memset or copy
 * engine request: it only launches kernels on `hip_stream`.
 *   - `state` (DEVICE, 256-byte aligned, >= apollo_state_bytes(cfg, shapes, n_tensors)) is the
 *     caller's, with the layout documented at apollo_state_bytes; it is zero-filled first (by a
 *     kernel) if `zero_state` is not 0, otherwise it holds what the previous step left.
 *   - At most APOLLO_NOALLOC_MAX_TENSORS tensors per call, and apollo_workspace_bytes(cfg, shapes,
 *     n_tensors) must not exceed APOLLO_NOALLOC_SCRATCH_BYTES: otherwise APOLLO_EUNSUPPORTED, with
 *     the sizes in apollo_last_error(NULL), and nothing is launched.  (One LLaMA-7B layer fits at
 *     rank 1; larger lists go through apollo_init / apollo_step, or layer by layer.)
 *   - The device of `hip_stream` must be the current device.  `cfg->schedule` is ignored (serial).
 *   - P is generated in every call (the scratch keeps nothing from one call to the next), the
 *     random stream and every result are the ones apollo_step gives for the same (seed, step,
 *     tensor index in the list).
 *   - All calls on one GPU share that GPU's scratch: two calls whose kernels may overlap in time
 *     (different streams without an ordering between them, different host threads) race; calls
 *     on one stream are safe. */
#define APOLLO_NOALLOC_SCRATCH_BYTES (32 * 1024 * 1024)
#define APOLLO_NOALLOC_MAX_TENSORS 64
apollo_status_t apollo_step_noalloc(const apollo_config_t* cfg, const apollo_shape_t* shapes,
                                    const apollo_tensor_t* tensors, int32_t n_tensors, void* state,
                                    size_t state_bytes, int32_t zero_state, int64_t step, float lr,
                                    void* hip_stream);

/* Writes the unit-variance projection z (P = z / sqrt(r)) that `step` would use for tensor
 * `tensor`, as a row-major r x m matrix of `dtype` (APOLLO_F32: the fp32 variates; APOLLO_BF16:
 * rounded to bf16, nearest-even) into `out` (DEVICE, r*m elements). */
apollo_status_t apollo_debug_fill_projection(apollo_handle_t* h, int32_t tensor, int64_t step,
                                             void* out, int32_t dtype, void* hip_stream);

/* Copies one quantity (APOLLO_DBG_*) of tensor `tensor`, as left by the last step, to `out`
 * (DEVICE) in the canonical layout given with the selector; `bytes` must equal its size. */
apollo_status_t apollo_debug_get(apollo_handle_t* h, int32_t tensor, int32_t what, void* out,
                                 size_t bytes, void* hip_stream);

/* Generator building blocks, for bit-exact checks of the random stream.
 * apollo_debug_philox: out[4*i .. 4*i+3] (DEVICE, uint32) = Philox4x32-10 of counter
 * (ctr[4*i .. 4*i+3]) (DEVICE, uint32) under key (key0, key1), i < count.
 * apollo_debug_gauss_parts: for n = first .. first+count-1 (n < 2^24), the Box-Muller parts of
 * the 24-bit inputs: radius[i] = sqrt(-2 ln((n+1)/2^24)), cosv[i], sinv[i] = cos, sin of
 * 2 pi n / 2^24 (all DEVICE fp32, count elements each). */
apollo_status_t apollo_debug_philox(const void* ctr, uint32_t key0, uint32_t key1, void* out,
                                    int64_t count, void* hip_stream);
apollo_status_t apollo_debug_gauss_parts(uint32_t first, int64_t count, void* radius, void* cosv,
                                         void* sinv, void* hip_stream);

/* Plain device-to-device copy of `bytes` (a multiple of 16; both pointers DEVICE, 16-byte
 * aligned) by a one-thread-per-16-bytes kernel: a kernel of exactly known traffic, used to
 * calibrate hardware byte counters when profiling. */
apollo_status_t apollo_debug_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/* Which projection kernel serves tensor `tensor` (decided in apollo_init from shape, gradient type,
 * rank and side; pure host arithmetic, nothing is launched).  Writes one of APOLLO_PATH_* to *path
 * and, if `padded_copy` is not NULL, 1 there when the step first copies the gradient to rows padded
 * to 16 bytes (bf16 gradients, rows projected, odd row length).  For callers and tests that want to
 * know that a shape runs where they expect it to run. */
enum {
  APOLLO_PATH_RANK1 = 0,        /* streaming mat-vec kernels (rank 1; any row length, a tall tensor's
                                   rows up to 16384 elements)                                       */
  APOLLO_PATH_MATRIX_CORE = 1,  /* bf16 MFMA kernel (bf16 gradients, rank a multiple of 32, projected
                                   dimension a multiple of 64, at least 256 channels): Algorithm 1's
                                   steps 1-3 in one kernel -- the moment update and the channel norms
                                   follow in the epilogue, R never leaves the registers and has no
                                   scratch                                                         */
  APOLLO_PATH_GENERAL = 2,      /* fp32 FMA kernel, any shape, rank and gradient type              */
  APOLLO_PATH_NONE = 3          /* APOLLO_PROJ_IDENTITY: nothing is projected                      */
};
apollo_status_t apollo_debug_path(const apollo_handle_t* h, int32_t tensor, int32_t* path, int32_t* padded_copy);

/* Phase timing for benchmarks.  After apollo_profile_enable(h, 1) every apollo_step records
 * HIP events on its stream around its five phases: [0] P scratch fill, [1] projection R = P G,
 * [2] low-rank moments + factors, [3] limiter scalars, [4] weight update.  apollo_profile_read
 * waits for the recorded events, adds each phase's elapsed milliseconds over the steps recorded
 * since the last read into ms[0..4] (HOST, 5 floats) and their count into *n_steps, and
 * forgets them.  At most 1024 steps are kept between reads; later ones are not recorded. */
apollo_status_t apollo_profile_enable(apollo_handle_t* h, int32_t on);
apollo_status_t apollo_profile_read(apollo_handle_t* h, float* ms, int32_t* n_steps);

/* Text of the last error on this handle; with h == NULL, of the last failed call of this
 * thread that had no handle (apollo_init, the size queries, the generator checks).  The
 * string stays valid until the next call on the same handle / thread. */
const char* apollo_last_error(const apollo_handle_t* h);

/* Frees the host-side handle.  Does not touch device memory or synchronise. */
void apollo_destroy(apollo_handle_t* h);

/* ------------------------------------------------------------------------------------------
 * Element-wise AdamW for the parameters that are not projected (embeddings, norm gains, the
 * output head; the paper applies APOLLO to the attention and MLP matrices only and its step
 * times cover the whole model).  Section 3.1, Eq. 1: M <- beta1 M + (1 - beta1) G,
 * V <- beta2 V + (1 - beta2) G^2, W <- W - lr * M^ / (sqrt(V^) + eps) - lr * lambda * W, with
 * the decoupled decay term of Algorithm 1 (step 4) and Adam's bias correction M^ = M / (1 -
 * beta1^t), V^ = V / (1 - beta2^t) (bias_correction = 0: Eq. 1 literally).  One kernel launch
 * covers the whole tensor list.  Same conventions as above: DEVICE buffers owned by the
 * caller, nothing allocated, nothing synchronised, status codes, apollo_last_error(NULL) for
 * calls without a handle.
 * ------------------------------------------------------------------------------------------ */
typedef struct apollo_adamw_handle apollo_adamw_handle_t; /* opaque, host-side */

typedef struct {
  int64_t numel;        /* elements of the tensor (any shape, handled flat), 1 .. 2^40         */
  int32_t grad_dtype;   /* APOLLO_F32 or APOLLO_BF16                                           */
  int32_t store_dtype;  /* APOLLO_F32 (0, default) or APOLLO_BF16: element type of this tensor's
                           W, M and V (bfloat16: rounded to nearest even when stored, later
                           arithmetic from the stored values, as for apollo_config_t)          */
} apollo_flat_shape_t;

typedef struct {
  float beta1, beta2;       /* in [0, 1)                                                        */
  float eps;                /* >= 0, added after the bias-corrected square root                 */
  float weight_decay;       /* lambda                                                           */
  int32_t bias_correction;  /* 1 (default) or 0                                                 */
  int32_t reserved;         /* set to 0                                                         */
} apollo_adamw_config_t;

/* Bytes of state: per tensor, in list order, each block on a 256-byte boundary: M[numel],
 * V[numel] in the tensor's store_dtype (V starts on a 256-byte boundary too).  0 on invalid
 * arguments. */
size_t apollo_adamw_state_bytes(const apollo_flat_shape_t* shapes, int32_t n_tensors);

/* Byte offsets of one tensor's M and V in the state buffer (either output may be NULL). */
apollo_status_t apollo_adamw_state_offsets(const apollo_flat_shape_t* shapes, int32_t n_tensors,
                                           int32_t tensor, size_t* m_offset, size_t* v_offset);

/* Bytes of scratch (descriptor table and the block-to-tensor table of the single launch).
 * 0 on invalid arguments. */
size_t apollo_adamw_workspace_bytes(const apollo_flat_shape_t* shapes, int32_t n_tensors);

/* Creates a handle for a fixed tensor list.  `state` and `workspace` are DEVICE buffers of at
 * least the sizes above, 256-byte aligned; the state is zero-filled on `hip_stream` unless
 * `zero_state` is 0 (resume).  Blocks the host until the block table is on the device. */
apollo_status_t apollo_adamw_init(apollo_adamw_handle_t** out, const apollo_adamw_config_t* cfg,
                                  const apollo_flat_shape_t* shapes, int32_t n_tensors,
                                  void* state, size_t state_bytes, void* workspace,
                                  size_t workspace_bytes, int32_t zero_state, void* hip_stream);

/* One AdamW step of every tensor at 1-based step `step` with learning rate `lr`: tensors[k].w
 * (DEVICE, store_dtype, updated in place) and tensors[k].g (DEVICE, grad_dtype, read only), both with
 * numel elements and 16-byte aligned.  Enqueues on `hip_stream`, does not synchronise. */
apollo_status_t apollo_adamw_step(apollo_adamw_handle_t* h, const apollo_tensor_t* tensors,
                                  int32_t n_tensors, int64_t step, float lr, void* hip_stream);

/* Text of the last error on this handle; with h == NULL, of the last failed AdamW call of this
 * thread that had no handle (apollo_adamw_init, the size queries). */
const char* apollo_adamw_last_error(const apollo_adamw_handle_t* h);

/* Frees the host-side handle.  Does not touch device memory. */
void apollo_adamw_destroy(apollo_adamw_handle_t* h);

#ifdef __cplusplus
}
#endif
#endif /* APOLLO_H_ */
