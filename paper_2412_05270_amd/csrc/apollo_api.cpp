// Host side of the APOLLO step library: argument checking, buffer layout, the per-step launch
// schedule.  The interface is documented in include/apollo.h.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/apollo.h"
#include "apollo_internal.h"

using namespace apollo;

namespace {

constexpr size_t kAlign = 256;
constexpr int64_t kMaxDim = 1 << 20;       // rows / cols limit (grid dimensions, int indexing)
constexpr int32_t kMaxTensors = 65535;     // gridDim.z
constexpr int kRingSlots = 4;
constexpr size_t kMergedUpdateMaxParams = 64u << 20;   // below this many parameters the update of all groups is one launch
constexpr size_t kChunkPBytes = 128u << 20;            // APOLLO_SCHEDULE_CHUNKED: scratch for the P of one chunk of tensors

inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

thread_local std::string g_last_error;

enum class Path { kRank1, kMfma, kGeneric, kIdentity };   // kIdentity: no projection (Section 3.2)

struct TensorPlan {
  int32_t rows, cols, m, n, m8;
  int32_t r;                                                    // rows of the moments: the rank, or m without projection
  bool left, bf16;
  Path path;
  int32_t n_slabs, k2_blocks;
  bool pad_g;                                                   // projection reads a row-padded copy of g
  bool fused;                                                   // the projection kernel also updates the moments (no R scratch)
  int32_t row_tiles;                                            // its row tiles per channel tile
  int32_t ldg;                                                  // row pitch (elements) of what it reads
  size_t ws_gpad;
  size_t st_m, st_v, st_norm;                                   // offsets into the state buffer
  size_t ws_p, ws_r, ws_colsq, ws_s, ws_partials, ws_scal;       // offsets into the workspace
  int32_t desc_index;                                           // position in the grouped descriptor table
};

struct Group {
  int32_t first, count;          // range in the descriptor table
  int32_t rows, cols, m, n, m8;
  bool left, bf16;
  Path path;
  int32_t n_slabs;
  bool pad_g, fused;
  int32_t ldg, row_tiles;
  int32_t chunk;                 // APOLLO_SCHEDULE_CHUNKED: tensors whose P share the scratch at a time (else count)
};

struct Plan {
  std::vector<TensorPlan> t;
  std::vector<Group> groups;
  size_t state_bytes = 0, workspace_bytes = 0, desc_bytes = 0;
  size_t ws_step = 0;            // offset of the StepState (device copy of a step's scalars) in the workspace
};

int fail(std::string& dst, int code, const char* fmt, long long a = 0, long long b = 0, long long c = 0) {
  char buf[256];
  std::snprintf(buf, sizeof buf, fmt, a, b, c);
  dst = buf;
  return code;
}

// Validates the configuration and the shapes and lays out both buffers.  Host arithmetic only.
int make_plan(const apollo_config_t* cfg, const apollo_shape_t* shapes, int32_t n, Plan& plan, std::string& err) {
  if (!cfg || !shapes) return fail(err, APOLLO_EINVAL, "null config or shape list");
  if (n < 1 || n > kMaxTensors) return fail(err, APOLLO_EINVAL, "n_tensors %lld outside 1..65535", n);
  if (cfg->projection != APOLLO_PROJ_RANDOM && cfg->projection != APOLLO_PROJ_IDENTITY)
    return fail(err, APOLLO_EINVAL, "unknown projection %lld", cfg->projection);
  const bool identity = cfg->projection == APOLLO_PROJ_IDENTITY;
  if (!identity && cfg->rank < 1) return fail(err, APOLLO_EINVAL, "rank %lld < 1", cfg->rank);
  if (cfg->mode != APOLLO_CHANNEL && cfg->mode != APOLLO_TENSOR) return fail(err, APOLLO_EINVAL, "unknown mode %lld", cfg->mode);
  if (cfg->side < APOLLO_SIDE_AUTO || cfg->side > APOLLO_SIDE_RIGHT) return fail(err, APOLLO_EINVAL, "unknown side %lld", cfg->side);
  if (cfg->refresh_interval < 1) return fail(err, APOLLO_EINVAL, "refresh_interval %lld < 1", cfg->refresh_interval);
  if (!(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f))
    return fail(err, APOLLO_EINVAL, "betas must lie in [0, 1)");
  if (!(cfg->eps >= 0.f) || !(cfg->nl_gamma >= 0.f) || !std::isfinite(cfg->scale) || !std::isfinite(cfg->weight_decay))
    return fail(err, APOLLO_EINVAL, "eps / nl_gamma negative or scale / weight_decay not finite");
  if ((cfg->weight_dtype != APOLLO_F32 && cfg->weight_dtype != APOLLO_BF16 && cfg->weight_dtype != APOLLO_Q8) ||
      (cfg->state_dtype != APOLLO_F32 && cfg->state_dtype != APOLLO_BF16))
    return fail(err, APOLLO_EUNSUPPORTED, "weight_dtype must be fp32, bf16 or q8 and state_dtype fp32 or bf16");
  if (cfg->weight_rounding != APOLLO_ROUND_NEAREST && cfg->weight_rounding != APOLLO_ROUND_STOCHASTIC)
    return fail(err, APOLLO_EINVAL, "unknown weight_rounding %lld", cfg->weight_rounding);
  if (cfg->schedule != APOLLO_SCHEDULE_OVERLAP && cfg->schedule != APOLLO_SCHEDULE_SERIAL && cfg->schedule != APOLLO_SCHEDULE_CHUNKED)
    return fail(err, APOLLO_EINVAL, "unknown schedule %lld", cfg->schedule);
  const bool chunked = cfg->schedule == APOLLO_SCHEDULE_CHUNKED;
  const size_t state_elem = cfg->state_dtype == APOLLO_BF16 ? 2 : sizeof(float);

  plan.t.resize(n);
  size_t st = 0;
  for (int32_t k = 0; k < n; ++k) {
    const apollo_shape_t& s = shapes[k];
    TensorPlan& t = plan.t[k];
    if (s.rows < 1 || s.cols < 1) return fail(err, APOLLO_EINVAL, "tensor %lld: rows/cols must be >= 1", k);
    if (s.grad_dtype != APOLLO_F32 && s.grad_dtype != APOLLO_BF16)
      return fail(err, APOLLO_EUNSUPPORTED, "tensor %lld: gradient dtype %lld is neither fp32 nor bf16", k, s.grad_dtype);
    if (s.rows > kMaxDim || s.cols > kMaxDim)
      return fail(err, APOLLO_EUNSUPPORTED, "tensor %lld: dimension above %lld", k, kMaxDim);
    if (s.rows * s.cols >= (1ll << 31))
      return fail(err, APOLLO_EUNSUPPORTED, "tensor %lld: more than 2^31 - 1 elements", k);
    if (cfg->weight_dtype == APOLLO_Q8 && (s.cols % 128) != 0)
      return fail(err, APOLLO_EUNSUPPORTED, "tensor %lld: 8-bit weights need a row length that is a multiple of 128", k);
    t.rows = (int32_t)s.rows;
    t.cols = (int32_t)s.cols;
    t.bf16 = s.grad_dtype == APOLLO_BF16;
    t.left = cfg->side == APOLLO_SIDE_LEFT || (cfg->side == APOLLO_SIDE_AUTO && s.rows <= s.cols);
    t.m = t.left ? t.rows : t.cols;
    t.n = t.left ? t.cols : t.rows;
    t.m8 = (t.m + 7) & ~7;
    if (!identity && cfg->rank > t.m)
      return fail(err, APOLLO_EINVAL, "tensor %lld: rank %lld exceeds the projected dimension %lld", k, cfg->rank, t.m);
    t.r = identity ? t.m : cfg->rank;
    if (identity)
      t.path = Path::kIdentity;
    else if (cfg->rank == 1 && project_rank1_supported(t.rows, t.cols, t.left, t.bf16))
      t.path = Path::kRank1;
    else if (project_mfma_supported(t.rows, t.cols, t.left, t.bf16, cfg->rank))
      t.path = Path::kMfma;
    else
      t.path = Path::kGeneric;
    t.pad_g = t.path == Path::kMfma && project_mfma_needs_padding(t.rows, t.cols, t.left);
    t.fused = t.path == Path::kMfma;
    t.row_tiles = t.fused ? project_mfma_row_tiles(cfg->rank) : 1;
    t.ldg = t.pad_g ? (t.cols + 7) & ~7 : t.cols;
    t.n_slabs = 1;
    if (t.path == Path::kRank1 && t.left) {
      int32_t sl = (t.rows + 511) / 512;
      if (sl > 16) sl = 16;
      if ((t.rows + sl - 1) / sl > 1020) sl = (t.rows + 1019) / 1020;
      t.n_slabs = sl;
    }
    t.k2_blocks = adam_norms_blocks(t.n);                                 // blocks that leave four partial sums each
    if (identity && !t.left) t.k2_blocks = (t.n + 3) / 4;                 // of adam_identity_rows_kernel
    if (t.fused) t.k2_blocks = project_mfma_tiles(t.n);                   // of the fused projection kernel
    const size_t rn = (size_t)t.r * (size_t)t.n * state_elem;
    st = align_up(st);
    t.st_m = st;
    t.st_v = st + rn;
    t.st_norm = st + 2 * rn;
    st = t.st_norm + sizeof(float);
  }
  plan.state_bytes = align_up(st);

  // group tensors of identical shape / dtype (orientation and path follow from those)
  std::vector<int32_t> group_of(n, -1);
  for (int32_t k = 0; k < n; ++k) {
    if (group_of[k] >= 0) continue;
    const TensorPlan& a = plan.t[k];
    Group g{};
    g.rows = a.rows; g.cols = a.cols; g.m = a.m; g.n = a.n; g.m8 = a.m8;
    g.left = a.left; g.bf16 = a.bf16; g.path = a.path; g.n_slabs = a.n_slabs; g.pad_g = a.pad_g; g.fused = a.fused; g.row_tiles = a.row_tiles; g.ldg = a.ldg;
    g.count = 0;
    g.chunk = 0;
    const int32_t gi = (int32_t)plan.groups.size();
    for (int32_t j = k; j < n; ++j) {
      const TensorPlan& b = plan.t[j];
      if (group_of[j] < 0 && b.rows == a.rows && b.cols == a.cols && b.bf16 == a.bf16) {
        group_of[j] = gi;
        ++g.count;
      }
    }
    plan.groups.push_back(g);
  }
  int32_t pos = 0;
  for (size_t gi = 0; gi < plan.groups.size(); ++gi) {
    plan.groups[gi].first = pos;
    for (int32_t k = 0; k < n; ++k)
      if (group_of[k] == (int32_t)gi) plan.t[k].desc_index = pos++;
  }

  // workspace: descriptor table, then per tensor P, padded gradient copy, R, colsq, s, partials, scalars
  size_t ws = 0;
  plan.desc_bytes = (size_t)n * sizeof(TensorDesc);
  ws = align_up(plan.desc_bytes);
  plan.ws_step = ws;
  ws = align_up(ws + sizeof(StepState));
  for (int32_t k = 0; k < n; ++k) {
    TensorPlan& t = plan.t[k];
    t.ws_p = ws;
    if (!chunked && t.path != Path::kRank1 && t.path != Path::kIdentity) ws = align_up(ws + (size_t)cfg->rank * t.m8 * (t.bf16 ? 2 : 4));
    t.ws_gpad = ws;
    if (t.pad_g) ws = align_up(ws + (size_t)t.rows * t.ldg * 2);
    t.ws_r = ws;
    if (t.fused) {     // no R; with several row tiles per channel tile their channel sums
      if (t.row_tiles > 1) ws = align_up(ws + (size_t)t.row_tiles * 2 * t.n * sizeof(float));
    } else if (t.path != Path::kIdentity) {
      ws = align_up(ws + (size_t)t.n_slabs * cfg->rank * t.n * sizeof(float));
    }
    t.ws_colsq = ws;
    ws = align_up(ws + (size_t)t.n_slabs * t.n * sizeof(float));
    t.ws_s = ws;
    ws = align_up(ws + (size_t)t.n * sizeof(float));
    t.ws_partials = ws;
    ws = align_up(ws + (size_t)t.k2_blocks * 4 * sizeof(float));
    t.ws_scal = ws;
    ws = align_up(ws + 8 * sizeof(float));
  }
  // P scratch of the chunked schedule: one region, used by one chunk of a group's tensors at a time
  for (Group& g : plan.groups) g.chunk = g.count;
  if (chunked) {
    const size_t region = ws;
    size_t region_bytes = 0;
    for (Group& g : plan.groups) {
      if (g.path == Path::kRank1 || g.path == Path::kIdentity) continue;
      const size_t pb = align_up((size_t)cfg->rank * g.m8 * (g.bf16 ? 2 : 4));
      g.chunk = (int32_t)std::max<size_t>(1, std::min<size_t>((size_t)g.count, kChunkPBytes / pb));
      region_bytes = std::max(region_bytes, (size_t)g.chunk * pb);
    }
    for (int32_t k = 0; k < n; ++k) {
      TensorPlan& t = plan.t[k];
      const Group& g = plan.groups[group_of[k]];
      if (g.path == Path::kRank1 || g.path == Path::kIdentity) continue;
      const size_t pb = align_up((size_t)cfg->rank * g.m8 * (g.bf16 ? 2 : 4));
      t.ws_p = region + (size_t)((t.desc_index - g.first) % g.chunk) * pb;
    }
    ws = align_up(ws + region_bytes);
  }
  plan.workspace_bytes = ws;
  return APOLLO_OK;
}

}  // namespace

struct apollo_handle {
  apollo_config_t cfg;
  Plan plan;
  char* state = nullptr;
  char* ws = nullptr;
  std::vector<TensorDesc> desc;           // host copy, descriptor-table order
  std::vector<apollo_tensor_t> last;      // pointers of the previous step, caller order
  TensorDesc* ring[kRingSlots] = {nullptr, nullptr, nullptr, nullptr};   // pinned staging copies
  hipEvent_t ring_ev[kRingSlots] = {nullptr, nullptr, nullptr, nullptr};
  bool ring_used[kRingSlots] = {false, false, false, false};
  int ring_next = 0;
  bool have_ptrs = false;
  int64_t p_epoch = -1;                   // refresh epoch whose P the workspace scratch holds (-1: none)
  hipStream_t p_stream = nullptr;         // stream on which that P was written
  bool profiling = false;
  hipStream_t side = nullptr;             // second stream of the overlapped schedule (created at init)
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  std::vector<hipEvent_t> ev_proj;        // one per group: its projection has finished
  bool overlap = false;                   // the overlapped schedule applies to this tensor list
  std::vector<hipEvent_t> prof_events;    // 6 per recorded step
  size_t prof_used = 0;                   // events recorded since the last read
  std::string err;
};

namespace {

int hip_fail(std::string& dst, hipError_t e, const char* what) {
  dst = std::string(what) + ": " + hipGetErrorString(e);
  return APOLLO_EHIP;
}

StepParams make_step_params(const apollo_config_t& c, int64_t step, float lr) {
  StepParams sp{};
  sp.ks = philox_key_schedule(c.seed);
  sp.epoch = (uint32_t)(((uint64_t)(step - 1) / (uint64_t)c.refresh_interval) & 0xffffffffu);
  sp.r = c.rank;
  sp.tensor_mode = c.mode == APOLLO_TENSOR;
  sp.rsqrt_r = c.rank > 0 ? (float)(1.0 / std::sqrt((double)c.rank)) : 1.0f;
  sp.beta1 = c.beta1;
  sp.beta2 = c.beta2;
  sp.omb1 = 1.0f - c.beta1;
  sp.omb2 = 1.0f - c.beta2;
  sp.eps = c.eps;
  if (c.bias_correction) {
    sp.inv_bc1 = (float)(1.0 / (1.0 - std::pow((double)c.beta1, (double)step)));
    sp.inv_bc2 = (float)(1.0 / (1.0 - std::pow((double)c.beta2, (double)step)));
  } else {
    sp.inv_bc1 = sp.inv_bc2 = 1.0f;
  }
  sp.alpha = c.scale;
  sp.gamma = c.nl_gamma;
  sp.lr = lr;
  sp.lr_decay = lr * c.weight_decay;
  sp.step_lo = (uint32_t)((uint64_t)step & 0xffffffffu);
  sp.q8_stochastic = c.weight_rounding == APOLLO_ROUND_STOCHASTIC;
  return sp;
}

// Copies the host descriptor table to the device through a pinned staging slot.
int upload_descs(apollo_handle* h, hipStream_t st) {
  const int slot = h->ring_next;
  h->ring_next = (slot + 1) % kRingSlots;
  hipError_t e;
  if (h->ring_used[slot]) {
    e = hipEventSynchronize(h->ring_ev[slot]);
    if (e != hipSuccess) return hip_fail(h->err, e, "hipEventSynchronize");
  }
  std::memcpy(h->ring[slot], h->desc.data(), h->plan.desc_bytes);
  e = hipMemcpyAsync(h->ws, h->ring[slot], h->plan.desc_bytes, hipMemcpyHostToDevice, st);
  if (e != hipSuccess) return hip_fail(h->err, e, "hipMemcpyAsync(descriptor table)");
  e = hipEventRecord(h->ring_ev[slot], st);
  if (e != hipSuccess) return hip_fail(h->err, e, "hipEventRecord");
  h->ring_used[slot] = true;
  return APOLLO_OK;
}

// The launches of one shape group, phase by phase; `what` names the last one for error texts.
struct GroupLaunches {
  const apollo_config_t& cfg;
  const TensorDesc* dd;        // DEVICE descriptor table
  StepArgs sa;                 // the step's scalars: by value, or in device memory (replayable step)
  bool regenerate;             // launch the kernel that writes the scratch copy of P before projecting
  const char* what;

  // the transient copy of P (and of a gradient whose rows need padding) for the groups that read it from scratch
  hipError_t fill(const Group& g, hipStream_t s) {
    if (g.path == Path::kRank1 || g.path == Path::kIdentity) return hipSuccess;
    what = "projection fill";
    hipError_t r = regenerate ? launch_fill_projection(dd + g.first, g.count, sa.host.r, g.m8, g.bf16, sa, s) : hipSuccess;
    if (r == hipSuccess && g.pad_g) {
      what = "gradient padding";
      r = launch_pad_gradient(dd + g.first, g.count, g.rows, g.cols, g.ldg, s);
    }
    return r;
  }
  // R = P G and the per-channel squared norms of G
  hipError_t project(const Group& g, hipStream_t s) {
    what = "projection";
    if (g.path == Path::kIdentity) return hipSuccess;
    if (g.path == Path::kRank1)
      return launch_project_rank1(dd + g.first, g.count, g.rows, g.cols, g.left, g.bf16, g.n_slabs, sa, s);
    if (g.path == Path::kMfma)     // (fused: Algorithm 1's steps 1-3 in one kernel, see moments())
      return launch_project_mfma(dd + g.first, g.count, g.rows, g.cols, g.left, g.pad_g, g.fused,
                                 cfg.state_dtype == APOLLO_BF16, nullptr, sa, s);
    return launch_project_generic(dd + g.first, g.count, g.n, g.bf16, sa, s);
  }
  // low-rank Adam moments, channel factors, block partial sums
  hipError_t moments(const Group& g, hipStream_t s) {
    what = "moment update";
    if (g.fused)                         // done in the projection kernel's epilogue, up to the sum over its row tiles
      return g.row_tiles > 1 ? launch_channel_factors(dd + g.first, g.count, g.n, g.row_tiles, s) : hipSuccess;
    const bool state_bf16 = cfg.state_dtype == APOLLO_BF16;
    if (g.path == Path::kIdentity)
      return launch_adam_identity(dd + g.first, g.count, g.rows, g.cols, g.left, g.bf16, state_bf16, sa, s);
    return launch_adam_norms(dd + g.first, g.count, g.n, state_bf16, sa, s);
  }
  hipError_t update(const Group& g, hipStream_t s) {
    what = "weight update";
    if (cfg.weight_dtype == APOLLO_Q8)
      return launch_update_q8(dd + g.first, g.count, g.rows, g.cols, g.left, g.bf16, sa, s);
    return launch_update(dd + g.first, g.count, g.rows, g.cols, g.left, g.bf16, cfg.weight_dtype == APOLLO_BF16, sa, s);
  }
};

// Fills the descriptor of tensor k (descriptor-table order is the plan's) from the plan and the two buffers.
void fill_desc(TensorDesc& d, const TensorPlan& t, int32_t k, char* state, char* ws) {
  std::memset(&d, 0, sizeof d);
  d.M = state + t.st_m;
  d.V = state + t.st_v;
  d.prev_norm = reinterpret_cast<float*>(state + t.st_norm);
  d.P = (t.path == Path::kRank1 || t.path == Path::kIdentity) ? nullptr : static_cast<void*>(ws + t.ws_p);
  d.gpad = t.pad_g ? static_cast<void*>(ws + t.ws_gpad) : nullptr;
  d.ldg = t.ldg;
  d.R = (t.path == Path::kIdentity || (t.fused && t.row_tiles == 1)) ? nullptr : reinterpret_cast<float*>(ws + t.ws_r);
  d.colsq = reinterpret_cast<float*>(ws + t.ws_colsq);
  d.s = reinterpret_cast<float*>(ws + t.ws_s);
  d.partials = reinterpret_cast<float*>(ws + t.ws_partials);
  d.scal = reinterpret_cast<float*>(ws + t.ws_scal);
  d.rows = t.rows; d.cols = t.cols; d.m = t.m; d.n = t.n; d.m8 = t.m8;
  d.left = t.left; d.tensor_id = k; d.n_slabs = t.n_slabs; d.k2_blocks = t.k2_blocks;
}

// Serial schedule of one step, phase by phase, every shape group in turn (the one that is timed
// phase by phase when profiling: pev, if not null, are the six events around the five phases, the
// first already recorded).
hipError_t run_serial(GroupLaunches& L, const Plan& plan, hipStream_t st, hipEvent_t* pev) {
  hipError_t e = hipSuccess;
  for (const Group& g : plan.groups) {
    if (e != hipSuccess) break;
    e = L.fill(g, st);
  }
  if (pev && e == hipSuccess) e = hipEventRecord(pev[1], st);
  // the matrix-core groups share one launch (a small set then fills the chip at once, a large one has
  // a single tail); the others are launched group by group
  std::vector<MfmaGroupShape> mfma;
  for (const Group& g : plan.groups) {
    if (e != hipSuccess) break;
    if (g.path == Path::kMfma) mfma.push_back(MfmaGroupShape{g.first, g.count, g.rows, g.cols, g.left, g.pad_g});
    else e = L.project(g, st);
  }
  if (e == hipSuccess && !mfma.empty()) {
    L.what = "projection";
    e = launch_project_mfma_groups(L.dd, mfma.data(), (int)mfma.size(), true, L.cfg.state_dtype == APOLLO_BF16, nullptr,
                                   L.sa, st);
  }
  if (pev && e == hipSuccess) e = hipEventRecord(pev[2], st);
  for (const Group& g : plan.groups) {
    if (e != hipSuccess) break;
    e = L.moments(g, st);
  }
  if (pev && e == hipSuccess) e = hipEventRecord(pev[3], st);
  // per-tensor factor, norm and limiter, all tensors in one launch
  if (e == hipSuccess) {
    L.what = "limiter";
    e = launch_finalize(L.dd, (int)plan.t.size(), L.sa, st);
  }
  if (pev && e == hipSuccess) e = hipEventRecord(pev[4], st);
  // A small set (bound by launch latency, and its per-group launches do not fill the chip) updates all
  // groups of one gradient type in one launch; a large one group by group (the same arithmetic either way).
  size_t params = 0;
  for (const TensorPlan& t : plan.t) params += (size_t)t.rows * t.cols;
  const bool merged = params < kMergedUpdateMaxParams && L.cfg.weight_dtype != APOLLO_Q8 && plan.groups.size() > 1;
  if (merged) {
    for (int pass = 0; pass < 2 && e == hipSuccess; ++pass) {       // bf16 gradients, then fp32 gradients
      std::vector<UpdateGroupShape> ug;
      for (const Group& g : plan.groups)
        if (g.bf16 == (pass == 0)) ug.push_back(UpdateGroupShape{g.first, g.count, g.rows, g.cols, g.left});
      if (ug.empty()) continue;
      L.what = "weight update";
      e = launch_update_groups(L.dd, ug.data(), (int)ug.size(), pass == 0, L.cfg.weight_dtype == APOLLO_BF16, L.sa, st);
    }
  } else {
    for (const Group& g : plan.groups) {
      if (e != hipSuccess) break;
      e = L.update(g, st);
    }
  }
  if (pev && e == hipSuccess) e = hipEventRecord(pev[5], st);
  return e;
}

// APOLLO_SCHEDULE_CHUNKED: as run_serial, but P is generated anew in every step, chunk by chunk of a
// group's tensors over one scratch region, each chunk projected before the next one overwrites it.
hipError_t run_chunked(GroupLaunches& L, const Plan& plan, hipStream_t st, hipEvent_t* pev) {
  hipError_t e = hipSuccess;
  if (pev) e = hipEventRecord(pev[1], st);      // (generation and projection alternate: both count as projection)
  const bool state_bf16 = L.cfg.state_dtype == APOLLO_BF16;
  for (const Group& g : plan.groups) {
    if (e != hipSuccess) break;
    if (g.path == Path::kRank1 || g.path == Path::kIdentity) {
      e = L.project(g, st);
      continue;
    }
    if (g.pad_g) {
      L.what = "gradient padding";
      e = launch_pad_gradient(L.dd + g.first, g.count, g.rows, g.cols, g.ldg, st);
    }
    for (int32_t c0 = 0; c0 < g.count && e == hipSuccess; c0 += g.chunk) {
      const int32_t cnt = std::min(g.chunk, g.count - c0);
      const TensorDesc* d0 = L.dd + g.first + c0;
      L.what = "projection fill";
      e = launch_fill_projection(d0, cnt, L.sa.host.r, g.m8, g.bf16, L.sa, st);
      if (e != hipSuccess) break;
      L.what = "projection";
      e = g.path == Path::kMfma ? launch_project_mfma(d0, cnt, g.rows, g.cols, g.left, g.pad_g, g.fused, state_bf16, nullptr, L.sa, st)
                                : launch_project_generic(d0, cnt, g.n, g.bf16, L.sa, st);
    }
  }
  if (pev && e == hipSuccess) e = hipEventRecord(pev[2], st);
  for (const Group& g : plan.groups) {
    if (e != hipSuccess) break;
    e = L.moments(g, st);
  }
  if (pev && e == hipSuccess) e = hipEventRecord(pev[3], st);
  if (e == hipSuccess) {
    L.what = "limiter";
    e = launch_finalize(L.dd, (int)plan.t.size(), L.sa, st);
  }
  if (pev && e == hipSuccess) e = hipEventRecord(pev[4], st);
  for (const Group& g : plan.groups) {
    if (e != hipSuccess) break;
    e = L.update(g, st);
  }
  if (pev && e == hipSuccess) e = hipEventRecord(pev[5], st);
  return e;
}

}  // namespace

extern "C" {

size_t apollo_state_bytes(const apollo_config_t* cfg, const apollo_shape_t* shapes, int32_t n_tensors) {
  Plan p;
  if (make_plan(cfg, shapes, n_tensors, p, g_last_error) != APOLLO_OK) return 0;
  return p.state_bytes;
}

size_t apollo_workspace_bytes(const apollo_config_t* cfg, const apollo_shape_t* shapes, int32_t n_tensors) {
  Plan p;
  if (make_plan(cfg, shapes, n_tensors, p, g_last_error) != APOLLO_OK) return 0;
  return p.workspace_bytes;
}

apollo_status_t apollo_state_offsets(const apollo_config_t* cfg, const apollo_shape_t* shapes, int32_t n_tensors,
                                     int32_t tensor, size_t* m_offset, size_t* v_offset, size_t* norm_offset) {
  Plan p;
  const int rc = make_plan(cfg, shapes, n_tensors, p, g_last_error);
  if (rc != APOLLO_OK) return rc;
  if (tensor < 0 || tensor >= n_tensors) return fail(g_last_error, APOLLO_EINVAL, "tensor index %lld out of range", tensor);
  if (m_offset) *m_offset = p.t[tensor].st_m;
  if (v_offset) *v_offset = p.t[tensor].st_v;
  if (norm_offset) *norm_offset = p.t[tensor].st_norm;
  return APOLLO_OK;
}

apollo_status_t apollo_init(apollo_handle_t** out, const apollo_config_t* cfg, const apollo_shape_t* shapes,
                            int32_t n_tensors, void* state, size_t state_bytes, void* workspace,
                            size_t workspace_bytes, int32_t zero_state, void* hip_stream) {
  if (!out) return fail(g_last_error, APOLLO_EINVAL, "null output handle pointer");
  *out = nullptr;
  apollo_handle* h = new (std::nothrow) apollo_handle();
  if (!h) return fail(g_last_error, APOLLO_ENOMEM, "out of host memory");
  int rc = make_plan(cfg, shapes, n_tensors, h->plan, g_last_error);
  if (rc == APOLLO_OK && (!state || !workspace)) rc = fail(g_last_error, APOLLO_EINVAL, "null state or workspace buffer");
  if (rc == APOLLO_OK && (((uintptr_t)state | (uintptr_t)workspace) & (kAlign - 1)))
    rc = fail(g_last_error, APOLLO_ESTATE, "state / workspace not 256-byte aligned");
  if (rc == APOLLO_OK && state_bytes < h->plan.state_bytes)
    rc = fail(g_last_error, APOLLO_ESTATE, "state buffer has %lld bytes, %lld needed", (long long)state_bytes,
              (long long)h->plan.state_bytes);
  if (rc == APOLLO_OK && workspace_bytes < h->plan.workspace_bytes)
    rc = fail(g_last_error, APOLLO_ESTATE, "workspace has %lld bytes, %lld needed", (long long)workspace_bytes,
              (long long)h->plan.workspace_bytes);
  if (rc != APOLLO_OK) {
    delete h;
    return rc;
  }
  h->cfg = *cfg;
  h->state = static_cast<char*>(state);
  h->ws = static_cast<char*>(workspace);
  h->desc.resize(n_tensors);
  h->last.assign(n_tensors, apollo_tensor_t{nullptr, nullptr, nullptr});
  for (int32_t k = 0; k < n_tensors; ++k) {
    const TensorPlan& t = h->plan.t[k];
    fill_desc(h->desc[t.desc_index], t, k, h->state, h->ws);
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e = hipSuccess;
  for (int i = 0; i < kRingSlots && e == hipSuccess; ++i) {
    e = hipHostMalloc(reinterpret_cast<void**>(&h->ring[i]), h->plan.desc_bytes, hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&h->ring_ev[i], hipEventDisableTiming);
  }
  // Overlapped schedule (see apollo_step): only where a projection runs on the matrix cores, i.e.
  // leaves HBM bandwidth unused that another group's streaming kernels can take.
  h->overlap = cfg->schedule == APOLLO_SCHEDULE_OVERLAP && h->plan.groups.size() > 1;
  if (h->overlap) {
    bool any_mfma = false;
    for (const Group& g : h->plan.groups) any_mfma = any_mfma || g.path == Path::kMfma;
    h->overlap = any_mfma;
  }
  if (e == hipSuccess && h->overlap) {
    e = hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking);       // default priority
    if (e == hipSuccess) e = hipEventCreateWithFlags(&h->ev_fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&h->ev_join, hipEventDisableTiming);
    h->ev_proj.assign(h->plan.groups.size(), nullptr);
    for (size_t i = 0; i < h->ev_proj.size() && e == hipSuccess; ++i)
      e = hipEventCreateWithFlags(&h->ev_proj[i], hipEventDisableTiming);
  }
  if (e == hipSuccess && zero_state) e = launch_fill_zero(h->state, h->plan.state_bytes, st);
  // the device copy of the step scalars starts with "the scratch holds no P"
  if (e == hipSuccess)
    e = launch_set_step(reinterpret_cast<StepState*>(h->ws + h->plan.ws_step), make_step_params(*cfg, 1, 0.f), false, true, st);
  if (e != hipSuccess) {
    hip_fail(g_last_error, e, "apollo_init");
    apollo_destroy(h);
    return APOLLO_EHIP;
  }
  *out = h;
  return APOLLO_OK;
}

apollo_status_t apollo_step(apollo_handle_t* h, const apollo_tensor_t* tensors, int32_t n_tensors, int64_t step,
                            float lr, void* hip_stream) {
  if (!h) return fail(g_last_error, APOLLO_EINVAL, "null handle");
  const int32_t n = (int32_t)h->plan.t.size();
  if (!tensors) return fail(h->err, APOLLO_EINVAL, "null tensor list");
  if (n_tensors != n) return fail(h->err, APOLLO_EINVAL, "n_tensors %lld differs from the %lld given to apollo_init", n_tensors, n);
  if (step < 1) return fail(h->err, APOLLO_EINVAL, "step %lld < 1 (steps are 1-based)", step);
  if (!std::isfinite(lr)) return fail(h->err, APOLLO_EINVAL, "learning rate is not finite");
  bool changed = !h->have_ptrs;
  for (int32_t k = 0; k < n; ++k) {
    if (!tensors[k].w || !tensors[k].g) return fail(h->err, APOLLO_EINVAL, "tensor %lld: null w or g", k);
    if (((uintptr_t)tensors[k].w | (uintptr_t)tensors[k].g) & 15u)
      return fail(h->err, APOLLO_EINVAL, "tensor %lld: w / g not 16-byte aligned", k);
    if (h->cfg.weight_dtype == APOLLO_Q8 && (!tensors[k].w_meta || ((uintptr_t)tensors[k].w_meta & 7u)))
      return fail(h->err, APOLLO_EINVAL, "tensor %lld: w_meta null or not 8-byte aligned", k);
    if (tensors[k].w != h->last[k].w || tensors[k].g != h->last[k].g || tensors[k].w_meta != h->last[k].w_meta) changed = true;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (changed) {
    for (int32_t k = 0; k < n; ++k) {
      TensorDesc& d = h->desc[h->plan.t[k].desc_index];
      d.w = tensors[k].w;
      d.w_meta = static_cast<float*>(tensors[k].w_meta);
      d.g = tensors[k].g;
      h->last[k] = tensors[k];
    }
    const int rc = upload_descs(h, st);
    if (rc != APOLLO_OK) return rc;
    h->have_ptrs = true;
  }
  const StepParams sp = make_step_params(h->cfg, step, lr);
  const TensorDesc* dd = reinterpret_cast<const TensorDesc*>(h->ws);
  hipError_t e = hipSuccess;
  hipEvent_t* pev = nullptr;              // six events around the five phases, when profiling
  if (h->profiling && h->prof_used + 6 <= 6 * 1024) {
    while (h->prof_events.size() < h->prof_used + 6 && e == hipSuccess) {
      hipEvent_t ev;
      e = hipEventCreate(&ev);
      if (e == hipSuccess) h->prof_events.push_back(ev);
    }
    if (e != hipSuccess) return hip_fail(h->err, e, "hipEventCreate");
    pev = h->prof_events.data() + h->prof_used;
    h->prof_used += 6;
    e = hipEventRecord(pev[0], st);
  }
  // Algorithm 1 keeps P_t until the next re-sampling.  So does the scratch copy: it is generated
  // when the step's refresh epoch differs from the one the workspace holds (first step, every T
  // steps, after a jump in the step number) or when the caller switched streams (the copy was
  // written in the other stream's order); otherwise the step reads what is there.
  const int64_t epoch = (step - 1) / (int64_t)h->cfg.refresh_interval;
  const bool chunked = h->cfg.schedule == APOLLO_SCHEDULE_CHUNKED;       // the scratch never holds a whole step's P
  const bool regenerate = chunked || epoch != h->p_epoch || st != h->p_stream;
  h->p_epoch = -1;                      // until this step is enqueued completely
  GroupLaunches L{h->cfg, dd, StepArgs{sp, nullptr}, regenerate, ""};
  const char*& what = L.what;
  if (regenerate && e == hipSuccess) {
    // the ordinary step keeps its books on the host; the device-side books of the replayable step
    // (apollo_step_launch) must not believe in a P that this step is about to replace
    what = "step state";
    e = launch_set_step(reinterpret_cast<StepState*>(h->ws + h->plan.ws_step), sp, false, true, st);
  }
  auto fill = [&](const Group& g, hipStream_t s) { return L.fill(g, s); };
  auto project = [&](const Group& g, hipStream_t s) { return L.project(g, s); };
  auto moments = [&](const Group& g, hipStream_t s) { return L.moments(g, s); };
  auto update = [&](const Group& g, hipStream_t s) { return L.update(g, s); };

  if (h->overlap && !pev) {
    // Overlapped schedule.  Each shape group is a chain fill -> projection -> moments -> limiter ->
    // update that touches only its own tensors and scratch; chains alternate between the caller's
    // stream and the library's second stream, and a projection waits for the previous group's
    // projection.  So the matrix-core projection of one group, which leaves more than half of the
    // HBM bandwidth unused, runs while the streaming kernels (moments, update) of the group before
    // it use that bandwidth.  The second stream starts after everything queued on the caller's
    // stream so far and is joined back before the call returns: to the caller the step is ordinary
    // work on its stream.
    hipStream_t streams[2] = {st, h->side};
    e = hipEventRecord(h->ev_fork, st);
    if (e == hipSuccess) e = hipStreamWaitEvent(h->side, h->ev_fork, 0);
    what = "stream fork";
    for (size_t gi = 0; gi < h->plan.groups.size() && e == hipSuccess; ++gi) {
      const Group& g = h->plan.groups[gi];
      hipStream_t s = streams[gi & 1];
      if (gi > 0) e = hipStreamWaitEvent(s, h->ev_proj[gi - 1], 0);
      if (e == hipSuccess) e = fill(g, s);
      if (e == hipSuccess) e = project(g, s);
      if (e == hipSuccess) e = hipEventRecord(h->ev_proj[gi], s);
      if (e == hipSuccess) e = moments(g, s);
      if (e == hipSuccess) {
        what = "limiter";
        e = launch_finalize(dd + g.first, g.count, L.sa, s);
      }
      if (e == hipSuccess) e = update(g, s);
    }
    // join even after a failed launch, so that the second stream never runs ahead of the caller's
    hipError_t ej = hipEventRecord(h->ev_join, h->side);
    if (ej == hipSuccess) ej = hipStreamWaitEvent(st, h->ev_join, 0);
    if (e == hipSuccess && ej != hipSuccess) {
      e = ej;
      what = "stream join";
    }
    if (e != hipSuccess) return hip_fail(h->err, e, what);
    h->p_epoch = epoch;
    h->p_stream = st;
    return APOLLO_OK;
  }

  if (e == hipSuccess) e = chunked ? run_chunked(L, h->plan, st, pev) : run_serial(L, h->plan, st, pev);
  if (e != hipSuccess) return hip_fail(h->err, e, what);
  h->p_epoch = epoch;
  h->p_stream = st;
  return APOLLO_OK;
}

apollo_status_t apollo_step_prepare(apollo_handle_t* h, int64_t step, float lr, void* hip_stream) {
  if (!h) return fail(g_last_error, APOLLO_EINVAL, "null handle");
  if (step < 1) return fail(h->err, APOLLO_EINVAL, "step %lld < 1 (steps are 1-based)", step);
  if (!std::isfinite(lr)) return fail(h->err, APOLLO_EINVAL, "learning rate is not finite");
  const hipError_t e = launch_set_step(reinterpret_cast<StepState*>(h->ws + h->plan.ws_step), make_step_params(h->cfg, step, lr),
                                       false, false, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return hip_fail(h->err, e, "step state");
  return APOLLO_OK;
}

apollo_status_t apollo_step_launch(apollo_handle_t* h, const apollo_tensor_t* tensors, int32_t n_tensors, void* hip_stream) {
  if (!h) return fail(g_last_error, APOLLO_EINVAL, "null handle");
  if (h->cfg.schedule == APOLLO_SCHEDULE_CHUNKED)
    return fail(h->err, APOLLO_EUNSUPPORTED, "the replayable step is not offered with APOLLO_SCHEDULE_CHUNKED");
  const int32_t n = (int32_t)h->plan.t.size();
  if (!tensors) return fail(h->err, APOLLO_EINVAL, "null tensor list");
  if (n_tensors != n) return fail(h->err, APOLLO_EINVAL, "n_tensors %lld differs from the %lld given to apollo_init", n_tensors, n);
  bool changed = !h->have_ptrs;
  for (int32_t k = 0; k < n; ++k) {
    if (!tensors[k].w || !tensors[k].g) return fail(h->err, APOLLO_EINVAL, "tensor %lld: null w or g", k);
    if (((uintptr_t)tensors[k].w | (uintptr_t)tensors[k].g) & 15u)
      return fail(h->err, APOLLO_EINVAL, "tensor %lld: w / g not 16-byte aligned", k);
    if (h->cfg.weight_dtype == APOLLO_Q8 && (!tensors[k].w_meta || ((uintptr_t)tensors[k].w_meta & 7u)))
      return fail(h->err, APOLLO_EINVAL, "tensor %lld: w_meta null or not 8-byte aligned", k);
    if (tensors[k].w != h->last[k].w || tensors[k].g != h->last[k].g || tensors[k].w_meta != h->last[k].w_meta) changed = true;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (changed) {       // (a copy request: not what a stream under capture should see -- see the header)
    for (int32_t k = 0; k < n; ++k) {
      TensorDesc& d = h->desc[h->plan.t[k].desc_index];
      d.w = tensors[k].w;
      d.w_meta = static_cast<float*>(tensors[k].w_meta);
      d.g = tensors[k].g;
      h->last[k] = tensors[k];
    }
    const int rc = upload_descs(h, st);
    if (rc != APOLLO_OK) return rc;
    h->have_ptrs = true;
  }
  // The kernels read the step's scalars from device memory; what the host passes by value only shapes
  // the launches (rank, mode).  The kernel that writes P is always launched and decides on the device
  // (it returns at once unless apollo_step_prepare found the scratch to hold another epoch's P).
  h->p_epoch = -1;     // the host no longer knows which P the scratch holds: the next apollo_step writes it again
  const TensorDesc* dd = reinterpret_cast<const TensorDesc*>(h->ws);
  GroupLaunches L{h->cfg, dd, StepArgs{make_step_params(h->cfg, 1, 0.f), reinterpret_cast<StepState*>(h->ws + h->plan.ws_step)},
                  true, ""};
  const hipError_t e = run_serial(L, h->plan, st, nullptr);
  if (e != hipSuccess) return hip_fail(h->err, e, L.what);
  return APOLLO_OK;
}

apollo_status_t apollo_debug_path(const apollo_handle_t* h, int32_t tensor, int32_t* path, int32_t* padded_copy) {
  if (!h) return fail(g_last_error, APOLLO_EINVAL, "null handle");
  if (tensor < 0 || tensor >= (int32_t)h->plan.t.size() || !path) return APOLLO_EINVAL;
  const TensorPlan& t = h->plan.t[tensor];
  switch (t.path) {
    case Path::kRank1: *path = APOLLO_PATH_RANK1; break;
    case Path::kMfma: *path = APOLLO_PATH_MATRIX_CORE; break;
    case Path::kGeneric: *path = APOLLO_PATH_GENERAL; break;
    case Path::kIdentity: *path = APOLLO_PATH_NONE; break;
  }
  if (padded_copy) *padded_copy = t.pad_g ? 1 : 0;
  return APOLLO_OK;
}

apollo_status_t apollo_profile_enable(apollo_handle_t* h, int32_t on) {
  if (!h) return fail(g_last_error, APOLLO_EINVAL, "null handle");
  h->profiling = on != 0;
  return APOLLO_OK;
}

apollo_status_t apollo_profile_read(apollo_handle_t* h, float* ms, int32_t* n_steps) {
  if (!h) return fail(g_last_error, APOLLO_EINVAL, "null handle");
  if (!ms || !n_steps) return fail(h->err, APOLLO_EINVAL, "null output");
  for (int p = 0; p < 5; ++p) ms[p] = 0.f;
  *n_steps = (int32_t)(h->prof_used / 6);
  for (size_t k = 0; k + 6 <= h->prof_used; k += 6) {
    hipError_t e = hipEventSynchronize(h->prof_events[k + 5]);
    for (int p = 0; p < 5 && e == hipSuccess; ++p) {
      float t = 0.f;
      e = hipEventElapsedTime(&t, h->prof_events[k + p], h->prof_events[k + p + 1]);
      ms[p] += t;
    }
    if (e != hipSuccess) {
      h->prof_used = 0;
      return hip_fail(h->err, e, "phase timing");
    }
  }
  h->prof_used = 0;
  return APOLLO_OK;
}

apollo_status_t apollo_debug_fill_projection(apollo_handle_t* h, int32_t tensor, int64_t step, void* out,
                                             int32_t dtype, void* hip_stream) {
  if (!h) return fail(g_last_error, APOLLO_EINVAL, "null handle");
  if (tensor < 0 || tensor >= (int32_t)h->plan.t.size()) return fail(h->err, APOLLO_EINVAL, "tensor index %lld out of range", tensor);
  if (!out) return fail(h->err, APOLLO_EINVAL, "null output");
  if (step < 1) return fail(h->err, APOLLO_EINVAL, "step %lld < 1", step);
  if (dtype != APOLLO_F32 && dtype != APOLLO_BF16) return fail(h->err, APOLLO_EUNSUPPORTED, "dtype %lld", dtype);
  if (h->cfg.projection == APOLLO_PROJ_IDENTITY) return fail(h->err, APOLLO_EINVAL, "this configuration has no projection matrix");
  const StepParams sp = make_step_params(h->cfg, step, 0.f);
  const hipError_t e = launch_fill_projection_rowmajor(out, dtype == APOLLO_BF16, h->cfg.rank, h->plan.t[tensor].m,
                                                       (uint32_t)tensor, sp, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return hip_fail(h->err, e, "projection fill (debug)");
  return APOLLO_OK;
}

apollo_status_t apollo_debug_get(apollo_handle_t* h, int32_t tensor, int32_t what, void* out, size_t bytes,
                                 void* hip_stream) {
  if (!h) return fail(g_last_error, APOLLO_EINVAL, "null handle");
  if (tensor < 0 || tensor >= (int32_t)h->plan.t.size()) return fail(h->err, APOLLO_EINVAL, "tensor index %lld out of range", tensor);
  if (!out) return fail(h->err, APOLLO_EINVAL, "null output");
  const TensorPlan& t = h->plan.t[tensor];
  const size_t rn = (size_t)t.r * t.n * sizeof(float);
  const void* src = nullptr;
  size_t need = 0;
  bool widen = false;     // the source is bfloat16 and is delivered as fp32
  switch (what) {
    case APOLLO_DBG_M: src = h->state + t.st_m; need = rn; widen = h->cfg.state_dtype == APOLLO_BF16; break;
    case APOLLO_DBG_V: src = h->state + t.st_v; need = rn; widen = h->cfg.state_dtype == APOLLO_BF16; break;
    case APOLLO_DBG_S:
      if (h->cfg.mode == APOLLO_TENSOR) { src = h->ws + t.ws_scal + 3 * sizeof(float); need = sizeof(float); }
      else { src = h->ws + t.ws_s; need = (size_t)t.n * sizeof(float); }
      break;
    case APOLLO_DBG_NORM: src = h->state + t.st_norm; need = sizeof(float); break;
    case APOLLO_DBG_C: src = h->ws + t.ws_scal + sizeof(float); need = sizeof(float); break;
    case APOLLO_DBG_R:
      if (t.path == Path::kIdentity) return fail(h->err, APOLLO_EINVAL, "no projected gradient without a projection");
      if (t.fused) {
        // no R is kept for this tensor (the projection kernel consumes it in registers): compute it
        // again into `out`, from the gradient buffer of the last step and the P the workspace holds
        if (bytes != rn) return fail(h->err, APOLLO_EINVAL, "selector %lld holds %lld bytes, %lld given", what, (long long)rn, (long long)bytes);
        if (!h->have_ptrs || h->p_epoch < 0) return fail(h->err, APOLLO_EINVAL, "no step has run on this handle yet");
        StepParams sp = make_step_params(h->cfg, h->p_epoch * (int64_t)h->cfg.refresh_interval + 1, 0.f);
        if (h->cfg.schedule == APOLLO_SCHEDULE_CHUNKED) {      // the scratch holds the P of a group's last chunk
          const hipError_t ef = launch_fill_projection(reinterpret_cast<const TensorDesc*>(h->ws) + t.desc_index, 1, h->cfg.rank, t.m8,
                                                       t.bf16, StepArgs{sp, nullptr}, static_cast<hipStream_t>(hip_stream));
          if (ef != hipSuccess) return hip_fail(h->err, ef, "projection fill (debug)");
        }
        const hipError_t e = launch_project_mfma(reinterpret_cast<const TensorDesc*>(h->ws) + t.desc_index, 1, t.rows, t.cols,
                                                 t.left, t.pad_g, false, false, static_cast<float*>(out), StepArgs{sp, nullptr},
                                                 static_cast<hipStream_t>(hip_stream));
        if (e != hipSuccess) return hip_fail(h->err, e, "projection (debug)");
        return APOLLO_OK;
      }
      src = h->ws + t.ws_r; need = rn; break;
    case APOLLO_DBG_COLSQ: src = h->ws + t.ws_colsq; need = (size_t)t.n * sizeof(float); break;
    default: return fail(h->err, APOLLO_EINVAL, "unknown selector %lld", what);
  }
  if (bytes != need) return fail(h->err, APOLLO_EINVAL, "selector %lld holds %lld bytes, %lld given", what, (long long)need, (long long)bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const hipError_t e = widen ? launch_bf16_to_f32(static_cast<float*>(out), src, need / sizeof(float), st)
                             : hipMemcpyAsync(out, src, need, hipMemcpyDeviceToDevice, st);
  if (e != hipSuccess) return hip_fail(h->err, e, "copy (debug)");
  return APOLLO_OK;
}

apollo_status_t apollo_debug_philox(const void* ctr, uint32_t key0, uint32_t key1, void* out, int64_t count,
                                    void* hip_stream) {
  if (count < 0 || (count > 0 && (!ctr || !out))) return fail(g_last_error, APOLLO_EINVAL, "bad arguments");
  const hipError_t e = launch_philox_words(static_cast<const uint32_t*>(ctr), key0, key1, static_cast<uint32_t*>(out),
                                           count, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return hip_fail(g_last_error, e, "philox (debug)");
  return APOLLO_OK;
}

apollo_status_t apollo_debug_gauss_parts(uint32_t first, int64_t count, void* radius, void* cosv, void* sinv,
                                         void* hip_stream) {
  if (count < 0 || (uint64_t)first + (uint64_t)count > (1ull << 24) || (count > 0 && (!radius || !cosv || !sinv)))
    return fail(g_last_error, APOLLO_EINVAL, "bad arguments (inputs are 24-bit: first + count <= 2^24)");
  const hipError_t e = launch_gauss_parts(first, count, static_cast<float*>(radius), static_cast<float*>(cosv),
                                          static_cast<float*>(sinv), static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return hip_fail(g_last_error, e, "gauss parts (debug)");
  return APOLLO_OK;
}

apollo_status_t apollo_debug_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  if (!dst || !src || (bytes & 15) || (((uintptr_t)dst | (uintptr_t)src) & 15) || bytes >= (1ull << 40))
    return fail(g_last_error, APOLLO_EINVAL, "bad arguments (16-byte aligned pointers, bytes a multiple of 16)");
  const hipError_t e = launch_copy(dst, src, bytes, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return hip_fail(g_last_error, e, "copy (debug)");
  return APOLLO_OK;
}

// ---------------------------------------------------------------------------------------------
// apollo_step_noalloc: the step with its scratch in a static device array instead of a caller's
// workspace, for callers that cannot allocate.
// ---------------------------------------------------------------------------------------------
}  // extern "C"

// The scratch of apollo_step_noalloc: one copy per GPU the library runs on, held until the process
// ends.  In host code the name is only a stand-in for the symbol: the device address comes from
// hipGetSymbolAddress (noalloc_scratch below) and is what every launch and copy receives.
static __device__ __align__(256) unsigned char scratch[APOLLO_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<unsigned char*> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up once per device).
int noalloc_scratch(unsigned char** out, std::string& err) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(err, e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(err, APOLLO_EUNSUPPORTED, "device index %lld outside 0..63", dev);
  unsigned char* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (!p) {
      void* sym = nullptr;
      e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !sym) return hip_fail(err, e, "hipGetSymbolAddress(scratch)");
      p = static_cast<unsigned char*>(sym);
      g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
  }
  *out = p;
  return APOLLO_OK;
}

// Descriptors travel to the device as a kernel argument (no staging buffer, no copy engine): up to
// kPackDescs per launch, read word by word from the kernel-argument segment.
constexpr int kPackDescs = 16;
struct DescPack {
  TensorDesc d[kPackDescs];
};
static_assert(sizeof(DescPack) <= 3072 && sizeof(TensorDesc) % 4 == 0, "descriptor pack must fit the kernel arguments");

__global__ __launch_bounds__(64) void stage_descs_kernel(DescPack pack, TensorDesc* dst, int count) {
  (void)pack;   // first argument: offset 0 of the kernel-argument segment
  typedef __attribute__((address_space(4))) const uint32_t karg_word_t;
  karg_word_t* src = (karg_word_t*)__builtin_amdgcn_kernarg_segment_ptr();
  uint32_t* out = reinterpret_cast<uint32_t*>(dst);
  const int words = count * (int)(sizeof(TensorDesc) / 4);
  for (int i = threadIdx.x; i < words; i += 64) out[i] = src[i];
}

}  // namespace

extern "C" {

apollo_status_t apollo_step_noalloc(const apollo_config_t* cfg, const apollo_shape_t* shapes,
                                    const apollo_tensor_t* tensors, int32_t n_tensors, void* state,
                                    size_t state_bytes, int32_t zero_state, int64_t step, float lr,
                                    void* hip_stream) {
  std::string& err = g_last_error;
  if (n_tensors > APOLLO_NOALLOC_MAX_TENSORS)
    return fail(err, APOLLO_EUNSUPPORTED, "apollo_step_noalloc takes at most %lld tensors per call, %lld given",
                APOLLO_NOALLOC_MAX_TENSORS, n_tensors);
  Plan plan;
  if (!cfg) return fail(err, APOLLO_EINVAL, "null config or shape list");
  apollo_config_t serial_cfg = *cfg;      // one call, one pass over P: the schedule does not apply
  if (serial_cfg.schedule == APOLLO_SCHEDULE_OVERLAP || serial_cfg.schedule == APOLLO_SCHEDULE_CHUNKED)
    serial_cfg.schedule = APOLLO_SCHEDULE_SERIAL;
  int rc = make_plan(&serial_cfg, shapes, n_tensors, plan, err);
  if (rc != APOLLO_OK) return rc;
  if (!tensors || !state) return fail(err, APOLLO_EINVAL, "null tensor list or state buffer");
  if ((uintptr_t)state & (kAlign - 1)) return fail(err, APOLLO_ESTATE, "state not 256-byte aligned");
  if (state_bytes < plan.state_bytes)
    return fail(err, APOLLO_ESTATE, "state buffer has %lld bytes, %lld needed", (long long)state_bytes, (long long)plan.state_bytes);
  if (plan.workspace_bytes > (size_t)APOLLO_NOALLOC_SCRATCH_BYTES)
    return fail(err, APOLLO_EUNSUPPORTED,
                "this tensor list needs %lld bytes of scratch, the static scratch of apollo_step_noalloc holds %lld: "
                "pass fewer or smaller tensors per call, or use apollo_init / apollo_step with a workspace",
                (long long)plan.workspace_bytes, (long long)APOLLO_NOALLOC_SCRATCH_BYTES);
  if (step < 1) return fail(err, APOLLO_EINVAL, "step %lld < 1 (steps are 1-based)", step);
  if (!std::isfinite(lr)) return fail(err, APOLLO_EINVAL, "learning rate is not finite");
  for (int32_t k = 0; k < n_tensors; ++k) {
    if (!tensors[k].w || !tensors[k].g) return fail(err, APOLLO_EINVAL, "tensor %lld: null w or g", k);
    if (((uintptr_t)tensors[k].w | (uintptr_t)tensors[k].g) & 15u)
      return fail(err, APOLLO_EINVAL, "tensor %lld: w / g not 16-byte aligned", k);
    if (cfg->weight_dtype == APOLLO_Q8 && (!tensors[k].w_meta || ((uintptr_t)tensors[k].w_meta & 7u)))
      return fail(err, APOLLO_EINVAL, "tensor %lld: w_meta null or not 8-byte aligned", k);
  }
  unsigned char* ws = nullptr;
  rc = noalloc_scratch(&ws, err);
  if (rc != APOLLO_OK) return rc;

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  TensorDesc* dd = reinterpret_cast<TensorDesc*>(ws);
  DescPack pack;
  for (int32_t first = 0; first < n_tensors; first += kPackDescs) {
    const int32_t cnt = std::min<int32_t>(kPackDescs, n_tensors - first);
    std::memset(&pack, 0, sizeof pack);
    for (int32_t k = 0; k < n_tensors; ++k) {        // descriptor-table order is the plan's (grouped by shape)
      const TensorPlan& t = plan.t[k];
      if (t.desc_index < first || t.desc_index >= first + cnt) continue;
      TensorDesc& d = pack.d[t.desc_index - first];
      fill_desc(d, t, k, static_cast<char*>(state), reinterpret_cast<char*>(ws));
      d.w = tensors[k].w;
      d.w_meta = static_cast<float*>(tensors[k].w_meta);
      d.g = tensors[k].g;
    }
    hipLaunchKernelGGL(stage_descs_kernel, dim3(1), dim3(64), 0, st, pack, dd + first, (int)cnt);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(err, e, "descriptor staging");
  }
  hipError_t e = hipSuccess;
  if (zero_state) {
    e = launch_fill_zero(state, plan.state_bytes, st);
    if (e != hipSuccess) return hip_fail(err, e, "state fill");
  }
  const StepParams sp = make_step_params(*cfg, step, lr);
  // the scratch is shared by every call on this GPU and keeps nothing between calls: P is generated
  // in every call (nothing else in it is read before it is written within a step)
  GroupLaunches L{*cfg, dd, StepArgs{sp, nullptr}, true, ""};
  e = run_serial(L, plan, st, nullptr);
  if (e != hipSuccess) return hip_fail(err, e, L.what);
  return APOLLO_OK;
}

const char* apollo_last_error(const apollo_handle_t* h) { return h ? h->err.c_str() : g_last_error.c_str(); }

void apollo_destroy(apollo_handle_t* h) {
  if (!h) return;
  for (int i = 0; i < kRingSlots; ++i) {
    if (h->ring_used[i]) (void)hipEventSynchronize(h->ring_ev[i]);   // its own pending upload only
    if (h->ring_ev[i]) (void)hipEventDestroy(h->ring_ev[i]);
    if (h->ring[i]) (void)hipHostFree(h->ring[i]);
  }
  for (hipEvent_t ev : h->prof_events) (void)hipEventDestroy(ev);
  for (hipEvent_t ev : h->ev_proj)
    if (ev) (void)hipEventDestroy(ev);
  if (h->ev_fork) (void)hipEventDestroy(h->ev_fork);
  if (h->ev_join) (void)hipEventDestroy(h->ev_join);
  if (h->side) {
    (void)hipStreamSynchronize(h->side);      // its own stream only
    (void)hipStreamDestroy(h->side);
  }
  delete h;
}

}  // extern "C"
