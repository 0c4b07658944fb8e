// Host side of the element-wise AdamW path (non-projected parameters): argument checking, buffer
// layout, descriptor upload, the single launch per step.  Interface in include/apollo.h.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/apollo.h"
#include "apollo_internal.h"

using namespace apollo;

namespace {

constexpr size_t kAlign = 256;
constexpr int32_t kMaxTensors = 65535;
constexpr int64_t kMaxNumel = 1ll << 40;
constexpr int kRingSlots = 4;

inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

thread_local std::string g_adamw_error;

int fail(std::string& dst, int code, const char* fmt, long long a = 0, long long b = 0) {
  char buf[256];
  std::snprintf(buf, sizeof buf, fmt, a, b);
  dst = buf;
  return code;
}

struct FlatPlan {
  struct T {
    uint64_t numel;
    bool bf16, store16;
    size_t st_m, st_v;
    uint32_t first_block, n_blocks;
  };
  std::vector<T> t;
  size_t state_bytes = 0, desc_bytes = 0, table_offset = 0, workspace_bytes = 0;
  uint32_t n_blocks = 0;
};

// Validates the shape list and lays out state and workspace.  Host arithmetic only.
int make_flat_plan(const apollo_flat_shape_t* shapes, int32_t n, FlatPlan& plan, std::string& err) {
  if (!shapes) return fail(err, APOLLO_EINVAL, "null shape list");
  if (n < 1 || n > kMaxTensors) return fail(err, APOLLO_EINVAL, "n_tensors %lld outside 1..65535", n);
  plan.t.resize(n);
  size_t st = 0;
  uint64_t blocks = 0;
  for (int32_t k = 0; k < n; ++k) {
    const apollo_flat_shape_t& s = shapes[k];
    if (s.numel < 1) return fail(err, APOLLO_EINVAL, "tensor %lld: numel must be >= 1", k);
    if (s.numel > kMaxNumel) return fail(err, APOLLO_EUNSUPPORTED, "tensor %lld: more than 2^40 elements", k);
    if (s.grad_dtype != APOLLO_F32 && s.grad_dtype != APOLLO_BF16)
      return fail(err, APOLLO_EUNSUPPORTED, "tensor %lld: gradient dtype %lld is neither fp32 nor bf16", k, s.grad_dtype);
    if (s.store_dtype != APOLLO_F32 && s.store_dtype != APOLLO_BF16)
      return fail(err, APOLLO_EUNSUPPORTED, "tensor %lld: storage dtype %lld is neither fp32 nor bf16", k, s.store_dtype);
    FlatPlan::T& t = plan.t[k];
    t.numel = (uint64_t)s.numel;
    t.bf16 = s.grad_dtype == APOLLO_BF16;
    t.store16 = s.store_dtype == APOLLO_BF16;
    const size_t elem = t.store16 ? 2 : sizeof(float);
    st = align_up(st);
    t.st_m = st;
    st = align_up(st + t.numel * elem);
    t.st_v = st;
    st += t.numel * elem;
    const uint64_t nb = (t.numel + kAdamwBlockElems - 1) / kAdamwBlockElems;
    t.first_block = (uint32_t)blocks;
    t.n_blocks = (uint32_t)nb;
    blocks += nb;
    if (blocks >= (1ull << 31)) return fail(err, APOLLO_EUNSUPPORTED, "tensor list needs 2^31 or more blocks of 1024 elements");
  }
  plan.state_bytes = align_up(st);
  plan.n_blocks = (uint32_t)blocks;
  plan.desc_bytes = (size_t)n * sizeof(AdamwDesc);
  plan.table_offset = align_up(plan.desc_bytes);
  plan.workspace_bytes = align_up(plan.table_offset + (size_t)blocks * sizeof(uint32_t));
  return APOLLO_OK;
}

int check_config(const apollo_adamw_config_t* cfg, std::string& err) {
  if (!cfg) return fail(err, APOLLO_EINVAL, "null config");
  if (!(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f))
    return fail(err, APOLLO_EINVAL, "betas must lie in [0, 1)");
  if (!(cfg->eps >= 0.f) || !std::isfinite(cfg->weight_decay)) return fail(err, APOLLO_EINVAL, "eps negative or weight_decay not finite");
  if (cfg->bias_correction != 0 && cfg->bias_correction != 1) return fail(err, APOLLO_EINVAL, "bias_correction must be 0 or 1");
  return APOLLO_OK;
}

}  // namespace

struct apollo_adamw_handle {
  apollo_adamw_config_t cfg;
  FlatPlan plan;
  char* state = nullptr;
  char* ws = nullptr;
  std::vector<AdamwDesc> desc;
  std::vector<apollo_tensor_t> last;
  AdamwDesc* ring[kRingSlots] = {nullptr, nullptr, nullptr, nullptr};   // pinned staging copies
  hipEvent_t ring_ev[kRingSlots] = {nullptr, nullptr, nullptr, nullptr};
  bool ring_used[kRingSlots] = {false, false, false, false};
  int ring_next = 0;
  bool have_ptrs = false;
  std::string err;
};

namespace {

int hip_fail(std::string& dst, hipError_t e, const char* what) {
  dst = std::string(what) + ": " + hipGetErrorString(e);
  return APOLLO_EHIP;
}

}  // namespace

extern "C" {

size_t apollo_adamw_state_bytes(const apollo_flat_shape_t* shapes, int32_t n_tensors) {
  FlatPlan p;
  if (make_flat_plan(shapes, n_tensors, p, g_adamw_error) != APOLLO_OK) return 0;
  return p.state_bytes;
}

size_t apollo_adamw_workspace_bytes(const apollo_flat_shape_t* shapes, int32_t n_tensors) {
  FlatPlan p;
  if (make_flat_plan(shapes, n_tensors, p, g_adamw_error) != APOLLO_OK) return 0;
  return p.workspace_bytes;
}

apollo_status_t apollo_adamw_state_offsets(const apollo_flat_shape_t* shapes, int32_t n_tensors, int32_t tensor,
                                           size_t* m_offset, size_t* v_offset) {
  FlatPlan p;
  const int rc = make_flat_plan(shapes, n_tensors, p, g_adamw_error);
  if (rc != APOLLO_OK) return rc;
  if (tensor < 0 || tensor >= n_tensors) return fail(g_adamw_error, APOLLO_EINVAL, "tensor index %lld out of range", tensor);
  if (m_offset) *m_offset = p.t[tensor].st_m;
  if (v_offset) *v_offset = p.t[tensor].st_v;
  return APOLLO_OK;
}

apollo_status_t apollo_adamw_init(apollo_adamw_handle_t** out, const apollo_adamw_config_t* cfg,
                                  const apollo_flat_shape_t* shapes, int32_t n_tensors, void* state, size_t state_bytes,
                                  void* workspace, size_t workspace_bytes, int32_t zero_state, void* hip_stream) {
  if (!out) return fail(g_adamw_error, APOLLO_EINVAL, "null output handle pointer");
  *out = nullptr;
  int rc = check_config(cfg, g_adamw_error);
  if (rc != APOLLO_OK) return rc;
  apollo_adamw_handle* h = new (std::nothrow) apollo_adamw_handle;
  if (!h) return fail(g_adamw_error, APOLLO_ENOMEM, "out of host memory");
  rc = make_flat_plan(shapes, n_tensors, h->plan, g_adamw_error);
  if (rc == APOLLO_OK && (!state || !workspace)) rc = fail(g_adamw_error, APOLLO_EINVAL, "null state or workspace buffer");
  if (rc == APOLLO_OK && (((uintptr_t)state | (uintptr_t)workspace) & (kAlign - 1)))
    rc = fail(g_adamw_error, APOLLO_ESTATE, "state / workspace not 256-byte aligned");
  if (rc == APOLLO_OK && state_bytes < h->plan.state_bytes)
    rc = fail(g_adamw_error, APOLLO_ESTATE, "state has %lld bytes, %lld needed", (long long)state_bytes, (long long)h->plan.state_bytes);
  if (rc == APOLLO_OK && workspace_bytes < h->plan.workspace_bytes)
    rc = fail(g_adamw_error, APOLLO_ESTATE, "workspace has %lld bytes, %lld needed", (long long)workspace_bytes,
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
  std::vector<uint32_t> table(h->plan.n_blocks);
  for (int32_t k = 0; k < n_tensors; ++k) {
    const FlatPlan::T& t = h->plan.t[k];
    AdamwDesc& d = h->desc[k];
    std::memset(&d, 0, sizeof d);
    d.m = h->state + t.st_m;
    d.v = h->state + t.st_v;
    d.numel = t.numel;
    d.first_block = t.first_block;
    d.bf16 = t.bf16 ? 1u : 0u;
    d.store16 = t.store16 ? 1u : 0u;
    for (uint32_t b = 0; b < t.n_blocks; ++b) table[t.first_block + b] = (uint32_t)k;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e = hipSuccess;
  for (int i = 0; i < kRingSlots && e == hipSuccess; ++i) {
    e = hipHostMalloc(reinterpret_cast<void**>(&h->ring[i]), h->plan.desc_bytes, hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&h->ring_ev[i], hipEventDisableTiming);
  }
  // the block table never changes: a blocking copy from pageable memory, done once
  if (e == hipSuccess)
    e = hipMemcpy(h->ws + h->plan.table_offset, table.data(), table.size() * sizeof(uint32_t), hipMemcpyHostToDevice);
  if (e == hipSuccess && zero_state) e = launch_fill_zero(h->state, h->plan.state_bytes, st);
  if (e != hipSuccess) {
    hip_fail(g_adamw_error, e, "apollo_adamw_init");
    apollo_adamw_destroy(h);
    return APOLLO_EHIP;
  }
  *out = h;
  return APOLLO_OK;
}

apollo_status_t apollo_adamw_step(apollo_adamw_handle_t* h, const apollo_tensor_t* tensors, int32_t n_tensors,
                                  int64_t step, float lr, void* hip_stream) {
  if (!h) return fail(g_adamw_error, APOLLO_EINVAL, "null handle");
  const int32_t n = (int32_t)h->plan.t.size();
  if (!tensors) return fail(h->err, APOLLO_EINVAL, "null tensor list");
  if (n_tensors != n) return fail(h->err, APOLLO_EINVAL, "n_tensors %lld differs from the %lld given to apollo_adamw_init", n_tensors, n);
  if (step < 1) return fail(h->err, APOLLO_EINVAL, "step %lld < 1 (steps are 1-based)", step);
  if (!std::isfinite(lr)) return fail(h->err, APOLLO_EINVAL, "learning rate is not finite");
  bool changed = !h->have_ptrs;
  for (int32_t k = 0; k < n; ++k) {
    if (!tensors[k].w || !tensors[k].g) return fail(h->err, APOLLO_EINVAL, "tensor %lld: null w or g", k);
    if (((uintptr_t)tensors[k].w | (uintptr_t)tensors[k].g) & 15u)
      return fail(h->err, APOLLO_EINVAL, "tensor %lld: w / g not 16-byte aligned", k);
    if (tensors[k].w != h->last[k].w || tensors[k].g != h->last[k].g) changed = true;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (changed) {
    for (int32_t k = 0; k < n; ++k) {
      h->desc[k].w = tensors[k].w;
      h->desc[k].g = tensors[k].g;
      h->last[k] = tensors[k];
    }
    const int slot = h->ring_next;
    h->ring_next = (slot + 1) % kRingSlots;
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
    h->have_ptrs = true;
  }
  AdamwParams p{};
  const apollo_adamw_config_t& c = h->cfg;
  p.beta1 = c.beta1; p.beta2 = c.beta2; p.omb1 = 1.f - c.beta1; p.omb2 = 1.f - c.beta2; p.eps = c.eps;
  p.inv_bc1 = c.bias_correction ? (float)(1.0 / (1.0 - std::pow((double)c.beta1, (double)step))) : 1.f;
  p.inv_bc2 = c.bias_correction ? (float)(1.0 / (1.0 - std::pow((double)c.beta2, (double)step))) : 1.f;
  p.lr = lr;
  p.lr_decay = lr * c.weight_decay;
  e = launch_adamw(reinterpret_cast<const AdamwDesc*>(h->ws), reinterpret_cast<const uint32_t*>(h->ws + h->plan.table_offset),
                   h->plan.n_blocks, p, st);
  if (e != hipSuccess) return hip_fail(h->err, e, "AdamW launch");
  return APOLLO_OK;
}

const char* apollo_adamw_last_error(const apollo_adamw_handle_t* h) { return h ? h->err.c_str() : g_adamw_error.c_str(); }

void apollo_adamw_destroy(apollo_adamw_handle_t* h) {
  if (!h) return;
  for (int i = 0; i < kRingSlots; ++i) {
    if (h->ring_used[i]) (void)hipEventSynchronize(h->ring_ev[i]);
    if (h->ring_ev[i]) (void)hipEventDestroy(h->ring_ev[i]);
    if (h->ring[i]) (void)hipHostFree(h->ring[i]);
  }
  delete h;
}

}  // extern "C"
