// C ABI of the chunked block-diffusion attention library: plan objects, device
// upload of the per-iteration work list, and the enqueue of the kernels.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "plan_internal.h"

namespace optimus {

static thread_local std::string g_hip_error;

void set_hip_error(int hip_err, const char* where) {
  g_hip_error = std::string(where) + ": " + hipGetErrorString((hipError_t)hip_err);
}

DeviceGuard::DeviceGuard(int device) {
  hipError_t e = hipGetDevice(&prev_);
  if (e == hipSuccess && prev_ != device) {
    e = hipSetDevice(device);
    switched_ = e == hipSuccess;
  }
  if (e != hipSuccess) {
    set_hip_error((int)e, "hipSetDevice");
    status_ = OPTIMUS_ERR_HIP;
  }
}

DeviceGuard::~DeviceGuard() {
  if (switched_) (void)hipSetDevice(prev_);
}

#define OPT_HIP(call, where)                          \
  do {                                                \
    hipError_t e_ = (call);                           \
    if (e_ != hipSuccess) {                           \
      optimus::set_hip_error((int)e_, where);         \
      return OPTIMUS_ERR_HIP;                         \
    }                                                 \
  } while (0)

}  // namespace optimus

using namespace optimus;

struct optimus_attn_plan {
  optimus_attn_params_t params{};
  int device = -1;
  int num_cus = 256;
  Tuning tuning;
  HostPlan host;
  bool planned = false;

  // Device copy of the descriptors and the work list.  plan_update fills one
  // slot of a ring of pinned staging buffers; the first device call after it
  // enqueues the host-to-device copy on the caller's stream (kernel threads read
  // the pinned buffer: cheaper than the copy engine for a few tens of KB), so the
  // upload is ordered behind the kernels of earlier iterations that still read
  // the list.
  static constexpr int kRing = 4;
  int32_t* staging[kRing] = {nullptr, nullptr, nullptr, nullptr};
  size_t staging_cap[kRing] = {0, 0, 0, 0};   // in int32
  hipEvent_t staging_done[kRing] = {nullptr, nullptr, nullptr, nullptr};
  bool staging_busy[kRing] = {false, false, false, false};
  int slot = 0;
  bool dirty = false;          // staging[slot] not yet copied to dev_buf
  size_t upload_i32 = 0;
  int32_t* dev_buf = nullptr;
  size_t dev_cap = 0;          // in int32
  std::vector<int32_t*> retired;  // outgrown device buffers, freed with the plan
  // offsets (int32 units) into dev_buf
  size_t off_items = 0, off_merges = 0, off_runs = 0, off_cu_q = 0, off_prefix = 0, off_bstart = 0;

  void* static_scratch = nullptr;  // this device's copy of the library's static scratch

  int32_t timing_every = 0;      // 0 = off, n = the attention kernel of every n-th forward is timed
  int64_t forwards_seen = 0;     // forwards since set_timing
  std::vector<hipEvent_t> events;  // pairs (start, stop), created on demand
  size_t events_used = 0;
};

// Every device entry point works on the plan's device and leaves the caller's current device
// as it found it.
#define OPT_ON_PLAN_DEVICE(plan)                                   \
  if ((plan)->device < 0) return OPTIMUS_ERR_NO_DEVICE;            \
  DeviceGuard device_guard_((plan)->device);                       \
  if (device_guard_.status() != OPTIMUS_OK) return device_guard_.status()

extern "C" {

int optimus_attn_plan_create(const optimus_attn_params_t* params, int device,
                             optimus_attn_plan_t** plan_out) {
  if (!params || !plan_out || device < -1) return OPTIMUS_ERR_INVALID_ARGUMENT;
  *plan_out = nullptr;
  int rc = validate_params(*params);
  if (rc != OPTIMUS_OK) return rc;
  optimus_attn_plan* plan = new (std::nothrow) optimus_attn_plan();
  if (!plan) return OPTIMUS_ERR_INVALID_ARGUMENT;
  plan->params = *params;
  plan->device = device;
  if (device >= 0) {
    hipDeviceProp_t prop;
    const hipError_t e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) {
      set_hip_error((int)e, "plan_create");
      optimus_attn_plan_destroy(plan);  // releases whatever was created
      return OPTIMUS_ERR_HIP;
    }
    plan->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    // address of the static scratch on this device (looked up once per device, here at set-up,
    // so that optimus_attn_forward_static has nothing left to set up); a failure only
    // disables that entry point
    DeviceGuard guard(device);
    if (guard.status() == OPTIMUS_OK) (void)static_scratch_for_current_device(device, &plan->static_scratch);
  }
  *plan_out = plan;
  return OPTIMUS_OK;
}

int optimus_attn_plan_set_tuning(optimus_attn_plan_t* plan, int32_t target_items,
                                 int32_t min_split_tokens, int32_t max_split_tokens) {
  if (!plan || target_items < 0 || min_split_tokens < 0 || max_split_tokens < 0)
    return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (min_split_tokens % kTileTokens != 0 || max_split_tokens % kTileTokens != 0)
    return OPTIMUS_ERR_INVALID_ARGUMENT;
  plan->tuning.target_items = target_items;
  plan->tuning.min_split_tokens = min_split_tokens;
  plan->tuning.max_split_tokens = max_split_tokens;
  return OPTIMUS_OK;
}

int optimus_attn_plan_update(optimus_attn_plan_t* plan, int32_t batch, const int32_t* cu_q_host,
                             const int32_t* prefix_len_host, const int32_t* block_start_host,
                             const int32_t* block_table_host, size_t* workspace_bytes_out) {
  if (!plan) return OPTIMUS_ERR_INVALID_ARGUMENT;
  plan->planned = false;
  int rc = build_host_plan(plan->params, plan->tuning, plan->num_cus, batch, cu_q_host,
                           prefix_len_host, block_start_host, block_table_host, &plan->host);
  if (rc != OPTIMUS_OK) return rc;
  if (workspace_bytes_out) *workspace_bytes_out = plan->host.workspace_bytes;
  if (plan->device < 0 || batch == 0) {
    plan->planned = true;
    return OPTIMUS_OK;
  }
  OPT_ON_PLAN_DEVICE(plan);

  const HostPlan& hp = plan->host;
  static_assert(sizeof(optimus_work_item_t) == 32 && sizeof(MergeItem) == 32, "8 x int32 records");
  size_t off = 0;
  auto take = [&](size_t n_i32) { size_t o = off; off += (n_i32 + 3) & ~size_t(3); return o; };
  plan->off_items = take(hp.items.size() * 8);
  plan->off_merges = take(hp.merges.size() * 8);
  plan->off_runs = take(hp.append_runs.size());
  plan->off_cu_q = take(hp.cu_q.size());
  plan->off_prefix = take(hp.prefix_len.size());
  plan->off_bstart = take(hp.block_start.size());
  const size_t total = off;

  const int sl = (plan->slot + 1) % optimus_attn_plan::kRing;
  if (plan->staging_busy[sl]) {
    // the copy out of this slot was enqueued kRing updates ago; wait for it
    OPT_HIP(hipEventSynchronize(plan->staging_done[sl]), "hipEventSynchronize(staging)");
    plan->staging_busy[sl] = false;
  }
  if (plan->staging_cap[sl] < total) {
    if (plan->staging[sl]) OPT_HIP(hipHostFree(plan->staging[sl]), "hipHostFree");
    plan->staging[sl] = nullptr;
    plan->staging_cap[sl] = 0;
    const size_t cap = total + total / 2 + 1024;
    OPT_HIP(hipHostMalloc((void**)&plan->staging[sl], cap * sizeof(int32_t), hipHostMallocDefault),
            "hipHostMalloc");
    plan->staging_cap[sl] = cap;
  }
  if (!plan->staging_done[sl])
    OPT_HIP(hipEventCreateWithFlags(&plan->staging_done[sl], hipEventDisableTiming), "hipEventCreate");
  if (plan->dev_cap < total) {
    // kernels already enqueued may still read the old buffer: retire it, do not free it now
    if (plan->dev_buf) plan->retired.push_back(plan->dev_buf);
    plan->dev_buf = nullptr;
    plan->dev_cap = 0;
    const size_t cap = total + total / 2 + 1024;
    OPT_HIP(hipMalloc((void**)&plan->dev_buf, cap * sizeof(int32_t)), "hipMalloc");
    plan->dev_cap = cap;
  }
  int32_t* h = plan->staging[sl];
  if (!hp.items.empty()) std::memcpy(h + plan->off_items, hp.items.data(), hp.items.size() * 32);
  if (!hp.merges.empty()) std::memcpy(h + plan->off_merges, hp.merges.data(), hp.merges.size() * 32);
  if (!hp.append_runs.empty())
    std::memcpy(h + plan->off_runs, hp.append_runs.data(), hp.append_runs.size() * 4);
  std::memcpy(h + plan->off_cu_q, hp.cu_q.data(), hp.cu_q.size() * 4);
  std::memcpy(h + plan->off_prefix, hp.prefix_len.data(), hp.prefix_len.size() * 4);
  std::memcpy(h + plan->off_bstart, hp.block_start.data(), hp.block_start.size() * 4);
  plan->slot = sl;
  plan->upload_i32 = total;
  plan->dirty = true;
  plan->planned = true;
  return OPTIMUS_OK;
}

// Enqueue the pending work-list upload (if any) on the caller's stream.
static int flush_upload(optimus_attn_plan* plan, hipStream_t s) {
  if (!plan->dirty) return OPTIMUS_OK;
  const int sl = plan->slot;
  const int rc = launch_upload(plan->dev_buf, plan->staging[sl], plan->upload_i32, s);
  if (rc != OPTIMUS_OK) return rc;
  OPT_HIP(hipEventRecord(plan->staging_done[sl], s), "hipEventRecord(staging)");
  plan->staging_busy[sl] = true;
  plan->dirty = false;
  return OPTIMUS_OK;
}

int optimus_kv_append(optimus_attn_plan_t* plan, void* k_pool, void* v_pool, const void* k_new,
                      const void* v_new, const int32_t* block_table, void* hip_stream) {
  if (!plan) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (!plan->planned) return OPTIMUS_ERR_NOT_PLANNED;
  if (plan->device < 0) return OPTIMUS_ERR_NO_DEVICE;
  if (plan->host.total_q == 0) return OPTIMUS_OK;
  if (!k_pool || !v_pool || !k_new || !v_new || !block_table) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (((uintptr_t)k_pool | (uintptr_t)v_pool | (uintptr_t)k_new | (uintptr_t)v_new) & 15)
    return OPTIMUS_ERR_INVALID_ARGUMENT;
  OPT_ON_PLAN_DEVICE(plan);
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  const int n_runs = (int32_t)(plan->host.append_runs.size() / 4);
  if (!plan->dirty) {
    return launch_kv_append(plan->params, (uint16_t*)k_pool, (uint16_t*)v_pool, (const uint16_t*)k_new,
                            (const uint16_t*)v_new, block_table, plan->dev_buf + plan->off_runs,
                            plan->host.append_runs.data(), n_runs, nullptr, nullptr, 0, hip_stream);
  }
  // a work-list upload is pending: it rides in the same launch, and the runs are read from the
  // pinned copy
  const int sl = plan->slot;
  const int rc = launch_kv_append(plan->params, (uint16_t*)k_pool, (uint16_t*)v_pool, (const uint16_t*)k_new,
                        (const uint16_t*)v_new, block_table, plan->staging[sl] + plan->off_runs,
                        plan->host.append_runs.data(), n_runs, plan->dev_buf, plan->staging[sl],
                        plan->upload_i32, hip_stream);
  if (rc != OPTIMUS_OK) return rc;
  OPT_HIP(hipEventRecord(plan->staging_done[sl], s), "hipEventRecord(staging)");
  plan->staging_busy[sl] = true;
  plan->dirty = false;
  return OPTIMUS_OK;
}

int optimus_kv_write(const optimus_attn_params_t* params, int device, void* k_pool, void* v_pool,
                     const void* k_src, const void* v_src, const int32_t* block_table, int32_t req,
                     int32_t first_slot, int32_t n, void* hip_stream) {
  if (!params || device < 0 || req < 0 || first_slot < 0 || n < 0) return OPTIMUS_ERR_INVALID_ARGUMENT;
  const int rc = validate_params(*params);
  if (rc != OPTIMUS_OK) return rc;
  if ((int64_t)first_slot + n > (int64_t)INT32_MAX - kTileTokens) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (n == 0) return OPTIMUS_OK;
  if (((int64_t)first_slot + n + params->page_size - 1) / params->page_size > params->max_pages_per_req)
    return OPTIMUS_ERR_BLOCK_TABLE_TOO_SHORT;
  if (!k_pool || !v_pool || !k_src || !v_src || !block_table) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (((uintptr_t)k_pool | (uintptr_t)v_pool | (uintptr_t)k_src | (uintptr_t)v_src) & 15)
    return OPTIMUS_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(device);
  if (guard.status() != OPTIMUS_OK) return guard.status();
  return launch_kv_write(*params, (uint16_t*)k_pool, (uint16_t*)v_pool, (const uint16_t*)k_src,
                         (const uint16_t*)v_src, block_table, req, first_slot, n, hip_stream);
}

// Shared by the two forward entry points; `workspace` holds at least hp.workspace_bytes.
static int forward_impl(optimus_attn_plan_t* plan, const void* q, const void* k_pool, const void* v_pool,
                        const int32_t* block_table, const int32_t* q_pos, void* out, void* workspace,
                        bool allow_timing, void* hip_stream) {
  const HostPlan& hp = plan->host;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  int rc = flush_upload(plan, s);
  if (rc != OPTIMUS_OK) return rc;
  const optimus_attn_params_t& p = plan->params;
  const int32_t* d = plan->dev_buf;
  KernelArgs a{};
  a.q = (const uint16_t*)q;
  a.k_pool = (const uint16_t*)k_pool;
  a.v_pool = (const uint16_t*)v_pool;
  a.block_table = block_table;
  a.items = reinterpret_cast<const optimus_work_item_t*>(d + plan->off_items);
  a.merges = reinterpret_cast<const MergeItem*>(d + plan->off_merges);
  a.prefix_len = d + plan->off_prefix;
  a.block_start = d + plan->off_bstart;
  a.cu_q = d + plan->off_cu_q;
  a.q_pos = p.mask_mode == 1 ? q_pos : nullptr;
  a.out = out;
  a.ws_o = reinterpret_cast<float*>(workspace);
  a.ws_ml = a.ws_o ? a.ws_o + (size_t)hp.part_rows * p.head_dim : nullptr;
  a.k_stride_page = p.k_stride_page; a.k_stride_head = p.k_stride_head;
  a.v_stride_page = p.v_stride_page; a.v_stride_head = p.v_stride_head;
  a.num_q_heads = p.num_q_heads;
  a.group = p.num_q_heads / p.num_kv_heads;
  a.max_pages_per_req = p.max_pages_per_req;
  a.out_fp32 = p.out_dtype == 1;
  a.mask_mode = p.mask_mode;
  a.block_size = p.block_size;
  const float scale = p.softmax_scale > 0.f ? p.softmax_scale : 1.0f / std::sqrt((float)p.head_dim);
  a.scale_log2 = scale * 1.4426950408889634f;

  constexpr size_t kMaxTimedForwards = 4096;
  const bool timed = allow_timing && plan->timing_every > 0 &&
                     plan->forwards_seen++ % plan->timing_every == 0 &&
                     plan->events_used < 2 * kMaxTimedForwards;
  if (timed) {
    while (plan->events.size() < plan->events_used + 2) {
      hipEvent_t e;
      OPT_HIP(hipEventCreate(&e), "hipEventCreate");
      plan->events.push_back(e);
    }
    OPT_HIP(hipEventRecord(plan->events[plan->events_used], s), "hipEventRecord");
  }
  rc = launch_attention(p, a, (int32_t)hp.items.size(), hip_stream);
  if (rc != OPTIMUS_OK) return rc;
  if (timed) {
    OPT_HIP(hipEventRecord(plan->events[plan->events_used + 1], s), "hipEventRecord");
    plan->events_used += 2;
  }
  return launch_merge(p, a, (int32_t)hp.merges.size(), hip_stream);
}

int optimus_attn_forward(optimus_attn_plan_t* plan, const void* q, const void* k_pool,
                         const void* v_pool, const int32_t* block_table, void* out, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  return optimus_attn_forward_pos(plan, q, k_pool, v_pool, block_table, nullptr, out, workspace,
                                  workspace_bytes, hip_stream);
}

int optimus_attn_forward_pos(optimus_attn_plan_t* plan, const void* q, const void* k_pool,
                             const void* v_pool, const int32_t* block_table, const int32_t* q_pos,
                             void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!plan) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (!plan->planned) return OPTIMUS_ERR_NOT_PLANNED;
  if (plan->device < 0) return OPTIMUS_ERR_NO_DEVICE;
  const HostPlan& hp = plan->host;
  if (hp.items.empty()) return OPTIMUS_OK;
  if (!q || !k_pool || !v_pool || !block_table || !out) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (((uintptr_t)q | (uintptr_t)k_pool | (uintptr_t)v_pool | (uintptr_t)out | (uintptr_t)workspace) & 15)
    return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (hp.workspace_bytes > 0 && (!workspace || workspace_bytes < hp.workspace_bytes))
    return OPTIMUS_ERR_WORKSPACE_TOO_SMALL;
  OPT_ON_PLAN_DEVICE(plan);
  return forward_impl(plan, q, k_pool, v_pool, block_table, q_pos, out, workspace, true, hip_stream);
}

int optimus_attn_step(optimus_attn_plan_t* plan, int32_t batch, const int32_t* cu_q_host,
                      const int32_t* prefix_len_host, const int32_t* block_start_host,
                      const int32_t* block_table_host, const void* q, const void* k_new, const void* v_new,
                      void* k_pool, void* v_pool, const int32_t* block_table, const int32_t* q_pos,
                      void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = optimus_attn_plan_update(plan, batch, cu_q_host, prefix_len_host, block_start_host,
                                    block_table_host, nullptr);
  if (rc != OPTIMUS_OK) return rc;
  // nothing is launched when the workspace is too small for the new plan
  if (plan->host.workspace_bytes > 0 && (!workspace || workspace_bytes < plan->host.workspace_bytes))
    return OPTIMUS_ERR_WORKSPACE_TOO_SMALL;
  rc = optimus_kv_append(plan, k_pool, v_pool, k_new, v_new, block_table, hip_stream);
  if (rc != OPTIMUS_OK) return rc;
  return optimus_attn_forward_pos(plan, q, k_pool, v_pool, block_table, q_pos, out, workspace,
                                  workspace_bytes, hip_stream);
}

int optimus_attn_forward_static(optimus_attn_plan_t* plan, const void* q, const void* k_pool,
                                const void* v_pool, const int32_t* block_table, void* out,
                                void* hip_stream) {
  if (!plan) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (!plan->planned) return OPTIMUS_ERR_NOT_PLANNED;
  if (plan->device < 0) return OPTIMUS_ERR_NO_DEVICE;
  const HostPlan& hp = plan->host;
  if (hp.items.empty()) return OPTIMUS_OK;
  if (!q || !k_pool || !v_pool || !block_table || !out) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (((uintptr_t)q | (uintptr_t)k_pool | (uintptr_t)v_pool | (uintptr_t)out) & 15)
    return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (hp.workspace_bytes > kStaticScratchBytes) return OPTIMUS_ERR_WORKSPACE_TOO_SMALL;
  if (!plan->static_scratch) return OPTIMUS_ERR_HIP;   // its lookup failed when the plan was created
  OPT_ON_PLAN_DEVICE(plan);
  // no event is created here: this entry point allocates nothing, so it records no timing
  return forward_impl(plan, q, k_pool, v_pool, block_table, nullptr, out, plan->static_scratch, false,
                      hip_stream);
}

size_t optimus_attn_static_scratch_bytes(void) { return kStaticScratchBytes; }

void optimus_attn_plan_destroy(optimus_attn_plan_t* plan) {
  if (!plan) return;
  if (plan->device >= 0) {
    DeviceGuard guard(plan->device);
    if (guard.status() == OPTIMUS_OK) {
      (void)hipDeviceSynchronize();  // nothing of ours may still read the buffers
      if (plan->dev_buf) (void)hipFree(plan->dev_buf);
      for (int32_t* b : plan->retired) (void)hipFree(b);
      for (int r = 0; r < optimus_attn_plan::kRing; ++r) {
        if (plan->staging[r]) (void)hipHostFree(plan->staging[r]);
        if (plan->staging_done[r]) (void)hipEventDestroy(plan->staging_done[r]);
      }
      for (hipEvent_t e : plan->events) (void)hipEventDestroy(e);
    }
  }
  delete plan;
}

int32_t optimus_attn_plan_num_work_items(const optimus_attn_plan_t* plan) {
  return plan ? (int32_t)plan->host.items.size() : OPTIMUS_ERR_INVALID_ARGUMENT;
}

int32_t optimus_attn_plan_num_merge_items(const optimus_attn_plan_t* plan) {
  return plan ? (int32_t)plan->host.merges.size() : OPTIMUS_ERR_INVALID_ARGUMENT;
}

int32_t optimus_attn_plan_get_work_items(const optimus_attn_plan_t* plan,
                                         optimus_work_item_t* items_out, int32_t capacity) {
  if (!plan || capacity < 0 || (capacity > 0 && !items_out)) return OPTIMUS_ERR_INVALID_ARGUMENT;
  const int32_t n = std::min<int32_t>(capacity, (int32_t)plan->host.items.size());
  if (n > 0) std::memcpy(items_out, plan->host.items.data(), (size_t)n * sizeof(optimus_work_item_t));
  return n;
}

int optimus_attn_set_timing(optimus_attn_plan_t* plan, int32_t every) {
  if (!plan || every < 0) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (plan->device < 0) return OPTIMUS_ERR_NO_DEVICE;
  plan->timing_every = every;
  plan->forwards_seen = 0;
  plan->events_used = 0;
  return OPTIMUS_OK;
}

int optimus_attn_timing_read(optimus_attn_plan_t* plan, float* total_ms_out, int32_t* forwards_out) {
  if (!plan || !total_ms_out || !forwards_out) return OPTIMUS_ERR_INVALID_ARGUMENT;
  OPT_ON_PLAN_DEVICE(plan);
  float total = 0.f;
  for (size_t i = 0; i + 1 < plan->events_used; i += 2) {
    float ms = 0.f;
    OPT_HIP(hipEventSynchronize(plan->events[i + 1]), "hipEventSynchronize");
    OPT_HIP(hipEventElapsedTime(&ms, plan->events[i], plan->events[i + 1]), "hipEventElapsedTime");
    total += ms;
  }
  *total_ms_out = total;
  *forwards_out = (int32_t)(plan->events_used / 2);
  return OPTIMUS_OK;
}

const char* optimus_status_string(int status) {
  switch (status) {
    case OPTIMUS_OK: return "ok";
    case OPTIMUS_ERR_INVALID_ARGUMENT: return "invalid argument";
    case OPTIMUS_ERR_UNSUPPORTED_SHAPE: return "unsupported shape";
    case OPTIMUS_ERR_BAD_CU_Q: return "cu_q must start at 0 and be non-decreasing";
    case OPTIMUS_ERR_BAD_PREFIX: return "prefix length / block start out of range";
    case OPTIMUS_ERR_CHUNK_EXCEEDS_BLOCK: return "chunk leaves the current block in in-block mode";
    case OPTIMUS_ERR_BLOCK_TABLE_TOO_SHORT: return "block table row too short for prefix + chunk";
    case OPTIMUS_ERR_PAGE_OUT_OF_RANGE: return "block table entry outside the pool";
    case OPTIMUS_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case OPTIMUS_ERR_NOT_PLANNED: return "no successful plan_update (or nothing recorded) yet";
    case OPTIMUS_ERR_NO_DEVICE: return "host-only plan has no device";
    case OPTIMUS_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

const char* optimus_last_hip_error(void) { return g_hip_error.c_str(); }

}  // extern "C"
