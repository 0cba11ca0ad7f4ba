// Internal structures of the chunked block-diffusion attention library
// (host planner <-> kernels).  Not part of the C ABI.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "optimus_attn.h"

namespace optimus {

constexpr int kTileTokens = 32;     // keys per MFMA tile step (one 16x16x32 PV contraction)
constexpr int kRowsPerSubtile = 16; // query rows per MFMA N tile
constexpr int kWavesPerBlock = 4;
// Work items by query-row count.  A (request, kv head) pair with more than kMaxRowsPerItem
// rows is cut into row tiles of that many.  Pairs with more than kWideMinRows rows run the
// wide body (32 rows per wave, all their row tiles, also a narrow last one); of the others,
// items of at most 16 rows run the split-wave body (the waves split the keys) and items of
// 17..32 rows the lds-tile body (the waves split the rows, 16 each).  Measured on a mixed-chunk
// batch: the wide body from 33 rows on is 3 % faster than from 65 on (waves without rows idle
// there, but two waves then share every K/V operand read instead of four), from 17 on it is
// 10 % slower on a batch of one 32-row request.
constexpr int kMaxRowsPerItem = 128;
constexpr int kWideMinRows = 32;
constexpr int kNumXcd = 8;  // accelerator dies of an MI355X; workgroup i runs on die i % 8
// Relative cost of one 32-key tile for an item of `rows` query rows (measured on 32K-key
// scans: 16, 32..64 and 128 rows take 104, 114 and 113..128 us for the same key range).
// In tenths, so that costs stay small integers.
constexpr int tile_cost10_of_rows(int rows) { return rows <= 16 ? 10 : (rows <= kWideMinRows ? 11 : 12); }

// One merge job: `n_splits` partials of the same q tile, stored back to back
// (`row_count` rows each) starting at workspace row `first_part_row`.
struct MergeItem {
  int32_t kv_head;
  int32_t row_begin;
  int32_t row_count;
  int32_t q_token0;
  int32_t first_part_row;
  int32_t n_splits;
  int32_t pad0, pad1;
};

struct Tuning {
  int32_t target_items = 0;      // 0 -> default from the CU count
  int32_t min_split_tokens = 0;  // 0 -> default
  int32_t max_split_tokens = 0;  // 0 -> default
};

// Result of host planning for one iteration.
struct PlanGroup;  // planner-private
struct HostPlan {
  int32_t batch = 0;
  int32_t total_q = 0;
  std::vector<optimus_work_item_t> items;  // costliest first, interleaved over 8 XCD lanes
  std::vector<MergeItem> merges;
  // KV append runs, 4 x int32 each (request, first token, first logical slot, count <= 8):
  // the slots of a run lie in one aligned group of 8
  std::vector<int32_t> append_runs;
  std::vector<int32_t> cu_q, prefix_len, block_start;
  int64_t part_rows = 0;            // rows of split-KV partials in the workspace
  size_t workspace_bytes = 0;
  // planner scratch, kept for its capacity
  std::vector<int32_t> req_first_merge, scratch_order, scratch_pos, scratch_count;
  std::vector<int8_t> scratch_lane;
  std::vector<uint64_t> scratch_keys;
  struct Group { int32_t req, kv_head, kv_begin, kv_end, split, n_splits, n_row_tiles, cost10; };  // cost10: tenths of a tile
  std::vector<Group> scratch_groups;
  // per request with a non-empty chunk: key tiles, cost of a tile in tenths (and its
  // reciprocal), bounds of the tiles per item, items per key range (kv heads x row tiles)
  struct Shapes {
    std::vector<double> tiles, w10, inv_w10, lo, hi, mult;
    void clear() { tiles.clear(); w10.clear(); inv_w10.clear(); lo.clear(); hi.clear(); mult.clear(); }
  };
  Shapes scratch_shapes;

  void reset() {
    batch = 0; total_q = 0; part_rows = 0; workspace_bytes = 0;
    items.clear(); merges.clear(); append_runs.clear(); cu_q.clear(); prefix_len.clear();
    block_start.clear();
  }
};

// Pure host code: validate the descriptors and build the work list.
// Returns an optimus_status_t.
int build_host_plan(const optimus_attn_params_t& p, const Tuning& tuning, int num_cus,
                    int32_t batch, const int32_t* cu_q, const int32_t* prefix_len,
                    const int32_t* block_start, const int32_t* block_table, HostPlan* out);

int validate_params(const optimus_attn_params_t& p);

// Device-side argument block shared by the kernels.
struct KernelArgs {
  const uint16_t* q;
  const uint16_t* k_pool;
  const uint16_t* v_pool;
  const int32_t* block_table;
  const optimus_work_item_t* items;
  const MergeItem* merges;
  const int32_t* prefix_len;
  const int32_t* block_start;
  const int32_t* cu_q;    // [batch + 1]
  const int32_t* q_pos;   // [T] sequence positions of the chunk tokens, or null (mask mode 1 only)
  void* out;
  float* ws_o;    // [part_rows, D]
  float* ws_ml;   // [part_rows, 2]  (running max in log2 units, sum)
  int64_t k_stride_page, k_stride_head, v_stride_page, v_stride_head;
  int32_t num_q_heads, group, max_pages_per_req, out_fp32;
  int32_t mask_mode, block_size;
  float scale_log2;  // softmax scale * log2(e)
};

// Kernel launchers (kernels.hip).  `stream` is a hipStream_t.
int launch_attention(const optimus_attn_params_t& p, const KernelArgs& a, int32_t n_items,
                     void* stream);
int launch_merge(const optimus_attn_params_t& p, const KernelArgs& a, int32_t n_merges,
                 void* stream);
// `runs` may live in pinned host memory; `runs_host` (optional) is the same list in ordinary
// host memory, from which a short list is copied into the kernel's argument block.  If
// upload_i32 > 0 the launch also copies that many int32 (a multiple of 4) from upload_src
// (pinned host) to upload_dst (device).
int launch_kv_append(const optimus_attn_params_t& p, uint16_t* k_pool, uint16_t* v_pool,
                     const uint16_t* k_new, const uint16_t* v_new, const int32_t* block_table,
                     const int32_t* runs, const int32_t* runs_host, int32_t n_runs, int32_t* upload_dst,
                     const int32_t* upload_src, size_t upload_i32, void* stream);

// Tokens 0..n-1 of k_src / v_src ([n, Hkv, D]) -> logical slots first_slot.. of request `req`.
int launch_kv_write(const optimus_attn_params_t& p, uint16_t* k_pool, uint16_t* v_pool,
                    const uint16_t* k_src, const uint16_t* v_src, const int32_t* block_table,
                    int32_t req, int32_t first_slot, int32_t n, void* stream);

// Copy n_i32 (a multiple of 4) int32 from pinned host memory to device memory with a kernel on
// `stream` (shorter than the copy engine's start-up for the few tens of KB of a work list).
int launch_upload(int32_t* dst_device, const int32_t* src_pinned_host, size_t n_i32, void* stream);

void set_hip_error(int hip_err, const char* where);

// Size of the library's static device scratch (one copy per GPU) and its address on `device`,
// which must be the calling thread's current device.  The address is looked up once per device.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
int static_scratch_for_current_device(int device, void** ptr_out);

// Makes `device` the calling thread's current HIP device for the life of the object and puts
// the caller's device back afterwards.  status() is OPTIMUS_OK or OPTIMUS_ERR_HIP.
class DeviceGuard {
 public:
  explicit DeviceGuard(int device);
  ~DeviceGuard();
  DeviceGuard(const DeviceGuard&) = delete;
  DeviceGuard& operator=(const DeviceGuard&) = delete;
  int status() const { return status_; }

 private:
  int prev_ = -1;
  bool switched_ = false;
  int status_ = 0;
};

}  // namespace optimus
