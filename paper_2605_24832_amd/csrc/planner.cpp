// Host planner of the chunked block-diffusion attention step: validates the
// per-iteration descriptors (ragged chunk sizes c_i, cached lengths L_i, block
// origins s_i; Optimus Sec. 4.4: the chunk size changes every iteration) and
// turns them into a flat list of device work items.  Pure host code.
#include <algorithm>
#include <cmath>

#include "plan_internal.h"

namespace optimus {

int validate_params(const optimus_attn_params_t& p) {
  if (p.num_q_heads <= 0 || p.num_kv_heads <= 0 || p.block_size <= 0 || p.num_pages < 0 ||
      p.max_pages_per_req <= 0)
    return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (p.mask_mode != 0 && p.mask_mode != 1) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (p.out_dtype != 0 && p.out_dtype != 1) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (p.num_q_heads % p.num_kv_heads != 0) return OPTIMUS_ERR_UNSUPPORTED_SHAPE;
  if (p.head_dim != 64 && p.head_dim != 128) return OPTIMUS_ERR_UNSUPPORTED_SHAPE;
  if (p.page_size != 16 && p.page_size != 32 && p.page_size != 64 && p.page_size != 128)
    return OPTIMUS_ERR_UNSUPPORTED_SHAPE;
  if (p.kv_layout != 1) return OPTIMUS_ERR_UNSUPPORTED_SHAPE;
  const int64_t tile = (int64_t)p.page_size * p.head_dim;
  const int64_t strides[4] = {p.k_stride_page, p.k_stride_head, p.v_stride_page, p.v_stride_head};
  for (int64_t s : strides)
    if (s < 0 || s % 8 != 0) return OPTIMUS_ERR_INVALID_ARGUMENT;
  // tiles of different heads / pages must not overlap
  if (p.num_kv_heads > 1 && (p.k_stride_head < tile || p.v_stride_head < tile))
    return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (p.k_stride_page < tile || p.v_stride_page < tile) return OPTIMUS_ERR_INVALID_ARGUMENT;
  return OPTIMUS_OK;
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

int build_host_plan(const optimus_attn_params_t& p, const Tuning& tuning, int num_cus,
                    int32_t batch, const int32_t* cu_q, const int32_t* prefix_len,
                    const int32_t* block_start, const int32_t* block_table, HostPlan* out) {
  if (batch < 0 || !out) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (batch > 0 && (!cu_q || !prefix_len || !block_start)) return OPTIMUS_ERR_INVALID_ARGUMENT;
  HostPlan& hp = *out;
  hp = HostPlan();
  hp.batch = batch;
  if (batch == 0) return OPTIMUS_OK;

  const int P = p.page_size, B = p.block_size, Hkv = p.num_kv_heads;
  const int G = p.num_q_heads / p.num_kv_heads;

  // ---- validation (every failure is detectable without a device) ----
  if (cu_q[0] != 0) return OPTIMUS_ERR_BAD_CU_Q;
  for (int i = 0; i < batch; ++i)
    if (cu_q[i + 1] < cu_q[i]) return OPTIMUS_ERR_BAD_CU_Q;
  for (int i = 0; i < batch; ++i) {
    const int64_t L = prefix_len[i], s = block_start[i], c = cu_q[i + 1] - cu_q[i];
    if (L < 0 || s < 0 || s > L) return OPTIMUS_ERR_BAD_PREFIX;
    // in-block streaming never leaves the current block (Sec. 7.2)
    if (p.mask_mode == 0 && c > 0 && (L - s) + c > B) return OPTIMUS_ERR_CHUNK_EXCEEDS_BLOCK;
    if (L + c > (int64_t)INT32_MAX - kTileTokens) return OPTIMUS_ERR_INVALID_ARGUMENT;
    const int64_t need = ceil_div(L + c, P);
    if (c > 0 && need > p.max_pages_per_req) return OPTIMUS_ERR_BLOCK_TABLE_TOO_SHORT;
    if (block_table && c > 0) {
      const int32_t* row = block_table + (int64_t)i * p.max_pages_per_req;
      for (int64_t k = 0; k < need; ++k)
        if (row[k] < 0 || row[k] >= p.num_pages) return OPTIMUS_ERR_PAGE_OUT_OF_RANGE;
    }
  }

  hp.total_q = cu_q[batch];
  hp.cu_q.assign(cu_q, cu_q + batch + 1);
  hp.prefix_len.assign(prefix_len, prefix_len + batch);
  hp.block_start.assign(block_start, block_start + batch);
  hp.token_req.resize(hp.total_q);
  for (int i = 0; i < batch; ++i)
    for (int t = cu_q[i]; t < cu_q[i + 1]; ++t) hp.token_req[t] = i;

  // ---- how many keys one work item scans ----
  double total_cost = 0.0;
  for (int i = 0; i < batch; ++i) {
    const int64_t c = cu_q[i + 1] - cu_q[i];
    if (c == 0) continue;
    const int64_t rows = c * G;
    const int64_t tiles = ceil_div((int64_t)prefix_len[i] + c, kTileTokens);
    for (int64_t r0 = 0; r0 < rows; r0 += kMaxRowsPerItem)
      total_cost += (double)Hkv * tiles *
                    tile_cost_of_rows((int)std::min<int64_t>(kMaxRowsPerItem, rows - r0));
  }
  const int64_t target_items = tuning.target_items > 0 ? tuning.target_items : 4 * (int64_t)num_cus;
  const int64_t min_tiles =
      std::max<int64_t>(1, (tuning.min_split_tokens > 0 ? tuning.min_split_tokens : 256) / kTileTokens);
  const int64_t max_tiles = std::max<int64_t>(
      min_tiles, (tuning.max_split_tokens > 0 ? tuning.max_split_tokens : 8192) / kTileTokens);
  const double target_cost = total_cost / (double)std::max<int64_t>(target_items, 1);

  // ---- emit items ----
  // The row tiles of one (request, kv head, key range) scan the same K/V: they are emitted
  // next to each other (and have equal cost, so the stable sort keeps them together) and
  // thus run at the same time on neighbouring compute units, the later ones hitting the
  // caches instead of HBM.
  struct Keyed { optimus_work_item_t it; double cost; };
  std::vector<Keyed> keyed;
  int64_t part_rows = 0;
  for (int i = 0; i < batch; ++i) {
    const int c = cu_q[i + 1] - cu_q[i];
    if (c == 0) continue;
    const int kv_len = prefix_len[i] + c;
    const int rows = c * G;
    const int n_tiles = (int)ceil_div(kv_len, kTileTokens);
    const int n_row_tiles = (int)ceil_div(rows, kMaxRowsPerItem);
    // all row tiles of a pair use the split of the widest one, so that their key ranges match
    const int rc_max = std::min(kMaxRowsPerItem, rows);
    const double tile_cost_max = tile_cost_of_rows(rc_max);
    // a split costs one partial (rows x (D+2) floats written, then read by the merge): keep
    // it well below the K/V bytes the item streams (32 keys x 2 x D bf16 per tile)
    const int64_t min_tiles_rows = std::max<int64_t>(min_tiles, (rc_max + 7) / 8);
    const int64_t tiles_per_item =
        std::min(std::max(max_tiles, min_tiles_rows),
                 std::max(min_tiles_rows, (int64_t)std::ceil(target_cost / tile_cost_max)));
    const int n_splits = (int)ceil_div(n_tiles, tiles_per_item);
    const int tiles_per_split = (int)ceil_div(n_tiles, n_splits);
    for (int g = 0; g < Hkv; ++g) {
      std::vector<int32_t> first_part(n_row_tiles, -1);
      if (n_splits > 1) {
        for (int rt = 0; rt < n_row_tiles; ++rt) {
          const int r0 = rt * kMaxRowsPerItem, rc = std::min(kMaxRowsPerItem, rows - r0);
          first_part[rt] = (int32_t)part_rows;
          MergeItem m{};
          m.kv_head = g; m.row_begin = r0; m.row_count = rc; m.q_token0 = cu_q[i];
          m.first_part_row = first_part[rt]; m.n_splits = n_splits;
          hp.merges.push_back(m);
          part_rows += (int64_t)n_splits * rc;
        }
      }
      for (int s = 0; s < n_splits; ++s) {
        const int kv_begin = s * tiles_per_split * kTileTokens;
        const int kv_end = std::min(kv_len, (s + 1) * tiles_per_split * kTileTokens);
        if (kv_begin >= kv_end) {
          // cannot happen: tiles_per_split <= tiles_per_item, so (n_splits-1) splits never
          // cover all n_tiles
          return OPTIMUS_ERR_INVALID_ARGUMENT;
        }
        const int64_t tiles = ceil_div(kv_end - kv_begin, kTileTokens);
        for (int rt = 0; rt < n_row_tiles; ++rt) {
          const int r0 = rt * kMaxRowsPerItem, rc = std::min(kMaxRowsPerItem, rows - r0);
          optimus_work_item_t it{};
          it.req = i; it.kv_head = g; it.row_begin = r0; it.row_count = rc;
          it.kv_begin = kv_begin; it.kv_end = kv_end;
          it.part_row = n_splits > 1 ? first_part[rt] + s * rc : -1;
          it.q_token0 = cu_q[i];
          keyed.push_back({it, tiles * tile_cost_max});
        }
      }
    }
  }
  if (part_rows > (int64_t)INT32_MAX / 2) return OPTIMUS_ERR_INVALID_ARGUMENT;
  std::stable_sort(keyed.begin(), keyed.end(),
                   [](const Keyed& a, const Keyed& b) { return a.cost > b.cost; });
  // Workgroups go to the 8 XCDs (each with its own L2) round-robin by index.  Sibling row
  // tiles (same request, kv head and key range; adjacent after the stable sort) are put
  // into one of 8 lanes and the lanes are emitted interleaved, so siblings land on the same
  // XCD at indices p, p+8, ...: the second one finds the K/V stream in that XCD's L2.  The
  // lane is the one with the least cost so far, which also balances the XCDs.
  std::vector<Keyed> lanes[kNumXcd];
  double lane_cost[kNumXcd] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (size_t k = 0; k < keyed.size();) {
    size_t e = k + 1;
    while (e < keyed.size() && keyed[e].it.req == keyed[k].it.req &&
           keyed[e].it.kv_head == keyed[k].it.kv_head && keyed[e].it.kv_begin == keyed[k].it.kv_begin)
      ++e;
    int best = 0;
    for (int x = 1; x < kNumXcd; ++x)
      if (lane_cost[x] < lane_cost[best]) best = x;
    for (size_t j = k; j < e; ++j) {
      lanes[best].push_back(keyed[j]);
      lane_cost[best] += keyed[j].cost;
    }
    k = e;
  }
  hp.items.reserve(keyed.size());
  for (size_t depth = 0; hp.items.size() < keyed.size(); ++depth)
    for (int x = 0; x < kNumXcd; ++x)
      if (depth < lanes[x].size()) hp.items.push_back(lanes[x][depth].it);
  hp.part_rows = part_rows;
  hp.workspace_bytes = (size_t)part_rows * (size_t)(p.head_dim + 2) * sizeof(float);
  return OPTIMUS_OK;
}

}  // namespace optimus
