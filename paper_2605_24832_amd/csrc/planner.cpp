// Host planner of the chunked block-diffusion attention step: validates the
// per-iteration descriptors (ragged chunk sizes c_i, cached lengths L_i, block
// origins s_i; Optimus Sec. 4.4: the chunk size changes every iteration) and
// turns them into a flat list of device work items.  Pure host code.
#include <algorithm>
#include <cmath>
#include <cstdlib>

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
  // a page stride is used as a 32-bit byte count by the kernels
  if (p.k_stride_page >= ((int64_t)1 << 31) || p.v_stride_page >= ((int64_t)1 << 31))
    return OPTIMUS_ERR_INVALID_ARGUMENT;
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
  hp.reset();  // keeps the vectors' capacity: planning runs every iteration
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
      uint32_t worst = 0;  // as unsigned, a negative id is larger than any valid one
      for (int64_t k = 0; k < need; ++k) worst = std::max(worst, (uint32_t)row[k]);
      if (worst >= (uint32_t)p.num_pages) return OPTIMUS_ERR_PAGE_OUT_OF_RANGE;
    }
  }

  hp.total_q = cu_q[batch];
  hp.cu_q.assign(cu_q, cu_q + batch + 1);
  hp.prefix_len.assign(prefix_len, prefix_len + batch);
  hp.block_start.assign(block_start, block_start + batch);
  hp.append_runs.clear();
  for (int i = 0; i < batch; ++i) {
    const int c = cu_q[i + 1] - cu_q[i];
    for (int j = 0; j < c;) {
      const int slot = prefix_len[i] + j;
      const int count = std::min(c - j, 8 - (slot & 7));   // up to the end of the aligned group
      hp.append_runs.insert(hp.append_runs.end(), {i, cu_q[i] + j, slot, count});
      j += count;
    }
  }

  // ---- how many keys one work item scans ----
  // Every (request, kv head) pair is cut into equal key ranges of at most `tpi` tiles, with
  // tpi = ceil(item_cost / tile cost of the pair's row count), clamped; item_cost (tenths of
  // a split-wave tile) is the one free parameter.
  const int64_t min_tiles =
      std::max<int64_t>(1, (tuning.min_split_tokens > 0 ? tuning.min_split_tokens : 256) / kTileTokens);
  const int64_t max_tiles = std::max<int64_t>(
      min_tiles, tuning.max_split_tokens > 0 ? tuning.max_split_tokens / kTileTokens : (int64_t)1 << 40);
  HostPlan::Shapes& sh = hp.scratch_shapes;
  sh.clear();
  double total10 = 0.0;
  for (int i = 0; i < batch; ++i) {
    const int64_t c = cu_q[i + 1] - cu_q[i];
    if (c == 0) continue;
    const int64_t rows = c * G;
    const int rc_max = (int)std::min<int64_t>(kMaxRowsPerItem, rows);
    const double tiles = (double)ceil_div((int64_t)prefix_len[i] + c, kTileTokens);
    const double w10 = tile_cost10_of_rows(rc_max);
    // a split costs one partial (rows x (D+2) floats written, then read by the merge): keep
    // it well below the K/V bytes the item streams (32 keys x 2 x D bf16 per tile)
    const double lo = (double)std::max<int64_t>(min_tiles, (rc_max + 7) / 8);
    const double mult = (double)(Hkv * ceil_div(rows, kMaxRowsPerItem));
    sh.tiles.push_back(tiles); sh.w10.push_back(w10); sh.inv_w10.push_back(1.0 / w10);
    sh.lo.push_back(lo); sh.hi.push_back((double)std::max<int64_t>(max_tiles, (int64_t)lo));
    sh.mult.push_back(mult);
    total10 += mult * tiles * w10;
  }
  // the tiles-per-item rule, the same expression here and where the items are emitted
  auto tiles_per_item_of = [](double item_cost10, double inv_w10, double lo, double hi) {
    return std::min(hi, std::max(lo, std::ceil(item_cost10 * inv_w10)));
  };
  struct Fit { double n_items, cost_min, cost_max; };
  auto evaluate = [&](double item_cost10) {
    Fit f{0.0, 1e300, 0.0};
    const size_t n = sh.tiles.size();
    for (size_t k = 0; k < n; ++k) {
      const double tpi = tiles_per_item_of(item_cost10, sh.inv_w10[k], sh.lo[k], sh.hi[k]);
      const double ns = std::ceil(sh.tiles[k] / tpi);
      const double tps = std::ceil(sh.tiles[k] / ns);
      f.n_items += ns * sh.mult[k];
      f.cost_max = std::max(f.cost_max, tps * sh.w10[k]);
      f.cost_min = std::min(f.cost_min, (sh.tiles[k] - (ns - 1.0) * tps) * sh.w10[k]);
    }
    return f;
  };
  // Two workgroups are resident per CU, so `slots` items run at once.  Measured on mixed and
  // uniform batches: a list that fills the slots exactly once beats every finer cut when its
  // items are balanced (a second, partly filled round costs its whole length, and every
  // item pays a few microseconds of start-up), and a list slightly longer than a multiple of
  // the slots is the worst case.  So for lists of up to two rounds the item cost is fitted:
  // for k and k+1 rounds (k the fewest possible) take the smallest item cost whose list has
  // at most k * slots items, and keep the k whose estimated time is lower: one round lasts
  // as long as its longest item; several rounds last total / slots plus, as the drain at the
  // end of a costliest-first list, about one of the smallest items.
  const double slots = 2.0 * std::max(num_cus, 1);
  const double kItemOverhead10 = 40.0;   // start-up of an item in tenths of a tile (about 4 us)
  double item_cost10;
  if (tuning.target_items > 0) {
    item_cost10 = total10 / (double)tuning.target_items;
  } else {
    const Fit uncut = evaluate(1e300);
    if (uncut.n_items > 2.0 * slots) {
      item_cost10 = total10 / (2.0 * slots);
    } else {
      const double k_min = std::max(1.0, std::ceil(uncut.n_items / slots));
      double best_time = 1e300;
      item_cost10 = 1e300;
      for (double k = k_min; k <= k_min + 1.0; k += 1.0) {
        // smallest cost with at most k * slots items: the count falls as the cost grows
        double lo = total10 / (k * slots) * 0.5, hi = std::max(uncut.cost_max, lo);
        if (evaluate(lo).n_items <= k * slots) hi = lo;
        for (int it = 0; it < 14 && hi - lo > 0.5; ++it) {
          const double mid = 0.5 * (lo + hi);
          if (evaluate(mid).n_items <= k * slots) hi = mid; else lo = mid;
        }
        const Fit f = evaluate(hi);
        const double time = f.n_items <= slots
                                ? f.cost_max + kItemOverhead10
                                : (total10 + f.n_items * kItemOverhead10) / slots + f.cost_min + kItemOverhead10;
        if (time < best_time) { best_time = time; item_cost10 = hi; }
      }
    }
  }

  // ---- sibling groups ----
  // A group = the row tiles of one (request, kv head, key range): same K/V stream, same
  // cost.  Groups are sorted costliest first and dealt to 8 lanes (always the lane with
  // the least cost so far); lane x is emitted at work-list indices x, x+8, x+16, ...
  // Workgroups go to the 8 XCDs (each with its own L2) round-robin by index, so the row
  // tiles of a group run at the same time on the same XCD and the later ones find the K/V
  // stream in that XCD's L2; the dealing also balances the XCDs.
  using Group = HostPlan::Group;
  std::vector<Group>& groups = hp.scratch_groups;
  groups.clear();
  int64_t part_rows = 0;
  size_t n_items = 0;
  hp.req_first_merge.assign(batch, -1);
  size_t shape_k = 0;   // index into sh: one entry per request with a non-empty chunk
  for (int i = 0; i < batch; ++i) {
    const int c = cu_q[i + 1] - cu_q[i];
    if (c == 0) continue;
    const int kv_len = prefix_len[i] + c;
    const int rows = c * G;
    const int n_tiles = (int)ceil_div(kv_len, kTileTokens);
    const int n_row_tiles = (int)ceil_div(rows, kMaxRowsPerItem);
    // all row tiles of a pair use the split of the widest one, so that their key ranges match
    const int rc_max = std::min(kMaxRowsPerItem, rows);
    const int64_t tiles_per_item = (int64_t)tiles_per_item_of(item_cost10, sh.inv_w10[shape_k], sh.lo[shape_k], sh.hi[shape_k]);
    ++shape_k;
    const int n_splits = (int)ceil_div(n_tiles, tiles_per_item);
    const int tiles_per_split = (int)ceil_div(n_tiles, n_splits);
    if (n_splits > 1) {
      // merge jobs and partial rows of this request: [kv head][row tile], splits back to back
      hp.req_first_merge[i] = (int32_t)hp.merges.size();
      for (int g = 0; g < Hkv; ++g)
        for (int rt = 0; rt < n_row_tiles; ++rt) {
          const int r0 = rt * kMaxRowsPerItem, rc = std::min(kMaxRowsPerItem, rows - r0);
          MergeItem m{};
          m.kv_head = g; m.row_begin = r0; m.row_count = rc; m.q_token0 = cu_q[i];
          m.first_part_row = (int32_t)part_rows; m.n_splits = n_splits;
          hp.merges.push_back(m);
          part_rows += (int64_t)n_splits * rc;
        }
    }
    // emission order (request, kv head, split); the dealing below rotates its tie-break so
    // that the kv heads of a request spread over the XCDs
    for (int g = 0; g < Hkv; ++g)
      for (int s = 0; s < n_splits; ++s) {
        const int kv_begin = s * tiles_per_split * kTileTokens;
        const int kv_end = std::min(kv_len, (s + 1) * tiles_per_split * kTileTokens);
        if (kv_begin >= kv_end) {
          // cannot happen: tiles_per_split <= tiles_per_item, so (n_splits-1) splits never
          // cover all n_tiles
          return OPTIMUS_ERR_INVALID_ARGUMENT;
        }
        const int32_t cost10 = (int32_t)ceil_div(kv_end - kv_begin, kTileTokens) * tile_cost10_of_rows(rc_max);
        groups.push_back({i, g, kv_begin, kv_end, s, n_splits, n_row_tiles, cost10});
      }
    n_items += (size_t)n_splits * Hkv * n_row_tiles;
  }
  if (part_rows > (int64_t)INT32_MAX / 2) return OPTIMUS_ERR_INVALID_ARGUMENT;
  // costliest first; ties keep the emission order for determinism.  The cost in tenths of a
  // tile is a small integer, so this is a stable counting sort (a comparison sort of 2048
  // groups was half of the planning time); costs beyond the table fall back to sorting packed
  // integers (inverted cost in the high half, emission index in the low half).
  std::vector<uint64_t>& keys = hp.scratch_keys;
  std::vector<int32_t>& order = hp.scratch_order;
  order.resize(groups.size());
  keys.resize(groups.size());
  uint32_t cost_max = 0;
  bool sorted = true;   // already costliest first (a uniform batch): nothing to sort
  for (size_t k = 0; k < groups.size(); ++k) {
    keys[k] = (uint32_t)groups[k].cost10;
    cost_max = std::max(cost_max, (uint32_t)keys[k]);
    sorted &= k == 0 || keys[k] <= keys[k - 1];
  }
  constexpr uint32_t kCountingLimit = 1u << 16;
  if (sorted) {
    for (size_t k = 0; k < order.size(); ++k) order[k] = (int32_t)k;
  } else if (cost_max < kCountingLimit) {
    std::vector<int32_t>& first = hp.scratch_count;   // first[b]: output position of bucket b
    first.assign((size_t)cost_max + 2, 0);
    for (size_t k = 0; k < groups.size(); ++k) ++first[cost_max - (uint32_t)keys[k] + 1];
    for (size_t b = 1; b < first.size(); ++b) first[b] += first[b - 1];
    for (size_t k = 0; k < groups.size(); ++k) order[first[cost_max - (uint32_t)keys[k]]++] = (int32_t)k;
  } else {
    for (size_t k = 0; k < keys.size(); ++k) keys[k] = ((uint64_t)(0xffffffffu - (uint32_t)keys[k]) << 32) | (uint64_t)k;
    std::sort(keys.begin(), keys.end());
    for (size_t k = 0; k < order.size(); ++k) order[k] = (int32_t)(keys[k] & 0xffffffffu);
  }
  // deal the groups to the lanes: first pass sizes the lanes, second pass places the items
  int64_t lane_cost[kNumXcd] = {0, 0, 0, 0, 0, 0, 0, 0};
  size_t lane_len[kNumXcd] = {0, 0, 0, 0, 0, 0, 0, 0};
  std::vector<int8_t>& lane_of = hp.scratch_lane;
  lane_of.resize(groups.size());
  for (int32_t gi : order) {
    // Ties go to the first lane at or after (request + split) mod 8.  With a fixed first lane
    // the kv heads of every request (equal costs, dealt one after the other) would land on
    // the same lanes again and again, i.e. XCD x would read only head x of every page: one
    // 4 KB-aligned slice of the address space per XCD (no difference measured on the
    // high-load configuration, where it happens; kept so that no layout can make it matter).
    const int first = (groups[gi].req + groups[gi].split) & (kNumXcd - 1);
    int best = first;
    for (int k = 1; k < kNumXcd; ++k) {
      const int x = (first + k) & (kNumXcd - 1);
      if (lane_cost[x] < lane_cost[best]) best = x;
    }
    lane_of[gi] = (int8_t)best;
    lane_cost[best] += (int64_t)groups[gi].cost10 * groups[gi].n_row_tiles;
    lane_len[best] += groups[gi].n_row_tiles;
  }
  // work-list index of depth d in lane x = number of items at smaller (depth, lane); lanes
  // shorter than d have dropped out of the round-robin.  Tabulated once: lane_pos[x] + d.
  size_t lane_first[kNumXcd + 1];
  lane_first[0] = 0;
  for (int x = 0; x < kNumXcd; ++x) lane_first[x + 1] = lane_first[x] + lane_len[x];
  std::vector<int32_t>& pos = hp.scratch_pos;   // pos[lane_first[x] + d] = work-list index
  pos.resize(n_items);
  {
    size_t max_len = 0;
    for (int x = 0; x < kNumXcd; ++x) max_len = std::max(max_len, lane_len[x]);
    int32_t next = 0;
    for (size_t d = 0; d < max_len; ++d)
      for (int x = 0; x < kNumXcd; ++x)
        if (lane_len[x] > d) pos[lane_first[x] + d] = next++;
  }
  hp.items.resize(n_items);
  // Where the item of cost rank r of a lane goes (depth in the lane).  The workgroups of a launch
  // are handed to the compute units of a die round-robin, two per unit, so the items at depths d
  // and d + C of a lane (C = units per die) share a unit for their whole life, and a unit
  // works through the tiles of its two items at a rate that hardly depends on how they are
  // split between the two (measured per-unit time stamps on a mixed-chunk batch: unit loads
  // differed by 2x and the kernel lasted as long as the most loaded unit).  So the second C items of a
  // lane are placed in ascending order: the costliest item shares its unit with the cheapest
  // of the first 2C.  Later items start as units free up and keep the costliest-first order.
  const size_t units = (size_t)std::max(1, num_cus / kNumXcd);
  auto depth_of_rank = [units](size_t r, size_t lane_items) {
    const size_t first_round = std::min(lane_items, 2 * units);
    return (r >= units && r < first_round) ? units + (first_round - 1 - r) : r;
  };
  size_t lane_fill[kNumXcd] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int32_t gi : order) {
    const Group& gr = groups[gi];
    const int x = lane_of[gi];
    const int rows = (cu_q[gr.req + 1] - cu_q[gr.req]) * G;
    for (int rt = 0; rt < gr.n_row_tiles; ++rt) {
      const int r0 = rt * kMaxRowsPerItem, rc = std::min(kMaxRowsPerItem, rows - r0);
      optimus_work_item_t it{};
      it.req = gr.req; it.kv_head = gr.kv_head; it.row_begin = r0; it.row_count = rc;
      it.kv_begin = gr.kv_begin; it.kv_end = gr.kv_end;
      it.q_token0 = cu_q[gr.req];
      it.part_row = -1;
      if (gr.n_splits > 1) {
        const MergeItem& m = hp.merges[hp.req_first_merge[gr.req] + gr.kv_head * gr.n_row_tiles + rt];
        it.part_row = m.first_part_row + gr.split * rc;
      }
      hp.items[pos[lane_first[x] + depth_of_rank(lane_fill[x]++, lane_len[x])]] = it;
    }
  }
  hp.part_rows = part_rows;
  hp.workspace_bytes = (size_t)part_rows * (size_t)(p.head_dim + 2) * sizeof(float);
  return OPTIMUS_OK;
}

}  // namespace optimus
