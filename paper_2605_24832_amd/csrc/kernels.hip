// gfx950 (CDNA4) kernels of the chunked block-diffusion attention step
// (Optimus Sec. 6: paged attention over variable-length query chunks, plus
// the mapping of per-chunk KV into the paged cache).
//
// One attention kernel, one workgroup of 4 wave64 per work item = (request, kv
// head, <= 128 query rows, key range).  The rows of a (request, kv head) pair
// are all G query heads of the group x the chunk tokens, so K/V are fetched
// once per group.  Both products are transposed,
//       S^T = K Q^T   (v_mfma_f32_16x16x32_bf16, A = K tile, B = Q^T)
//       O^T = V^T P^T (A = V^T tile, B = P^T)
// which leaves the S^T accumulator of a lane exactly in the B-operand layout
// the second product needs, so P never moves between lanes; only the row max
// crosses lanes (two lane-swap steps over the 4 lane groups), and the row sum
// comes out of one more MFMA against a ones operand.
//
//   <= 16 rows ("split-wave" body): the 4 waves take the 32-key tiles of the
//   range round-robin, K and V go from HBM straight into MFMA operand
//   registers (the pool layout, K in 16-byte d-groups slot-major and V
//   slot-contiguous, makes every wave-wide load a contiguous run), each wave
//   keeps its own online-softmax state and the waves are merged through LDS.
//
//   17..32 rows ("lds-tile" body): all waves walk the same tiles, staged once
//   per workgroup in LDS, and each wave owns 16 of the rows.
//
//   pairs with more than 32 rows ("wide" body, further down): 32 rows per wave,
//   32x32x16 MFMA, tiles loaded from global memory straight into LDS.
//
// Key ranges split over several work items leave partials that the merge
// kernel combines (a fused "last block merges" variant was measured 4x slower:
// a device-scope fence on this multi-die part writes back and invalidates L2).
//
// 16x16x32 bf16 MFMA register layout (lane = 16*kg + r, kg 0..3, r 0..15):
//   A: row r,  k = 8*kg .. 8*kg+7      B: col r, k = 8*kg .. 8*kg+7
//   C/D: 4 floats, rows 4*kg .. 4*kg+3, col r
#include <hip/hip_runtime.h>

#include <cstring>

#include <mutex>

#include "plan_internal.h"

namespace optimus {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int W = kWavesPerBlock;
constexpr float kMaxSlack = 8.0f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Reductions over the 4 lane groups {l, l^16, l^32, l^48} with the gfx950 lane-swap
// instructions (plain VALU ops, no LDS-crossbar round trip).  With both operands equal to
// v, v_permlane16_swap returns (rows 0,0,2,2 ; rows 1,1,3,3) of v (row = 16 lanes) and
// v_permlane32_swap returns (low half twice ; high half twice); checked on the device.
// The results are copied to scalars before the bit cast: a bit cast applied directly to a
// vector subscript was seen to read element 0 for both.
__device__ __forceinline__ void swap16(float v, float& x, float& y) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned r0 = r[0], r1 = r[1];
  x = __builtin_bit_cast(float, r0);
  y = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ void swap32(float v, float& x, float& y) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const unsigned r0 = r[0], r1 = r[1];
  x = __builtin_bit_cast(float, r0);
  y = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float xor_max(float v) {
  float x, y;
  swap16(v, x, y);
  v = fmaxf(x, y);
  swap32(v, x, y);
  return fmaxf(x, y);
}
__device__ __forceinline__ float xor_sum(float v) {
  float x, y;
  swap16(v, x, y);
  v = x + y;
  swap32(v, x, y);
  return x + y;
}

// Block-causal mode (mask_mode 1): first logical key that chunk query j of the item's request may
// not see.  Without explicit positions the chunk follows the d_in cached tokens of the block
// contiguously.  With positions (q_pos, non-decreasing within a request's chunk): the chunk keys
// whose position lies before the end of query j's block, counted (for non-decreasing positions
// these are exactly the keys of blocks up to the query's).
__device__ __forceinline__ int block_causal_end(const KernelArgs& a, const optimus_work_item_t& it, int L,
                                                int d_in, int j) {
  const int B = a.block_size;
  if (!a.q_pos) return L + ((d_in + j) / B + 1) * B - d_in;
  const int32_t* pos = a.q_pos + it.q_token0;
  const int c = a.cu_q[it.req + 1] - it.q_token0;
  const int s = L - d_in;
  const int end_pos = s + ((pos[j] - s) / B + 1) * B;   // first position of the next block
  int n = 0;
  for (int k = 0; k < c; ++k) n += pos[k] < end_pos ? 1 : 0;
  return L + n;
}
// First key any query of the request might not see (wave-uniform); with explicit positions
// every tile that holds chunk keys takes the masked path.
__device__ __forceinline__ int block_causal_min(const KernelArgs& a, int L, int d_in) {
  const int B = a.block_size;
  return a.q_pos ? L : L + (d_in / B + 1) * B - d_in;
}

template <int D>
struct KvTile {
  bf16x8 k[2][D / 32];   // [16-key half][d step of 32]
  u32x2 v[D / 16][2];    // [16-wide d block][16-key half] : 4 keys x bf16
};

// Page ids of one 32-key tile (two pages at P = 16, else one).
struct TilePages { int32_t p0, p1; };

// `bt` is the request's block-table row, `last_page` the index of the last page that holds
// a key of this item, `tile_max` the item's last tile.  The tile index is clamped so that a
// look-ahead past the end still reads a valid entry.
// The table is read through the constant address space: no kernel of this library writes a
// block table, and only so does the compiler keep these uniform loads on the scalar unit
// (it otherwise sees stores to global memory in the same kernel and issues them as
// vector loads, which queue in the same counter as the K/V loads).
typedef const int32_t __attribute__((address_space(4)))* ConstI32Ptr;
template <int LGP>
__device__ __forceinline__ TilePages tile_pages(const int32_t* __restrict__ bt_generic, int tile, int tile_max,
                                                int last_page) {
  const ConstI32Ptr bt = (ConstI32Ptr)(uintptr_t)bt_generic;
  tile = min(tile, tile_max);
  if constexpr (LGP == 4) {
    // the second page may lie beyond the request's last page (then its keys are all
    // masked): clamp so the loads stay in a valid page
    const int pi0 = tile * 2;
    return TilePages{bt[pi0], bt[min(pi0 + 1, last_page)]};
  } else {
    const int32_t pg = bt[(tile * kTileTokens) >> LGP];
    return TilePages{pg, pg};
  }
}

// Issue the loads of one 32-key tile whose page ids are already known.
// K/V of the two narrow bodies are read exactly once per launch (a pair of at most 32 rows has
// a single row tile), so they are loaded with the non-temporal hint: measured 9 % faster on the
// memory-bound configuration (853 -> 774 us, 6.56 TB/s) than plain loads, which let the
// stream displace itself in the caches.  The wide body keeps plain loads: its sibling row
// tiles find the stream in L2, and the hint made it slower.
template <typename T>
__device__ __forceinline__ T stream_load(const T* p) { return __builtin_nontemporal_load(p); }
template <int D, int LGP>
__device__ __forceinline__ void load_tile(KvTile<D>& t, int tile, TilePages pg,
                                          const char* __restrict__ kbase,
                                          const char* __restrict__ vbase, int64_t k_stride_page_b,
                                          int64_t v_stride_page_b, int r16, int kg) {
  constexpr int P = 1 << LGP;
  constexpr int KS = D / 32, DB = D / 16;
  if constexpr (LGP == 4) {
    const char* k0 = kbase + (int64_t)pg.p0 * k_stride_page_b;
    const char* k1 = kbase + (int64_t)pg.p1 * k_stride_page_b;
    const char* v0 = vbase + (int64_t)pg.p0 * v_stride_page_b;
    const char* v1 = vbase + (int64_t)pg.p1 * v_stride_page_b;
    const uint32_t koff = (uint32_t)(kg * P + r16) * 16u;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      t.k[0][s] = stream_load(reinterpret_cast<const bf16x8*>(k0 + koff + s * (4 * P * 16)));
      t.k[1][s] = stream_load(reinterpret_cast<const bf16x8*>(k1 + koff + s * (4 * P * 16)));
    }
    const uint32_t voff = (uint32_t)(r16 * P + 4 * kg) * 2u;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      t.v[db][0] = stream_load(reinterpret_cast<const u32x2*>(v0 + voff + db * (16 * P * 2)));
      t.v[db][1] = stream_load(reinterpret_cast<const u32x2*>(v1 + voff + db * (16 * P * 2)));
    }
  } else {
    const int slot0 = (tile * kTileTokens) & (P - 1);
    const char* k0 = kbase + (int64_t)pg.p0 * k_stride_page_b;
    const char* v0 = vbase + (int64_t)pg.p0 * v_stride_page_b;
    const uint32_t koff = (uint32_t)(kg * P + slot0 + r16) * 16u;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      t.k[0][s] = stream_load(reinterpret_cast<const bf16x8*>(k0 + koff + s * (4 * P * 16)));
      t.k[1][s] = stream_load(reinterpret_cast<const bf16x8*>(k0 + koff + s * (4 * P * 16) + 16 * 16));
    }
    const uint32_t voff = (uint32_t)(r16 * P + slot0 + 4 * kg) * 2u;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      t.v[db][0] = stream_load(reinterpret_cast<const u32x2*>(v0 + voff + db * (16 * P * 2)));
      t.v[db][1] = stream_load(reinterpret_cast<const u32x2*>(v0 + voff + db * (16 * P * 2) + 16 * 2));
    }
  }
}

template <int D, int NT>
struct SoftmaxState {
  float m[NT];            // running max (log2 units), replicated over the 4 lane groups
  f32x4 lacc[NT];         // running sum of P over the keys, from an MFMA against a ones operand
                          // (all 4 entries equal): rescaled and accumulated exactly like acc
  f32x4 acc[NT][D / 16];  // O^T: rows d = 16*db + 4*kg + j, col = query row r16
};

__device__ __forceinline__ bf16x8 ones_bf16x8() {
  const u32x4 o = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
  return __builtin_bit_cast(bf16x8, o);
}

// One 32-key tile against NT x 16 query rows, operands already in registers.
//   k[a][s]: A operand of S^T for the a-th group of 16 keys, d step s
//   v[db]:   A operand of O^T for d block db; its 8 k-slots must be the keys of
//            this lane's score registers, s0[0..3] then s1[0..3], and the
//            elements of keys at or beyond kv_end must already be zero
//   key0/key1: logical slot of the key behind s0[0] / s1[0] of this lane
//   lim:     per subtile, first key this lane's query row may not see
//            (only looked at when `masked`)
template <int D, int NT>
__device__ __forceinline__ void compute_tile(SoftmaxState<D, NT>& st, const bf16x8 (&k)[2][D / 32],
                                             const bf16x8 (&v)[D / 16],
                                             const bf16x8 (&qreg)[NT][D / 32], int key0, int key1,
                                             const int (&lim)[NT], bool masked, float sc) {
  constexpr int KS = D / 32, DB = D / 16;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[0][s], qreg[nt][s], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[1][s], qreg[nt][s], s1, 0, 0, 0);
    }
    if (masked) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        s0[j] = key0 + j < lim[nt] ? s0[j] : -INFINITY;
        s1[j] = key1 + j < lim[nt] ? s1[j] : -INFINITY;
      }
    }
    float mx = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])),
                     fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
    mx = xor_max(mx);
    // The reference value m of the online softmax only has to keep exp2(s - m) in range:
    // it follows the running maximum lazily, moving only when the maximum has grown by more
    // than kMaxSlack (in log2 units), so p <= 2^kMaxSlack and the accumulators are rescaled
    // on few tiles.  All lanes of a query column hold the same mx, hence take the same branch.
    const float m_cand = fmaxf(st.m[nt], mx * sc);
    const float m_new = (m_cand - st.m[nt] > kMaxSlack) ? m_cand : st.m[nt];  // -inf -> first finite max
    const float m_use = m_new == -INFINITY ? 0.f : m_new;  // row with no visible key so far
    const float alpha = fast_exp2(st.m[nt] - m_use);
    st.m[nt] = m_new;
    float p[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      p[j] = fast_exp2(fmaf(s0[j], sc, -m_use));
      p[4 + j] = fast_exp2(fmaf(s1[j], sc, -m_use));
    }
    bf16x8 pt;
#pragma unroll
    for (int j = 0; j < 8; ++j) pt[j] = (__bf16)p[j];
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {  // wave-uniform: some column moved its m
#pragma unroll
      for (int db = 0; db < DB; ++db) st.acc[nt][db] *= alpha;
      st.lacc[nt] *= alpha;
    }
    // row sums of the bf16 P actually used in the product: one more MFMA, no VALU adds
    st.lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones_bf16x8(), pt, st.lacc[nt], 0, 0, 0);
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      st.acc[nt][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v[db], pt, st.acc[nt][db], 0, 0, 0);
    }
  }
}

// Keep the first `cnt` of the 2 x bf16 halves (cnt <= 0: none, >= 2: both).
__device__ __forceinline__ uint32_t keep_mask(int cnt) {
  return cnt >= 2 ? 0xffffffffu : (cnt == 1 ? 0x0000ffffu : 0u);
}

// Shared memory of the split-wave body, in floats.
template <int D, int NT>
constexpr int split_wave_smem_floats() { return W * 16 * (D + 4) + 2 * W * NT * 16; }

template <int D, int LGP, int NT>
__device__ __forceinline__ void split_wave_body(const KernelArgs& a, const optimus_work_item_t& it,
                                                float* smem) {
  constexpr int KS = D / 32, DB = D / 16;
  constexpr int OPAD = D + 4;
  float (*sm_o)[16][OPAD] = reinterpret_cast<float (*)[16][OPAD]>(smem);
  float (*sm_m)[NT * 16] = reinterpret_cast<float (*)[NT * 16]>(smem + W * 16 * OPAD);
  float (*sm_l)[NT * 16] = reinterpret_cast<float (*)[NT * 16]>(smem + W * 16 * OPAD + W * NT * 16);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r16 = lane & 15, kg = lane >> 4;
  const int G = a.group;

  // ---- start-up: page ids (scalar loads) and Q (vector loads) are requested together, and the
  // first K/V tile goes out as soon as the page ids are there, without waiting for Q: nothing
  // of Q is looked at before those loads are issued.  (Per-phase time stamps of a batch of one
  // request: page ids 0.2 us; issuing the first tiles of the unit's eight waves, 128 KB through
  // a 64 B/clk path, 3 us; their arrival 1.3 us more.)
  const int32_t* bt = a.block_table + (int64_t)it.req * a.max_pages_per_req;
  const int last_page = (it.kv_end - 1) >> LGP;
  const char* kbase = reinterpret_cast<const char*>(a.k_pool + (int64_t)it.kv_head * a.k_stride_head);
  const char* vbase = reinterpret_cast<const char*>(a.v_pool + (int64_t)it.kv_head * a.v_stride_head);
  const int64_t kspb = a.k_stride_page * 2, vspb = a.v_stride_page * 2;
  const float sc = a.scale_log2;

  const int tile_lo = it.kv_begin / kTileTokens;
  const int tile_hi = (it.kv_end + kTileTokens - 1) / kTileTokens;
  // this wave's tiles: tile_lo + wave + W*i, i in [0, n)
  const int n = (tile_hi - tile_lo - wave + W - 1) / W;
  const int t0 = tile_lo + wave;

  KvTile<D> ta, tb;
  auto PAGES = [&](int i) { return tile_pages<LGP>(bt, t0 + W * i, tile_hi - 1, last_page); };
  auto LOAD = [&](KvTile<D>& t, int i, TilePages pg) {
    load_tile<D, LGP>(t, t0 + W * i, pg, kbase, vbase, kspb, vspb, r16, kg);
  };
  // page ids of the wave's first three tiles (the index is clamped: valid also without tiles)
  TilePages pg0 = PAGES(0), pg1 = PAGES(1), pg2 = PAGES(2);

  // ---- Q^T B operands: col r16 = query row, k = d ----
  bf16x8 qreg[NT][KS];
  int vis_end[NT];
  // cached length and block offset only matter for the block-causal mask: keep their loads
  // (which depend on the item's own load) off the start-up path of the plain mode
  int L = 0, d_in = 0;
  if (a.mask_mode != 0) {
    L = a.prefix_len[it.req];
    d_in = L - a.block_start[it.req];
  }
  u32x4 qraw[NT][KS];
  int q_j[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int rl = nt * 16 + r16;
    const bool valid = rl < it.row_count;
    const int row = it.row_begin + (valid ? rl : 0);
    const int j = row / G, u = row - j * G;
    q_j[nt] = j;
    const uint16_t* qp =
        a.q + ((int64_t)(it.q_token0 + j) * a.num_q_heads + it.kv_head * G + u) * D + kg * 8;
#pragma unroll
    for (int s = 0; s < KS; ++s) qraw[nt][s] = *reinterpret_cast<const u32x4*>(qp + s * 32);
  }
  // the first tile's loads go out as soon as the page ids are there, behind the Q loads
  if (n > 0) LOAD(ta, 0, pg0);
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const bool valid = nt * 16 + r16 < it.row_count;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      u32x4 x = qraw[nt][s];
      if (!valid) x = u32x4{0u, 0u, 0u, 0u};
      qreg[nt][s] = __builtin_bit_cast(bf16x8, x);
    }
    // block-causal variant: chunk key k visible iff (d_in+k)/B <= (d_in+j)/B
    vis_end[nt] = a.mask_mode == 0 ? INT32_MAX : block_causal_end(a, it, L, d_in, q_j[nt]);
  }
  // first key any row of the request might not see (uniform)
  const int vis_min = a.mask_mode == 0 ? INT32_MAX : block_causal_min(a, L, d_in);
  const int mask_from = min(it.kv_end, vis_min);

  SoftmaxState<D, NT> st;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    st.m[nt] = -INFINITY;
    st.lacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int db = 0; db < DB; ++db) st.acc[nt][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  auto COMPUTE = [&](KvTile<D>& t, int i) {
    const int key_base = (t0 + W * i) * kTileTokens;
    const bool masked = key_base + kTileTokens > mask_from;
    // this lane's score registers: keys 4kg..4kg+3 of each 16-key half
    const int key0 = key_base + 4 * kg, key1 = key0 + 16;
    if (masked) {
      // zero V of keys outside the item so that 0 * garbage cannot become NaN
      const uint32_t m00 = keep_mask(it.kv_end - key0), m01 = keep_mask(it.kv_end - key0 - 2);
      const uint32_t m10 = keep_mask(it.kv_end - key1), m11 = keep_mask(it.kv_end - key1 - 2);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        t.v[db][0].x &= m00; t.v[db][0].y &= m01;
        t.v[db][1].x &= m10; t.v[db][1].y &= m11;
      }
    }
    bf16x8 vop[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      u32x4 vv = {t.v[db][0].x, t.v[db][0].y, t.v[db][1].x, t.v[db][1].y};
      vop[db] = __builtin_bit_cast(bf16x8, vv);
    }
    int lim[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) lim[nt] = min(it.kv_end, vis_end[nt]);
    compute_tile<D, NT>(st, t.k, vop, qreg, key0, key1, lim, masked, sc);
  };
  // Page ids are fetched two tiles ahead of their K/V loads: the memory counter retires in
  // order, so an id requested right before its use would wait behind the whole previous
  // tile and the next tile's loads could not be issued until that one had arrived.
  if (n > 0) {
    TilePages p1 = pg1, p2 = pg2;
    int i = 0;
    while (i + 2 < n) {
      const TilePages p3 = PAGES(i + 3);
      LOAD(tb, i + 1, p1);
      COMPUTE(ta, i);
      const TilePages p4 = PAGES(i + 4);
      LOAD(ta, i + 2, p2);
      COMPUTE(tb, i + 1);
      p1 = p3;
      p2 = p4;
      i += 2;
    }
    if (i + 1 < n) {
      LOAD(tb, i + 1, p1);
      COMPUTE(ta, i);
      COMPUTE(tb, i + 1);
    } else {
      COMPUTE(ta, i);
    }
  }

  // ---- merge the W waves through LDS ----
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const float lsum = st.lacc[nt][0];
    if (kg == 0) {
      sm_m[wave][nt * 16 + r16] = st.m[nt];
      sm_l[wave][nt * 16 + r16] = lsum;
    }
  }
  __syncthreads();
  float own_scale[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < W; ++w) M = fmaxf(M, sm_m[w][nt * 16 + r16]);
    const float Mu = M == -INFINITY ? 0.f : M;
    own_scale[nt] = fast_exp2(st.m[nt] - Mu);
  }
  const int tid = threadIdx.x;
  constexpr int CH = D / 16;              // floats per thread in the reduction (8 or 4)
  const int orow = tid >> 4, ocol = (tid & 15) * CH;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if (nt * 16 < it.row_count) {  // uniform
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        f32x4 v = st.acc[nt][db] * own_scale[nt];
        *reinterpret_cast<f32x4*>(&sm_o[wave][r16][db * 16 + 4 * kg]) = v;
      }
    }
    __syncthreads();
    const int rl = nt * 16 + orow;
    if (rl < it.row_count) {
      float M = -INFINITY;
#pragma unroll
      for (int w = 0; w < W; ++w) M = fmaxf(M, sm_m[w][rl]);
      const float Mu = M == -INFINITY ? 0.f : M;
      float lt = 0.f;
#pragma unroll
      for (int w = 0; w < W; ++w) lt += fast_exp2(sm_m[w][rl] - Mu) * sm_l[w][rl];
      float o[CH];
#pragma unroll
      for (int c = 0; c < CH; ++c) o[c] = 0.f;
#pragma unroll
      for (int w = 0; w < W; ++w)
#pragma unroll
        for (int c = 0; c < CH; c += 4) {
          f32x4 v = *reinterpret_cast<const f32x4*>(&sm_o[w][orow][ocol + c]);
          o[c] += v[0]; o[c + 1] += v[1]; o[c + 2] += v[2]; o[c + 3] += v[3];
        }
      if (it.part_row >= 0) {
        float* po = a.ws_o + (int64_t)(it.part_row + rl) * D + ocol;
#pragma unroll
        for (int c = 0; c < CH; c += 4)
          *reinterpret_cast<f32x4*>(po + c) = f32x4{o[c], o[c + 1], o[c + 2], o[c + 3]};
        if ((tid & 15) == 0) {
          float* pml = a.ws_ml + (int64_t)(it.part_row + rl) * 2;
          pml[0] = M;
          pml[1] = lt;
        }
      } else {
        const float inv = 1.f / lt;
        const int row = it.row_begin + rl;
        const int j = row / G, u = row - j * G;
        const int64_t off = ((int64_t)(it.q_token0 + j) * a.num_q_heads + it.kv_head * G + u) * D + ocol;
        if (a.out_fp32) {
          float* po = reinterpret_cast<float*>(a.out) + off;
#pragma unroll
          for (int c = 0; c < CH; c += 4)
            *reinterpret_cast<f32x4*>(po + c) =
                f32x4{o[c] * inv, o[c + 1] * inv, o[c + 2] * inv, o[c + 3] * inv};
        } else {
          __bf16* po = reinterpret_cast<__bf16*>(a.out) + off;
#pragma unroll
          for (int c = 0; c < CH; c += 4) {
            bf16x4 b;
#pragma unroll
            for (int e = 0; e < 4; ++e) b[e] = (__bf16)(o[c + e] * inv);
            *reinterpret_cast<bf16x4*>(po + c) = b;
          }
        }
      }
    }
    __syncthreads();
  }
}

// attention body for medium row tiles ("lds-tile"): up to 64*NT query rows per
// work item (instantiated with NT = 1; wider pairs take the wide body).  All 4 waves walk the same 32-key tiles, staged once per workgroup
// in LDS (coalesced global loads -> registers -> ds_write, double-buffered, two
// tiles of loads in flight), and each wave owns NT x 16 of the rows, so K/V
// leave HBM once however many query heads and chunk tokens share them.
// LDS layouts are chosen so that every operand read is a conflict-free
// ds_read_b128:
//   K: [d group of 8][position][8] with the 32 keys in MFMA row order: key
//      8x+4a+y (x 0..3, a 0..1, y 0..3) at position 16a+4x+y, so that the two
//      S^T products of a lane yield keys 8kg..8kg+7, the k-slots of one
//      16-byte V^T operand;
//   V: [key octet 0..3][d][8 keys].
// Both are XOR-swizzled at 16-byte granularity (K: position ^ 4 in the second half of a
// d group; V: d ^ 2*octet) so that the 8 lanes one LDS cycle serves hit 8 different
// 16-byte bank groups on the cooperative stores as well as on the operand reads.
template <int D>
constexpr int lds_tile_smem_floats() { return 4 * (D * 4) * 4; }  // 2 x (K + V) tiles of D*4 x 16 bytes

template <int D, int LGP, int NT>
__device__ __forceinline__ void lds_tile_body(const KernelArgs& a, const optimus_work_item_t& it,
                                              float* smem) {
  constexpr int KS = D / 32, DB = D / 16, P = 1 << LGP;
  constexpr int PIECES = D * 4;        // 16-byte pieces of a K (= of a V) tile
  constexpr int LPT = PIECES / 256;    // pieces per thread per tensor per tile
  constexpr int PF = 2;                // register sets of prefetched tiles
  u32x4 (*sm_k)[PIECES] = reinterpret_cast<u32x4 (*)[PIECES]>(smem);
  u32x4 (*sm_v)[PIECES] = reinterpret_cast<u32x4 (*)[PIECES]>(smem + 2 * PIECES * 4);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r16 = lane & 15, kg = lane >> 4;
  const int G = a.group;

  bf16x8 qreg[NT][KS];
  int vis_end[NT];
  // cached length and block offset only matter for the block-causal mask: keep their loads
  // (which depend on the item's own load) off the start-up path of the plain mode
  int L = 0, d_in = 0;
  if (a.mask_mode != 0) {
    L = a.prefix_len[it.req];
    d_in = L - a.block_start[it.req];
  }
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int rl = (wave * NT + nt) * 16 + r16;
    const bool valid = rl < it.row_count;
    const int row = it.row_begin + (valid ? rl : 0);
    const int j = row / G, u = row - j * G;
    const uint16_t* qp =
        a.q + ((int64_t)(it.q_token0 + j) * a.num_q_heads + it.kv_head * G + u) * D + kg * 8;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      u32x4 x = *reinterpret_cast<const u32x4*>(qp + s * 32);
      if (!valid) x = u32x4{0u, 0u, 0u, 0u};
      qreg[nt][s] = __builtin_bit_cast(bf16x8, x);
    }
    vis_end[nt] = a.mask_mode == 0 ? INT32_MAX : block_causal_end(a, it, L, d_in, j);
  }
  const int vis_min = a.mask_mode == 0 ? INT32_MAX : block_causal_min(a, L, d_in);
  const int mask_from = min(it.kv_end, vis_min);
  const bool wave_has_rows = wave * NT * 16 < it.row_count;  // uniform per wave

  SoftmaxState<D, NT> st;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    st.m[nt] = -INFINITY;
    st.lacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int db = 0; db < DB; ++db) st.acc[nt][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int32_t* bt = a.block_table + (int64_t)it.req * a.max_pages_per_req;
  const int last_page = (it.kv_end - 1) >> LGP;
  const char* kbase = reinterpret_cast<const char*>(a.k_pool + (int64_t)it.kv_head * a.k_stride_head);
  const char* vbase = reinterpret_cast<const char*>(a.v_pool + (int64_t)it.kv_head * a.v_stride_head);
  const int64_t kspb = a.k_stride_page * 2, vspb = a.v_stride_page * 2;
  const float sc = a.scale_log2;
  const int tile_lo = it.kv_begin / kTileTokens;
  const int n = (it.kv_end + kTileTokens - 1) / kTileTokens - tile_lo;

  // per-thread piece geometry (tile invariant)
  uint32_t ksrc[LPT], vsrc[LPT];   // byte offset inside the page (P = 16) or before slot0 is added
  int kdst[LPT], vdst[LPT];        // piece index in the LDS tile
  bool second_page[LPT][2];        // P = 16: piece comes from the tile's second page (K, V)
#pragma unroll
  for (int i = 0; i < LPT; ++i) {
    const int e = tid + 256 * i;
    const int chunk = e >> 5, kit = e & 31;
    const int pos = (((kit >> 2) & 1) << 4) + ((kit >> 3) << 2) + (kit & 3);
    kdst[i] = chunk * 32 + (pos ^ ((pos >> 4) << 2));   // bank swizzle, see the reads
    const int dd = e >> 2, q4 = e & 3;
    vdst[i] = q4 * D + (dd ^ (q4 << 1));                // bank swizzle, see the reads
    if constexpr (LGP == 4) {
      ksrc[i] = (uint32_t)(chunk * 16 + (kit & 15)) * 16u;
      vsrc[i] = (uint32_t)(dd * 32 + (q4 & 1) * 16);
      second_page[i][0] = kit >= 16;
      second_page[i][1] = q4 >= 2;
    } else {
      ksrc[i] = (uint32_t)(chunk * P + kit) * 16u;
      vsrc[i] = (uint32_t)(dd * P + 8 * q4) * 2u;
      second_page[i][0] = second_page[i][1] = false;
    }
  }

  u32x4 rk[PF][LPT], rv[PF][LPT];
  // page ids of item tile t (clamped to the item's last tile)
  auto PAGES = [&](int t) { return tile_pages<LGP>(bt, tile_lo + t, tile_lo + n - 1, last_page); };
  auto LOAD = [&](int set, int t, TilePages pg) {   // tile t of the item -> registers
    const int tile = tile_lo + t;
    if constexpr (LGP == 4) {
#pragma unroll
      for (int i = 0; i < LPT; ++i) {
        const char* kp = kbase + (int64_t)(second_page[i][0] ? pg.p1 : pg.p0) * kspb;
        const char* vp = vbase + (int64_t)(second_page[i][1] ? pg.p1 : pg.p0) * vspb;
        rk[set][i] = stream_load(reinterpret_cast<const u32x4*>(kp + ksrc[i]));
        rv[set][i] = stream_load(reinterpret_cast<const u32x4*>(vp + vsrc[i]));
      }
    } else {
      const uint32_t slot0 = (uint32_t)((tile * kTileTokens) & (P - 1));
      const char* kp = kbase + (int64_t)pg.p0 * kspb + slot0 * 16u;
      const char* vp = vbase + (int64_t)pg.p0 * vspb + slot0 * 2u;
#pragma unroll
      for (int i = 0; i < LPT; ++i) {
        rk[set][i] = stream_load(reinterpret_cast<const u32x4*>(kp + ksrc[i]));
        rv[set][i] = stream_load(reinterpret_cast<const u32x4*>(vp + vsrc[i]));
      }
    }
  };
  auto STORE = [&](int buf, int set) {  // registers -> LDS tile
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      sm_k[buf][kdst[i]] = rk[set][i];
      sm_v[buf][vdst[i]] = rv[set][i];
    }
  };
  auto COMPUTE = [&](int buf, int t) {
    if (!wave_has_rows) return;
    const int key_base = (tile_lo + t) * kTileTokens;
    const bool masked = key_base + kTileTokens > mask_from;
    const int key0 = key_base + 8 * kg, key1 = key0 + 4;
    bf16x8 kop[2][KS], vop[DB];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      kop[0][s] = __builtin_bit_cast(bf16x8, sm_k[buf][(4 * s + kg) * 32 + r16]);
      kop[1][s] = __builtin_bit_cast(bf16x8, sm_k[buf][(4 * s + kg) * 32 + 16 + (r16 ^ 4)]);
    }
    if (masked) {
      const int cnt = it.kv_end - key0;
      const uint32_t m0 = keep_mask(cnt), m1 = keep_mask(cnt - 2), m2 = keep_mask(cnt - 4),
                     m3 = keep_mask(cnt - 6);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        u32x4 vv = sm_v[buf][kg * D + 16 * db + (r16 ^ (kg << 1))];
        vv.x &= m0; vv.y &= m1; vv.z &= m2; vv.w &= m3;
        vop[db] = __builtin_bit_cast(bf16x8, vv);
      }
    } else {
#pragma unroll
      for (int db = 0; db < DB; ++db)
        vop[db] = __builtin_bit_cast(bf16x8, sm_v[buf][kg * D + 16 * db + (r16 ^ (kg << 1))]);
    }
    int lim[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) lim[nt] = min(it.kv_end, vis_end[nt]);
    compute_tile<D, NT>(st, kop, vop, qreg, key0, key1, lim, masked, sc);
  };

  // Software pipeline: at the top of iteration t LDS buffer t%2 holds tile t and register
  // set (t+k)%PF holds tile t+k for k = 1..PF (global loads in flight).  The loop is
  // unrolled by a multiple of 2 and PF so that every buffer / set index is a constant.
  constexpr int UNROLL = (PF % 2 == 0) ? PF : 2 * PF;
#pragma unroll
  for (int s0 = 0; s0 < PF; ++s0)
    if (s0 < n) LOAD(s0, s0, PAGES(s0));
  STORE(0, 0);
  if (PF < n) LOAD(0, PF, PAGES(PF));
  // Page ids are fetched one iteration before the loads that use them: asked for right before
  // its use, the (scalar) load's latency would be paid in every iteration.
  TilePages pg_next = PAGES(PF + 1);
  __syncthreads();
  // Steady state without a branch between the issue of a tile's loads and their use, so the
  // memory-counter waits the compiler inserts are exact (a conditional load makes it wait for
  // every outstanding load, which would undo the prefetch); the last tiles run in the
  // guarded loop below.
  int t = 0;
  for (; t + UNROLL + PF < n; t += UNROLL) {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      COMPUTE(u & 1, t + u);
      STORE((u + 1) & 1, (u + 1) % PF);
      LOAD((u + 1) % PF, t + u + 1 + PF, pg_next);
      pg_next = PAGES(t + u + 2 + PF);
      __syncthreads();
    }
  }
  for (; t < n; t += UNROLL) {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      if (t + u >= n) break;
      COMPUTE(u & 1, t + u);
      if (t + u + 1 < n) STORE((u + 1) & 1, (u + 1) % PF);
      if (t + u + 1 + PF < n) LOAD((u + 1) % PF, t + u + 1 + PF, pg_next);
      pg_next = PAGES(t + u + 2 + PF);
      __syncthreads();
    }
  }

  // ---- each wave owns its rows: finish them without any cross-wave step ----
  if (!wave_has_rows) return;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int rl = (wave * NT + nt) * 16 + r16;
    const float lsum = st.lacc[nt][0];
    if (rl >= it.row_count) continue;
    if (it.part_row >= 0) {
      float* po = a.ws_o + (int64_t)(it.part_row + rl) * D + 4 * kg;
#pragma unroll
      for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4*>(po + 16 * db) = st.acc[nt][db];
      if (kg == 0) {
        float* pml = a.ws_ml + (int64_t)(it.part_row + rl) * 2;
        pml[0] = st.m[nt];
        pml[1] = lsum;
      }
    } else {
      const float inv = 1.f / lsum;
      const int row = it.row_begin + rl;
      const int j = row / G, u = row - j * G;
      const int64_t off =
          ((int64_t)(it.q_token0 + j) * a.num_q_heads + it.kv_head * G + u) * D + 4 * kg;
      if (a.out_fp32) {
        float* po = reinterpret_cast<float*>(a.out) + off;
#pragma unroll
        for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4*>(po + 16 * db) = st.acc[nt][db] * inv;
      } else {
        __bf16* po = reinterpret_cast<__bf16*>(a.out) + off;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          bf16x4 b;
#pragma unroll
          for (int e = 0; e < 4; ++e) b[e] = (__bf16)(st.acc[nt][db][e] * inv);
          *reinterpret_cast<bf16x4*>(po + 16 * db) = b;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// attention kernel for the widest row tiles ("wide" body): 33..128 query rows.
// Each wave owns 32 rows and both products use the 32x32x16 bf16 MFMA, whose
// register layout (lane = 32*h + r, r 0..31, h 0..1) is
//   A: row r, k = 8h..8h+7     B: col r, k = 8h..8h+7
//   C/D: 16 floats, col r, register v -> row 8*(v/4) + 4h + v%4
// so a lane holds 16 scores of ONE query row per tile: the row maximum crosses
// lanes once, the per-row softmax bookkeeping is paid once per 16 scores, and
// the row sum is a packed bf16 dot product with ones (it adds up exactly the
// rounded P that enters the second product).
// K/V tiles reach LDS without passing through registers (global_load_lds, 16
// bytes per lane; lane i of an instruction writes piece base+i, so the LDS
// layout is produced by choosing which global piece each lane fetches), in a
// ring of kWideStages tiles that is filled three tiles ahead.  The loop is
// software-pipelined: the score product of tile t+1 is issued before the
// softmax of tile t, so MFMA and VALU work of one wave overlap; the waits on
// the load counter are written by hand (the ring is only correct because each
// wave issues exactly 2*LPT loads per tile and nothing else in the loop).
// LDS layouts (16-byte pieces):
//   K: piece 32*g + i holds d group g (8 values) of the key whose score lands in
//      row i of S^T; row i is key (i with bits 2 and 3 swapped), which makes the
//      8 scores a lane packs for one PV product 8 consecutive keys.  The operand
//      of step s is piece 64*s + lane: a contiguous read.
//   V: piece 4*d + (o ^ ((d >> 2) & 3)) holds keys 8o..8o+7 of row d; the XOR
//      spreads the 16 lanes one LDS cycle serves over all banks.
// With 16-key pages a tile spans two pages and the stage holds them one after the other
// exactly as they lie in memory (see the body), so that a load instruction never mixes pages:
// measured 12 % faster than selecting the page per lane (64-bit vector addresses).
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
constexpr int kWideStages = 4;

template <int D>
constexpr int wide_smem_floats() { return kWideStages * 2 * (D * 4) * 4; }

// s_waitcnt with only the vector-memory counter set (gfx9 encoding: vmcnt in bits 3:0 and
// 15:14, the other counters left at "no wait").
#define OPT_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
// Workgroup barrier without a memory fence (a fence would wait for every load in flight);
// the empty asm statements keep the compiler from moving LDS accesses across it.
#define OPT_BARRIER_NO_FENCE()          \
  do {                                  \
    asm volatile("" ::: "memory");      \
    __builtin_amdgcn_s_barrier();       \
    asm volatile("" ::: "memory");      \
  } while (0)

// 16 bytes per lane from global memory straight into LDS: lane i writes lds_addr + 16*i.
// Written as inline asm on purpose: when the compiler sees this instruction it makes every
// memory-counter wait it inserts anywhere in the kernel a wait for all loads, which would undo
// the prefetch of the other bodies.  The compiler therefore does not count these loads; the
// body below waits for them by hand, and a compiler-inserted wait for one of its own loads
// only waits longer than needed (the counter retires in order).  M0 holds the LDS address
// (one wait state between the scalar write of M0 and its use).
// STREAM adds the non-temporal hint (for tiles no other workgroup reads).
template <bool STREAM>
__device__ __forceinline__ void load_to_lds_16(const void* gptr, uint32_t lds_addr) {
  if constexpr (STREAM)
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt"
                 :
                 : "v"(gptr), "s"(lds_addr)
                 : "memory", "m0");
  else
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gptr), "s"(lds_addr)
                 : "memory", "m0");
}

// Same with a wave-uniform base address in scalar registers plus a 32-bit lane offset: no
// vector address arithmetic per load.
template <bool STREAM>
__device__ __forceinline__ void load_to_lds_16(const void* base_uniform, uint32_t lane_offset,
                                               uint32_t lds_addr) {
  if constexpr (STREAM)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                 :
                 : "v"(lane_offset), "s"(base_uniform), "s"(lds_addr)
                 : "memory", "m0");
  else
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_offset), "s"(base_uniform), "s"(lds_addr)
                 : "memory", "m0");
}

// STREAM: the pair has a single row tile, so nobody else reads its K/V in this launch.
template <int D, int LGP, bool STREAM>
__device__ __forceinline__ void wide_tile_body(const KernelArgs& a, const optimus_work_item_t& it,
                                               float* smem) {
  constexpr int KS = D / 16, DB = D / 32, P = 1 << LGP;
  constexpr int PIECES = D * 4;        // 16-byte pieces of a K (= of a V) tile
  constexpr int LPT = PIECES / 256;    // load instructions per wave per tensor per tile
  constexpr int S = kWideStages, STAGE = 2 * PIECES;
  u32x4* sm = reinterpret_cast<u32x4*>(smem);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r32 = lane & 31, h = lane >> 5;
  const int G = a.group;

  const int rl = wave * 32 + r32;
  const bool valid = rl < it.row_count;
  const int row = it.row_begin + (valid ? rl : 0);
  const int jq = row / G, uq = row - jq * G;
  const int64_t row_off = ((int64_t)(it.q_token0 + jq) * a.num_q_heads + it.kv_head * G + uq) * D;
  bf16x8 qreg[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    u32x4 x = *reinterpret_cast<const u32x4*>(a.q + row_off + s * 16 + h * 8);
    if (!valid) x = u32x4{0u, 0u, 0u, 0u};
    qreg[s] = __builtin_bit_cast(bf16x8, x);
  }
  // cached length and block offset only matter for the block-causal mask: keep their loads
  // (which depend on the item's own load) off the start-up path of the plain mode
  int L = 0, d_in = 0;
  if (a.mask_mode != 0) {
    L = a.prefix_len[it.req];
    d_in = L - a.block_start[it.req];
  }
  const int vis_end = a.mask_mode == 0 ? INT32_MAX : block_causal_end(a, it, L, d_in, jq);
  const int vis_min = a.mask_mode == 0 ? INT32_MAX : block_causal_min(a, L, d_in);
  const int mask_from = min(it.kv_end, vis_min);
  const int lim = min(it.kv_end, vis_end);
  const bool wave_has_rows = wave * 32 < it.row_count;  // uniform per wave

  float m = -INFINITY, m_use = 0.f, lsum = 0.f;
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;

  const int32_t* bt = a.block_table + (int64_t)it.req * a.max_pages_per_req;
  const int last_page = (it.kv_end - 1) >> LGP;
  const char* kbase = reinterpret_cast<const char*>(a.k_pool + (int64_t)it.kv_head * a.k_stride_head);
  const char* vbase = reinterpret_cast<const char*>(a.v_pool + (int64_t)it.kv_head * a.v_stride_head);
  const uint32_t kspb32 = (uint32_t)(a.k_stride_page * 2), vspb32 = (uint32_t)(a.v_stride_page * 2);
  const float sc = a.scale_log2;
  const int tile_lo = it.kv_begin / kTileTokens;
  const int n = (it.kv_end + kTileTokens - 1) / kTileTokens - tile_lo;

  // Pages that hold a whole tile (32 keys or more): which global piece this lane fetches for LDS
  // piece e = (4*i + wave)*64 + lane of the layouts above.
  // 16-key pages: a tile is two pages, and each page's K block ([d group][key][8]) and V block
  // ([d][16 keys]) goes to LDS as it lies in memory, page after page, so that every load
  // instruction reads 1 KB of one page (uniform base in scalar registers):
  //   K piece a*PIECES/2 + g8*16 + key%16,  V piece a*PIECES/2 + 2*d + (half ^ ((d>>3)&1))
  // (a = key/16).  The 16 lanes an LDS cycle serves (16 consecutive rows of S^T or of V^T)
  // read 16 different 16-byte bank groups in both products.
  uint32_t ksrc[LPT], vsrc[LPT];
  if constexpr (LGP != 4) {
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int e = (4 * i + wave) * 64 + lane;
      const int g8 = e >> 5, pos = e & 31;
      const int key = (pos & 19) | ((pos & 4) << 1) | ((pos & 8) >> 1);
      const int d = e >> 2, o = (e & 3) ^ ((d >> 2) & 3);
      ksrc[i] = (uint32_t)(g8 * P + key) * 16u;
      vsrc[i] = (uint32_t)(d * P + 8 * o) * 2u;
    }
  }
  const uint32_t lane16 = (uint32_t)lane * 16u;
  // V of a 16-key page: the two 16-byte halves of the rows d with bit 3 set are fetched
  // swapped, i.e. LDS piece 2*d + (half ^ ((d >> 3) & 1)) holds (d, half).  Sixteen
  // consecutive rows of one half, which is what 16 consecutive lanes read as an operand, then
  // lie in sixteen different 16-byte bank groups (unswizzled they would share eight).
  const uint32_t lane16_v = (uint32_t)(lane ^ ((lane >> 4) & 1)) * 16u;
  constexpr int IPP = D / 32;   // load instructions (1 KB each) per 16-key page and tensor
  // this lane's K operand piece within a stage (score product st adds 32*st resp. 64*st) and
  // its V operand piece for d = r32, key half 0 (see SOFTMAX_PV)
  const int r32key = (r32 & 19) | ((r32 & 4) << 1) | ((r32 & 8) >> 1);   // key of S^T row r32
  const int kpiece = LGP == 4 ? (r32 >> 4) * (PIECES / 2) + h * 16 + (r32key & 15) : lane;
  // Page ids live in a register, lane i holding the id of page page_base + i, and reach the
  // scalar unit through v_readlane: no memory access per tile (a load inside the loop would
  // make every wait for it drain the tile loads in flight).  Refilled every 64 pages.
  int page_base = 0, page_reg = 0;
  auto REFILL = [&](int first_page) {
    page_base = first_page;
    page_reg = bt[min(first_page + lane, last_page)];
    // consume the value here, so that the wait for this load sits inside the (rare) refill
    // path instead of at the join, where it would be taken on every tile
    asm volatile("" : "+v"(page_reg));
  };
  REFILL((tile_lo * kTileTokens) >> LGP);
  // item tile t -> ring stage t % S (K pieces first, then V), straight from global memory
  auto ISSUE = [&](int t) {
    const int tile = tile_lo + t;
    const int pi0 = (tile * kTileTokens) >> LGP;
    const int pi1 = LGP == 4 ? min(pi0 + 1, last_page) : pi0;   // clamped: its keys are masked
    if (pi1 - page_base >= 64) REFILL(pi0);
    const int32_t p0 = __builtin_amdgcn_readlane(page_reg, pi0 - page_base);
    const int32_t p1 = LGP == 4 ? __builtin_amdgcn_readlane(page_reg, pi1 - page_base) : p0;
    // low 32 bits of a generic pointer into LDS = the LDS byte address
    const uint32_t dst = (uint32_t)(uintptr_t)(sm + (t & (S - 1)) * STAGE + wave * 64);
    const uint32_t slot0 = LGP == 4 ? 0u : (uint32_t)((tile * kTileTokens) & (P - 1));
    // page ids are non-negative and the page stride fits 32 bits (checked by the launcher):
    // one 32 x 32 -> 64 bit multiply per base
    const char* k0 = kbase + (uint64_t)(uint32_t)p0 * kspb32 + slot0 * 16u;
    const char* k1 = kbase + (uint64_t)(uint32_t)p1 * kspb32;
    const char* v0 = vbase + (uint64_t)(uint32_t)p0 * vspb32 + slot0 * 2u;
    const char* v1 = vbase + (uint64_t)(uint32_t)p1 * vspb32;
    if constexpr (LGP == 4) {   // two pages per tile, one page per instruction
#pragma unroll
      for (int i = 0; i < LPT; ++i) {
        const int j = 4 * i + wave;   // uniform
        load_to_lds_16<STREAM>((j / IPP ? k1 : k0) + (j % IPP) * 1024, lane16, dst + 16u * (256 * i));
      }
#pragma unroll
      for (int i = 0; i < LPT; ++i) {
        const int j = 4 * i + wave;
        load_to_lds_16<STREAM>((j / IPP ? v1 : v0) + (j % IPP) * 1024, lane16_v, dst + 16u * (PIECES + 256 * i));
      }
    } else {
#pragma unroll
      for (int i = 0; i < LPT; ++i) load_to_lds_16<STREAM>(k0, ksrc[i], dst + 16u * (256 * i));
#pragma unroll
      for (int i = 0; i < LPT; ++i) load_to_lds_16<STREAM>(v0, vsrc[i], dst + 16u * (PIECES + 256 * i));
    }
  };
  // S^T of item tile t: register v of a lane is key 32*tile + 16*(v/8) + 8h + v%8, row r32
  auto QK = [&](int t, f32x16& s) {
    const u32x4* kb = sm + (t & (S - 1)) * STAGE + kpiece;
    constexpr int kStep = LGP == 4 ? 32 : 64;   // pieces between the d groups 2*st+h of successive st
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
    for (int st = 0; st < KS; ++st)
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kb[kStep * st]), qreg[st], s, 0, 0, 0);
  };
  // row maximum of the scores of tile t (scaled); returns the candidate for the running
  // maximum.  The reference value m_use of the exponentials follows the maximum lazily (see
  // compute_tile): MOVE below changes it only for rows whose maximum grew by more than
  // kMaxSlack, and only then is anything rescaled.
  auto STATS = [&](int t, f32x16& s, bool masked) -> float {
    if (masked) {
      const int key0 = (tile_lo + t) * kTileTokens + 8 * h;
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] = key0 + 16 * (v / 8) + (v % 8) < lim ? s[v] : -INFINITY;
    }
    float mx = s[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[v]);
    {
      float x, y;
      swap32(mx, x, y);
      mx = fmaxf(x, y);
    }
    return fmaxf(m, mx * sc);
  };
  auto SOFTMAX_PV = [&](int t, const f32x16& s, float m_use, bool masked) {
    bf16x8 pt[2];
#pragma unroll
    for (int v = 0; v < 16; ++v) pt[v / 8][v % 8] = (__bf16)fast_exp2(fmaf(s[v], sc, -m_use));
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int v = 0; v < 16; v += 2) {
      const bf16x2 pr = {pt[v / 8][v % 8], pt[v / 8][v % 8 + 1]};
      lsum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, lsum, false);
    }
    const u32x4* vb = sm + (t & (S - 1)) * STAGE + PIECES;
    const int key0 = (tile_lo + t) * kTileTokens + 8 * h;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int aa = 0; aa < 2; ++aa) {
        const int d = 32 * db + r32, o = 2 * aa + h;
        u32x4 vv = LGP == 4 ? vb[aa * (PIECES / 2) + 2 * d + (h ^ ((d >> 3) & 1))] : vb[4 * d + (o ^ ((d >> 2) & 3))];
        if (masked) {   // keys at or beyond kv_end may hold anything: zero them
          const int cnt = it.kv_end - (key0 + 16 * aa);
          vv.x &= keep_mask(cnt); vv.y &= keep_mask(cnt - 2);
          vv.z &= keep_mask(cnt - 4); vv.w &= keep_mask(cnt - 6);
        }
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), pt[aa], acc[db], 0, 0, 0);
      }
    }
  };
  // take over the candidate maximum where it moved far enough; all accumulated state is then
  // brought to the new reference (wave-uniform branch, taken on few tiles)
  auto MOVE = [&](float m_cand) {
    const bool moved = m_cand - m > kMaxSlack;   // m = -inf: first finite maximum moves it
    if (__builtin_amdgcn_ballot_w64(moved) != 0) {
      const float m_new = moved ? m_cand : m;
      const float mu_new = m_new == -INFINITY ? 0.f : m_new;   // row with no visible key so far
      const float alpha = fast_exp2(m - mu_new);
      m = m_new;
      m_use = mu_new;
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] *= alpha;
      lsum *= alpha;
    }
  };
  auto tile_masked = [&](int t) { return (tile_lo + t + 1) * kTileTokens > mask_from; };

  // ---- prologue: three tiles in flight, scores of tile 0
#pragma unroll
  for (int t0 = 0; t0 < S - 1; ++t0)
    if (t0 < n) ISSUE(t0);
  // tile 0 and the K half of tile 1 must have landed (see STEP below)
  if (n >= 3) OPT_WAIT_VMCNT(3 * LPT);
  else if (n == 2) OPT_WAIT_VMCNT(LPT);
  else OPT_WAIT_VMCNT(0);
  OPT_BARRIER_NO_FENCE();
  f32x16 sa, sb;
  float m_cand = -INFINITY;
  if (wave_has_rows) {
    QK(0, sa);
    m_cand = STATS(0, sa, tile_masked(0));
    MOVE(m_cand);
  }

  // One pipelined step: loads of tile t+3, scores of tile t+1, softmax and PV of tile t.
  // At its end tile t+1 (V) and tile t+2 (K) must have landed: all but the 2*LPT loads of
  // tile t+3 and the LPT V loads of tile t+2 (K is issued before V).
  auto STEP = [&](int t, f32x16& cur, f32x16& nxt) {
    ISSUE(t + 3);
    if (wave_has_rows) {
      QK(t + 1, nxt);
      SOFTMAX_PV(t, cur, m_use, false);
      m_cand = STATS(t + 1, nxt, false);
    }
    OPT_WAIT_VMCNT(3 * LPT);
    OPT_BARRIER_NO_FENCE();
    if (wave_has_rows) MOVE(m_cand);
  };
  int t = 0;
  const int n_plain = min(n, (mask_from - tile_lo * kTileTokens) / kTileTokens);  // leading unmasked tiles
  for (; t + 4 < n && t + 2 < n_plain; t += 2) {
    STEP(t, sa, sb);
    STEP(t + 1, sb, sa);
  }
  // ---- remaining tiles: same step with every condition checked.  Once nothing is issued any
  // more, what may still be in flight shrinks: with tile t+2 the last one only its V loads,
  // after that nothing.
  for (; t < n; ++t) {
    const bool has_next = t + 1 < n, issue = t + 3 < n;
    if (issue) ISSUE(t + 3);
    if (wave_has_rows) {
      if (has_next) QK(t + 1, sb);
      SOFTMAX_PV(t, sa, m_use, tile_masked(t));
      if (has_next) m_cand = STATS(t + 1, sb, tile_masked(t + 1));
    }
    if (issue) OPT_WAIT_VMCNT(3 * LPT);
    else if (t + 3 == n) OPT_WAIT_VMCNT(LPT);
    else OPT_WAIT_VMCNT(0);
    OPT_BARRIER_NO_FENCE();
    if (wave_has_rows && has_next) {
      MOVE(m_cand);
      sa = sb;
    }
  }

  if (!valid) return;
  {
    float x, y;
    swap32(lsum, x, y);
    lsum = x + y;
  }
  if (it.part_row >= 0) {
    float* po = a.ws_o + (int64_t)(it.part_row + rl) * D + 4 * h;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<f32x4*>(po + 32 * db + 8 * g) =
            f32x4{acc[db][4 * g], acc[db][4 * g + 1], acc[db][4 * g + 2], acc[db][4 * g + 3]};
    if (h == 0) {
      float* pml = a.ws_ml + (int64_t)(it.part_row + rl) * 2;
      pml[0] = m;
      pml[1] = lsum;
    }
  } else {
    const float inv = 1.f / lsum;
    if (a.out_fp32) {
      float* po = reinterpret_cast<float*>(a.out) + row_off + 4 * h;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<f32x4*>(po + 32 * db + 8 * g) =
              f32x4{acc[db][4 * g] * inv, acc[db][4 * g + 1] * inv, acc[db][4 * g + 2] * inv,
                    acc[db][4 * g + 3] * inv};
    } else {
      __bf16* po = reinterpret_cast<__bf16*>(a.out) + row_off + 4 * h;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 b;
#pragma unroll
          for (int e = 0; e < 4; ++e) b[e] = (__bf16)(acc[db][4 * g + e] * inv);
          *reinterpret_cast<bf16x4*>(po + 32 * db + 8 * g) = b;
        }
    }
  }
}

// One launch serves every kind of work item: the block looks at its item and runs the
// matching body, so that a ragged batch (chunk sizes 1..32 side by side) is one grid in
// costliest-first order instead of one small grid per kind.  All bodies fit two waves per SIMD.
//
template <int D, int LGP>
__global__ __launch_bounds__(W * 64, 2) void attn_kernel(KernelArgs a) {
  constexpr int kFloats0 = split_wave_smem_floats<D, 1>() > lds_tile_smem_floats<D>()
                               ? split_wave_smem_floats<D, 1>() : lds_tile_smem_floats<D>();
  constexpr int kFloats = kFloats0 > wide_smem_floats<D>() ? kFloats0 : wide_smem_floats<D>();
  __shared__ __attribute__((aligned(16))) float smem[kFloats];
  const optimus_work_item_t it = a.items[blockIdx.x];
  // all row tiles of a (request, kv head) pair with more than kWideMinRows rows take the wide
  // body, also a narrow last one, so that the siblings run the same schedule side by side.
  // A later row tile (row_begin > 0) belongs to a pair of more than 128 rows, and the first
  // one shows min(128, rows): the item alone tells, no further load is needed.
  static_assert(kWideMinRows < kMaxRowsPerItem, "a first row tile must be able to show it");
  if (it.row_count > kWideMinRows || it.row_begin > 0) {
    // a first row tile of fewer than 128 rows is the pair's only one: its K/V are read once
    if (it.row_begin == 0 && it.row_count < kMaxRowsPerItem) wide_tile_body<D, LGP, true>(a, it, smem);
    else wide_tile_body<D, LGP, false>(a, it, smem);
  }
  else if (it.row_count <= 16) split_wave_body<D, LGP, 1>(a, it, smem);
  else lds_tile_body<D, LGP, 1>(a, it, smem);
}

// Merge of split-KV partials: for each row, M = max_s m_s,
//   o = sum_s 2^(m_s-M) o_s / sum_s 2^(m_s-M) l_s.
// Block (256 threads) = (merge item, group of 16 rows); thread = (row, D/16 columns).
//
// One pass: the splits are taken KB at a time with every load of a batch (m, l and the
// partial rows) issued before the first use, and merged online (running maximum M, the sums
// rescaled when it grows), so a row with up to KB splits costs one memory round trip.
// Indices past the last split are clamped to it and get weight zero; KB is chosen close to
// the number of splits so that few loads are such repeats.
template <int D, int KB>
__device__ __forceinline__ void merge_splits(const KernelArgs& a, const MergeItem& mi, int rl, int ocol,
                                             float (&o)[D / 16], float& lt) {
  constexpr int CH = D / 16;
  const int ns = mi.n_splits;
  const int64_t pr0 = mi.first_part_row + rl;
  float M = -INFINITY;
  for (int s0 = 0; s0 < ns; s0 += KB) {
    float mv[KB], lv[KB];
    f32x4 ov[KB][CH / 4];
#pragma unroll
    for (int k = 0; k < KB; ++k) {
      const int64_t pr = pr0 + (int64_t)min(s0 + k, ns - 1) * mi.row_count;
      mv[k] = a.ws_ml[pr * 2];
      lv[k] = a.ws_ml[pr * 2 + 1];
#pragma unroll
      for (int c = 0; c < CH / 4; ++c) ov[k][c] = *reinterpret_cast<const f32x4*>(a.ws_o + pr * D + ocol + 4 * c);
    }
    float Mb = M;
#pragma unroll
    for (int k = 0; k < KB; ++k) Mb = fmaxf(Mb, mv[k]);
    const float Mu = Mb == -INFINITY ? 0.f : Mb;        // no visible key in any split so far
    const float keep = fast_exp2(M - Mu);                // M = -inf: 0, and the sums are 0 anyway
    lt *= keep;
#pragma unroll
    for (int c = 0; c < CH; ++c) o[c] *= keep;
    M = Mb;
#pragma unroll
    for (int k = 0; k < KB; ++k) {
      const float w = s0 + k < ns ? fast_exp2(mv[k] - Mu) : 0.f;
      lt = fmaf(w, lv[k], lt);
#pragma unroll
      for (int c = 0; c < CH / 4; ++c) {
        o[4 * c] = fmaf(w, ov[k][c][0], o[4 * c]); o[4 * c + 1] = fmaf(w, ov[k][c][1], o[4 * c + 1]);
        o[4 * c + 2] = fmaf(w, ov[k][c][2], o[4 * c + 2]); o[4 * c + 3] = fmaf(w, ov[k][c][3], o[4 * c + 3]);
      }
    }
  }
}

template <int D>
__global__ __launch_bounds__(256) void merge_kernel(KernelArgs a) {
  const MergeItem mi = a.merges[blockIdx.x];
  constexpr int CH = D / 16;
  const int tid = threadIdx.x;
  const int rl = blockIdx.y * 16 + (tid >> 4);
  const int ocol = (tid & 15) * CH;
  if (rl >= mi.row_count) return;
  float lt = 0.f;
  float o[CH];
#pragma unroll
  for (int c = 0; c < CH; ++c) o[c] = 0.f;
  if (mi.n_splits <= 2) merge_splits<D, 2>(a, mi, rl, ocol, o, lt);        // uniform per block
  else if (mi.n_splits <= 4) merge_splits<D, 4>(a, mi, rl, ocol, o, lt);
  else if (mi.n_splits <= 8) merge_splits<D, 8>(a, mi, rl, ocol, o, lt);
  else merge_splits<D, 16>(a, mi, rl, ocol, o, lt);
  const float inv = 1.f / lt;
  const int G = a.group;
  const int row = mi.row_begin + rl;
  const int j = row / G, u = row - j * G;
  const int64_t off = ((int64_t)(mi.q_token0 + j) * a.num_q_heads + mi.kv_head * G + u) * D + ocol;
  if (a.out_fp32) {
    float* po = reinterpret_cast<float*>(a.out) + off;
#pragma unroll
    for (int c = 0; c < CH; c += 4)
      *reinterpret_cast<f32x4*>(po + c) = f32x4{o[c] * inv, o[c + 1] * inv, o[c + 2] * inv, o[c + 3] * inv};
  } else {
    __bf16* po = reinterpret_cast<__bf16*>(a.out) + off;
#pragma unroll
    for (int c = 0; c < CH; c += 4) {
      bf16x4 b;
#pragma unroll
      for (int e = 0; e < 4; ++e) b[e] = (__bf16)(o[c + e] * inv);
      *reinterpret_cast<bf16x4*>(po + c) = b;
    }
  }
}

// KV append: chunk token j of request i -> logical slot L_i + j of the pool.  The planner cuts
// every chunk into runs of up to 8 tokens whose slots lie in one aligned group of 8 slots (so
// in one page).  Block = (run, slice of 256 elements of the token row).  K: 16-byte groups per
// token.  V is slot-contiguous (stride P between d), so a run is written per (head, d) with the
// widest aligned stores that fit (16, 8, 4 or 2 bytes): a 2-byte store costs a whole 32-byte
// memory write, which made the token-by-token version write 9x its payload.
struct AppendRun { int32_t req, token0, slot0, count; };

struct PoolGeometry {
  int32_t num_kv_heads, page_size, lgp, max_pages_per_req, num_pages;
  int64_t k_stride_page, k_stride_head, v_stride_page, v_stride_head;
};

// Writes the `r.count` (1..8) tokens src[r.token0 ..] to the logical slots r.slot0.. of request
// r.req; all of them lie in one aligned group of 8 slots.  The workgroup takes the 256 (head, d)
// elements of a token row that start at element 256 * blockIdx.y: one V element column and at most
// one 16-byte K piece per thread, so that a run is spread over Hkv * D / 256 workgroups (a
// batch of one request has only c / 8 runs; one workgroup per run took 12 us there).  A
// block-table entry outside the pool writes nothing.
template <int D>
__device__ __forceinline__ void write_run(uint16_t* __restrict__ k_pool, uint16_t* __restrict__ v_pool,
                                          const uint16_t* __restrict__ k_src, const uint16_t* __restrict__ v_src,
                                          const int32_t* __restrict__ block_table, const AppendRun r,
                                          const PoolGeometry& g) {
  const int64_t page = block_table[(int64_t)r.req * g.max_pages_per_req + (r.slot0 >> g.lgp)];
  if ((uint64_t)page >= (uint64_t)g.num_pages) return;   // uniform per block
  const int page_size = g.page_size;
  const int slot = r.slot0 & (page_size - 1);
  const int row_elems = g.num_kv_heads * D;              // elements per token of the source
  const int64_t row = row_elems;
  const uint16_t* ksrc = k_src + (int64_t)r.token0 * row;
  const uint16_t* vsrc = v_src + (int64_t)r.token0 * row;
  uint16_t* kp = k_pool + page * g.k_stride_page;
  uint16_t* vp = v_pool + page * g.v_stride_page;
  const int e0 = (int)blockIdx.y * 256;                  // first (head, d) element of this workgroup
  {
    // K: token j, 16-byte piece q of the 32 pieces that cover elements e0 .. e0 + 255
    const int j = threadIdx.x >> 5, q = threadIdx.x & 31;
    const int el = e0 + q * 8;
    if (j < r.count && el < row_elems) {
      const int h = el / D, dg = (el % D) / 8;
      const u32x4 x = *reinterpret_cast<const u32x4*>(ksrc + j * row + el);
      *reinterpret_cast<u32x4*>(kp + (int64_t)h * g.k_stride_head + ((int64_t)dg * page_size + slot + j) * 8) = x;
    }
  }
  const int e = e0 + (int)threadIdx.x;
  if (e < row_elems) {
    const int h = e / D, d = e % D;
    // w[p]: value for position p of the aligned group of 8 slots (register indices are
    // compile-time; first and count are the same for the whole block: no divergence)
    const int first = slot & 7;
    uint16_t* dst = vp + (int64_t)h * g.v_stride_head + (int64_t)d * page_size + (slot - first);
    uint32_t w[8];
    bool on[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int j = p - first;
      on[p] = j >= 0 && j < r.count;
      w[p] = on[p] ? vsrc[j * row + e] : 0u;
    }
    if (r.count == 8) {
      *reinterpret_cast<u32x4*>(dst) =
          u32x4{w[0] | (w[1] << 16), w[2] | (w[3] << 16), w[4] | (w[5] << 16), w[6] | (w[7] << 16)};
    } else {
#pragma unroll
      for (int q = 0; q < 8; q += 4) {
        if (on[q] && on[q + 1] && on[q + 2] && on[q + 3]) {
          *reinterpret_cast<u32x2*>(dst + q) = u32x2{w[q] | (w[q + 1] << 16), w[q + 2] | (w[q + 3] << 16)};
        } else {
#pragma unroll
          for (int p = q; p < q + 4; p += 2) {
            if (on[p] && on[p + 1]) *reinterpret_cast<uint32_t*>(dst + p) = w[p] | (w[p + 1] << 16);
            else if (on[p]) dst[p] = (uint16_t)w[p];
            else if (on[p + 1]) dst[p + 1] = (uint16_t)w[p + 1];
          }
        }
      }
    }
  }
}

template <int D>
__global__ __launch_bounds__(256) void kv_append_kernel(
    uint16_t* __restrict__ k_pool, uint16_t* __restrict__ v_pool, const uint16_t* __restrict__ k_new,
    const uint16_t* __restrict__ v_new, const int32_t* __restrict__ block_table,
    const AppendRun* __restrict__ runs, PoolGeometry g, u32x4* __restrict__ upload_dst,
    const u32x4* __restrict__ upload_src, size_t upload_n, int upload_blocks) {
  // The first upload_blocks workgroups carry a pending work-list upload (pinned host memory ->
  // device) so that it does not cost a launch of its own; `runs` then points into the pinned
  // copy, which is complete before the launch, not into the device copy being written.
  if ((int)blockIdx.x < upload_blocks) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.y == 0 && i < upload_n) upload_dst[i] = upload_src[i];
    return;
  }
  write_run<D>(k_pool, v_pool, k_new, v_new, block_table, runs[blockIdx.x - upload_blocks], g);
}

// The same with the runs in the kernel's argument block: a short list (a batch of a few dozen
// requests) then reaches the workgroups with the launch itself, where reading it from the
// pinned host copy costs every workgroup a trip over the host link before its first load.
constexpr int kInlineRuns = 192;   // 3 KB of the 4 KB an argument block may have
struct InlineRuns { AppendRun r[kInlineRuns]; };
template <int D>
__global__ __launch_bounds__(256) void kv_append_inline_kernel(
    uint16_t* __restrict__ k_pool, uint16_t* __restrict__ v_pool, const uint16_t* __restrict__ k_new,
    const uint16_t* __restrict__ v_new, const int32_t* __restrict__ block_table, PoolGeometry g,
    u32x4* __restrict__ upload_dst, const u32x4* __restrict__ upload_src, size_t upload_n,
    int upload_blocks, InlineRuns runs) {
  if ((int)blockIdx.x < upload_blocks) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.y == 0 && i < upload_n) upload_dst[i] = upload_src[i];
    return;
  }
  write_run<D>(k_pool, v_pool, k_new, v_new, block_table, runs.r[blockIdx.x - upload_blocks], g);
}

// Plan-independent writer: tokens 0..n-1 of (k_src, v_src) go to the logical slots
// first_slot.. of request `req`.  Block b takes the b-th aligned group of 8 slots the range touches.
template <int D>
__global__ __launch_bounds__(256) void kv_write_kernel(
    uint16_t* __restrict__ k_pool, uint16_t* __restrict__ v_pool, const uint16_t* __restrict__ k_src,
    const uint16_t* __restrict__ v_src, const int32_t* __restrict__ block_table, int req,
    int first_slot, int n, PoolGeometry g) {
  const int group = (first_slot >> 3) + (int)blockIdx.x;
  const int lo = max(first_slot, group * 8), hi = min(first_slot + n, group * 8 + 8);
  if (lo >= hi) return;
  write_run<D>(k_pool, v_pool, k_src, v_src, block_table, AppendRun{req, lo - first_slot, lo, hi - lo}, g);
}

// ------------------------------------------------------------------ static scratch
// Scratch for callers that cannot allocate: the split-KV partials of optimus_attn_forward_static
// live here instead of in a caller-provided workspace.  Every GPU the library runs on holds its
// own copy of this array, at its own address, until the process ends.  In host code the array's
// name is only a handle for the symbol lookup: the device address comes from
// hipGetSymbolAddress, once per device, and that pointer is what kernels are given.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];   // zero-initialised: not looked up yet

int static_scratch_for_current_device(int device, void** ptr_out) {
  if (device < 0 || device >= kMaxDevices || !ptr_out) return OPTIMUS_ERR_INVALID_ARGUMENT;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      set_hip_error((int)(e != hipSuccess ? e : hipErrorInvalidSymbol), "hipGetSymbolAddress(scratch)");
      return OPTIMUS_ERR_HIP;
    }
    g_scratch_ptr[device] = ptr;
  }
  *ptr_out = g_scratch_ptr[device];
  return OPTIMUS_OK;
}

// ------------------------------------------------------------------ launchers

template <int D>
static int launch_attention_d(const optimus_attn_params_t& p, const KernelArgs& a, int32_t n_items,
                              hipStream_t stream) {
  const dim3 grid(n_items), block(W * 64);
  switch (p.page_size) {
    case 16: hipLaunchKernelGGL((attn_kernel<D, 4>), grid, block, 0, stream, a); break;
    case 32: hipLaunchKernelGGL((attn_kernel<D, 5>), grid, block, 0, stream, a); break;
    case 64: hipLaunchKernelGGL((attn_kernel<D, 6>), grid, block, 0, stream, a); break;
    case 128: hipLaunchKernelGGL((attn_kernel<D, 7>), grid, block, 0, stream, a); break;
    default: return OPTIMUS_ERR_UNSUPPORTED_SHAPE;
  }
  return OPTIMUS_OK;
}

int launch_attention(const optimus_attn_params_t& p, const KernelArgs& a, int32_t n_items,
                     void* stream) {
  if (n_items <= 0) return OPTIMUS_OK;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  int rc;
  if (p.head_dim == 128) rc = launch_attention_d<128>(p, a, n_items, s);
  else if (p.head_dim == 64) rc = launch_attention_d<64>(p, a, n_items, s);
  else return OPTIMUS_ERR_UNSUPPORTED_SHAPE;
  if (rc != OPTIMUS_OK) return rc;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error((int)e, "attention kernel launch"); return OPTIMUS_ERR_HIP; }
  return OPTIMUS_OK;
}

int launch_merge(const optimus_attn_params_t& p, const KernelArgs& a, int32_t n_merges, void* stream) {
  if (n_merges <= 0) return OPTIMUS_OK;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const dim3 grid(n_merges, kMaxRowsPerItem / kRowsPerSubtile), block(256);
  if (p.head_dim == 128) hipLaunchKernelGGL((merge_kernel<128>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((merge_kernel<64>), grid, block, 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error((int)e, "merge kernel launch"); return OPTIMUS_ERR_HIP; }
  return OPTIMUS_OK;
}

static PoolGeometry pool_geometry(const optimus_attn_params_t& p) {
  PoolGeometry g{};
  g.num_kv_heads = p.num_kv_heads; g.page_size = p.page_size; g.lgp = 0;
  while ((1 << g.lgp) < p.page_size) ++g.lgp;
  g.max_pages_per_req = p.max_pages_per_req; g.num_pages = p.num_pages;
  g.k_stride_page = p.k_stride_page; g.k_stride_head = p.k_stride_head;
  g.v_stride_page = p.v_stride_page; g.v_stride_head = p.v_stride_head;
  return g;
}

int launch_kv_append(const optimus_attn_params_t& p, uint16_t* k_pool, uint16_t* v_pool,
                     const uint16_t* k_new, const uint16_t* v_new, const int32_t* block_table,
                     const int32_t* runs, const int32_t* runs_host, int32_t n_runs, int32_t* upload_dst,
                     const int32_t* upload_src, size_t upload_i32, void* stream) {
  if (n_runs <= 0) return upload_i32 ? launch_upload(upload_dst, upload_src, upload_i32, stream) : OPTIMUS_OK;
  if (upload_i32 % 4 != 0) return OPTIMUS_ERR_INVALID_ARGUMENT;
  const size_t up_n = upload_i32 / 4;
  const int up_blocks = (int)((up_n + 255) / 256);
  u32x4* ud = reinterpret_cast<u32x4*>(upload_dst);
  const u32x4* us = reinterpret_cast<const u32x4*>(upload_src);
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const dim3 grid(n_runs + up_blocks, (p.num_kv_heads * p.head_dim + 255) / 256), block(256);
  const AppendRun* r = reinterpret_cast<const AppendRun*>(runs);
  const PoolGeometry g = pool_geometry(p);
  if (runs_host && n_runs <= kInlineRuns) {
    InlineRuns in;
    std::memcpy(in.r, runs_host, (size_t)n_runs * sizeof(AppendRun));
    if (p.head_dim == 128)
      hipLaunchKernelGGL((kv_append_inline_kernel<128>), grid, block, 0, s, k_pool, v_pool, k_new, v_new,
                         block_table, g, ud, us, up_n, up_blocks, in);
    else
      hipLaunchKernelGGL((kv_append_inline_kernel<64>), grid, block, 0, s, k_pool, v_pool, k_new, v_new,
                         block_table, g, ud, us, up_n, up_blocks, in);
  } else if (p.head_dim == 128)
    hipLaunchKernelGGL((kv_append_kernel<128>), grid, block, 0, s, k_pool, v_pool, k_new, v_new,
                       block_table, r, g, ud, us, up_n, up_blocks);
  else
    hipLaunchKernelGGL((kv_append_kernel<64>), grid, block, 0, s, k_pool, v_pool, k_new, v_new,
                       block_table, r, g, ud, us, up_n, up_blocks);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error((int)e, "kv_append kernel launch"); return OPTIMUS_ERR_HIP; }
  return OPTIMUS_OK;
}

int launch_kv_write(const optimus_attn_params_t& p, uint16_t* k_pool, uint16_t* v_pool,
                    const uint16_t* k_src, const uint16_t* v_src, const int32_t* block_table,
                    int32_t req, int32_t first_slot, int32_t n, void* stream) {
  if (n <= 0) return OPTIMUS_OK;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const int groups = ((first_slot + n - 1) >> 3) - (first_slot >> 3) + 1;
  const dim3 grid(groups, (p.num_kv_heads * p.head_dim + 255) / 256), block(256);
  const PoolGeometry g = pool_geometry(p);
  if (p.head_dim == 128)
    hipLaunchKernelGGL((kv_write_kernel<128>), grid, block, 0, s, k_pool, v_pool, k_src, v_src,
                       block_table, req, first_slot, n, g);
  else
    hipLaunchKernelGGL((kv_write_kernel<64>), grid, block, 0, s, k_pool, v_pool, k_src, v_src,
                       block_table, req, first_slot, n, g);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error((int)e, "kv_write kernel launch"); return OPTIMUS_ERR_HIP; }
  return OPTIMUS_OK;
}

__global__ __launch_bounds__(256) void upload_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                     size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

int launch_upload(int32_t* dst_device, const int32_t* src_pinned_host, size_t n_i32, void* stream) {
  if (n_i32 == 0) return OPTIMUS_OK;
  if (n_i32 % 4 != 0) return OPTIMUS_ERR_INVALID_ARGUMENT;
  const size_t n = n_i32 / 4;
  hipLaunchKernelGGL(upload_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(stream), reinterpret_cast<u32x4*>(dst_device),
                     reinterpret_cast<const u32x4*>(src_pinned_host), n);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error((int)e, "upload kernel launch"); return OPTIMUS_ERR_HIP; }
  return OPTIMUS_OK;
}

}  // namespace optimus
