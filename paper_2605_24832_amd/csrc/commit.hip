// Commit step of block-diffusion decoding on gfx950 (Optimus Sec. 2.3 / 4.1:
// positions whose confidence exceeds a threshold are committed each iteration).
// Confidence = largest softmax probability of the position's logit row, token = first index
// attaining it; -inf and NaN logits are entries that cannot be chosen.
//
// HBM-bound scan of the logits with a co-critical exponential per entry (about five vector
// instructions per entry, one of them a quarter-rate v_exp_f32: at 152K entries per row the
// vector unit and the memory system are busy for about the same time).  One workgroup of 256
// threads owns one row, so no partial result leaves the workgroup (four rows are resident per
// compute unit; 128, 512 and 1024 threads per row measured 25 %, 6 % and 21 % slower).  A thread walks its 16-byte
// pieces eight at a time (eight loads in flight) and keeps
//   m     largest entry so far (bookkeeping for the token only),
//   base  first of its pieces that holds m,
//   r     reference of the exponentials in log2 units, s = sum of 2^(x log2 e - r).
// The reference is set from the thread's first piece and then followed lazily: it only moves
// (rare path, the eight pieces are summed again) when the maximum has grown more than 2^64
// beyond it, so the common path is unpack, max, fma, exp2, add and nothing else; the result
// 2^(M log2 e - R) / S does not depend on where the reference sits.  Entries that are -inf add
// exp2(-inf) = 0; when a sum comes out NaN (a NaN entry) the eight pieces are summed again
// with NaN entries skipped.  The threads are joined through the wave and LDS; the winning
// piece is read once more to find the first entry equal to the maximum.  A second, tiny kernel
// applies the per-request progress rule.  +inf entries are outside the definition (no access
// depends on a value, so they cannot cause one out of bounds).
#include <hip/hip_runtime.h>

#include <cmath>

#include "optimus_attn.h"
#include "plan_internal.h"

namespace optimus {

typedef unsigned int u32x4c __attribute__((ext_vector_type(4)));
constexpr int kRowThreads = 256;
constexpr int kPiece = 8;                       // bf16 per 16-byte load
constexpr int kInflight = 8;                    // 16-byte loads in flight per thread
constexpr int kRound = kInflight * kRowThreads; // pieces one workgroup takes per round
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRefSlack = 64.0f;              // the reference may trail the maximum by 2^64
constexpr uint32_t kNegInfPair = 0xff80ff80u;   // two bf16 -inf

struct RowState { float m, r, s; int32_t base; };   // LDS record of one wave's result

__device__ __forceinline__ bool is_nan_bits(float x) {   // the build assumes no NaN: compare bit patterns
  return (__float_as_uint(x) & 0x7fffffffu) > 0x7f800000u;
}

// Join with the state of lane (lane ^ off); plain scalars so that everything stays in registers.
// Equal maxima keep the smaller piece (pieces of different threads are disjoint index ranges).
__device__ __forceinline__ void join_xor(float& m, float& r, float& s, int32_t& base, int off) {
  const float bm = __shfl_xor(m, off, 64), br = __shfl_xor(r, off, 64), bs = __shfl_xor(s, off, 64);
  const int32_t bb = __shfl_xor(base, off, 64);
  const bool b_wins = bm > m || (bm == m && bb < base);
  const float R = fmaxf(r, br);
  // r = -inf on both sides: nothing summed yet (the difference would be NaN)
  s = R == -INFINITY ? 0.f : s * __builtin_amdgcn_exp2f(r - R) + bs * __builtin_amdgcn_exp2f(br - R);
  m = b_wins ? bm : m;
  base = b_wins ? bb : base;
  r = R;
}

__device__ __forceinline__ void unpack(const u32x4c raw, float (&x)[kPiece]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    x[2 * e] = __uint_as_float(raw[e] << 16);
    x[2 * e + 1] = __uint_as_float(raw[e] & 0xffff0000u);
  }
}

// Entries at or beyond the row's end read as -inf.
__device__ __forceinline__ void mask_row_end(float (&x)[kPiece], int base, int vocab) {
  if (base + kPiece > vocab) {
#pragma unroll
    for (int e = 0; e < kPiece; ++e)
      if (base + e >= vocab) x[e] = -INFINITY;
  }
}

// One round of a thread: pieces p0, p0 + kRowThreads, ... (kInflight of them).  CHECKED: the round may
// reach past the row (its last one); otherwise every piece lies inside the row.
template <bool CHECKED>
__device__ __forceinline__ void scan_round(const u32x4c* __restrict__ row, int p0, int n_pieces, int vocab,
                                           float& m, float& r, float& s, int32_t& best_base) {
  u32x4c raw[kInflight];
#pragma unroll
  for (int u = 0; u < kInflight; ++u) {
    const int pc = p0 + u * kRowThreads;
    if (CHECKED)
      raw[u] = pc < n_pieces ? __builtin_nontemporal_load(row + pc)   // read once
                             : u32x4c{kNegInfPair, kNegInfPair, kNegInfPair, kNegInfPair};
    else
      raw[u] = __builtin_nontemporal_load(row + pc);
  }
  if (r == -INFINITY) {
    // no reference yet (start of the row, or only masked entries so far): take it from this
    // thread's first piece of the round; v_max skips NaN operands
    float x[kPiece];
    unpack(raw[0], x);
    if (CHECKED) mask_row_end(x, p0 * kPiece, vocab);
    const float c0 = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    if (!is_nan_bits(c0)) r = c0 * kLog2e;    // still -inf if the piece is masked
  }
  const float s_before = s;
  float nr = r == -INFINITY ? 0.f : -r;       // exp2(-inf + 0) = 0 for masked entries
#pragma unroll
  for (int u = 0; u < kInflight; ++u) {
    const int base = (p0 + u * kRowThreads) * kPiece;
    if (CHECKED && __builtin_amdgcn_ballot_w64(base < vocab) == 0) continue;   // the whole wave is past the row
    float x[kPiece];
    unpack(raw[u], x);
    if (CHECKED) mask_row_end(x, base, vocab);
    // v_max returns the other operand when one is NaN: cm is the largest non-NaN entry
    const float cm = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    const float m_new = fmaxf(m, cm);         // m is never NaN, so neither is m_new
    best_base = m_new > m ? base : best_base; // strict: the earlier piece keeps a tie
    m = m_new;
#pragma unroll
    for (int e = 0; e < kPiece; ++e) s += __builtin_amdgcn_exp2f(fmaf(x[e], kLog2e, nr));
  }
  // Rare path: a NaN entry reached the sum, or the maximum has run away from the reference
  // (also: the first unmasked entries of a row whose first piece was masked).  Sum the round
  // again from its start with the reference at the maximum and NaN entries skipped.
  const bool redo = is_nan_bits(s) || (m != -INFINITY && (r == -INFINITY || fmaf(m, kLog2e, nr) > kRefSlack));
  if (__builtin_amdgcn_ballot_w64(redo) != 0) {
    const float r_new = m == -INFINITY ? r : fmaxf(r, m * kLog2e);
    s = r == -INFINITY ? 0.f : s_before * __builtin_amdgcn_exp2f(r - r_new);
    r = r_new;
    nr = r == -INFINITY ? 0.f : -r;
#pragma unroll
    for (int u = 0; u < kInflight; ++u) {
      const int base = (p0 + u * kRowThreads) * kPiece;
      float x[kPiece];
      unpack(raw[u], x);
      if (CHECKED) mask_row_end(x, base, vocab);
#pragma unroll
      for (int e = 0; e < kPiece; ++e)
        s += is_nan_bits(x[e]) ? 0.f : __builtin_amdgcn_exp2f(fmaf(x[e], kLog2e, nr));
    }
  }
}

// 4 waves per SIMD (at most 128 vector registers): four rows resident per compute unit
__global__ __launch_bounds__(kRowThreads, 4) void commit_row_kernel(
    const uint16_t* __restrict__ logits, int vocab, int64_t row_stride, float threshold,
    int32_t* __restrict__ token_out, float* __restrict__ conf_out, int32_t* __restrict__ commit_out) {
  const int t = blockIdx.x;
  // rows are padded to a multiple of 8 entries, so a piece that starts inside the row is
  // readable as a whole
  const u32x4c* row = reinterpret_cast<const u32x4c*>(logits + (int64_t)t * row_stride);
  const int n_pieces = (vocab + kPiece - 1) / kPiece;
  float pm = -INFINITY, pr = -INFINITY, ps = 0.f;
  int32_t pbase = 0x7fffffff;
  // all rounds but the last lie inside the row for every thread; the last one is checked
  const int full_rounds = (n_pieces - 1) / kRound;
  int p0 = threadIdx.x;
  for (int i = 0; i < full_rounds; ++i, p0 += kRound)
    scan_round<false>(row, p0, n_pieces, vocab, pm, pr, ps, pbase);
  scan_round<true>(row, p0, n_pieces, vocab, pm, pr, ps, pbase);

#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) join_xor(pm, pr, ps, pbase, off);
  __shared__ RowState sm[kRowThreads / 64];
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = RowState{pm, pr, ps, pbase};
  __syncthreads();
  if (threadIdx.x < 64) {
    const RowState w = sm[threadIdx.x & (kRowThreads / 64 - 1)];
    pm = w.m; pr = w.r; ps = w.s; pbase = w.base;
#pragma unroll
    for (int off = kRowThreads / 128; off >= 1; off >>= 1) join_xor(pm, pr, ps, pbase, off);
    if (threadIdx.x == 0) {
      const bool none = pm == -INFINITY;   // every entry masked
      int token = 0;
      if (!none) {
        // first entry of the winning piece equal to the maximum, compared as bit patterns
        // (+0 and -0 are equal); entries beyond the row are never equal to it: they are the
        // padding, and the maximum was taken over the row only, so stop at the row's end
        const u32x4c raw = row[pbase / kPiece];
        const uint32_t mb = __float_as_uint(pm);
        int ci = kPiece - 1;
#pragma unroll
        for (int e = kPiece - 2; e >= 0; --e) {
          const uint32_t xb = (e & 1) ? (raw[e / 2] & 0xffff0000u) : (raw[e / 2] << 16);
          ci = (xb == mb || ((xb | mb) & 0x7fffffffu) == 0u) ? e : ci;
        }
        token = min(pbase + ci, vocab - 1);
      }
      const float conf = none ? 0.f : __builtin_amdgcn_exp2f(fmaf(pm, kLog2e, -pr)) / ps;
      token_out[t] = token;
      conf_out[t] = conf;
      commit_out[t] = conf > threshold ? 1 : 0;
    }
  }
}

// Progress rule: a request with chunk tokens but none above the threshold commits its most
// confident one (first on ties).  One wave per request, 4 requests per block.
__global__ __launch_bounds__(256) void commit_progress_kernel(
    const float* __restrict__ conf, const int32_t* __restrict__ cu_q, int batch,
    int32_t* __restrict__ commit_out) {
  const int lane = threadIdx.x & 63;
  const int req = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (req >= batch) return;   // whole wave
  const int t_lo = cu_q[req], t_hi = cu_q[req + 1];
  if (t_hi <= t_lo) return;
  // candidates start at the request's first token, so the store below stays inside the request
  // whatever the confidences are
  float best_conf = -1.f;
  int best_t = t_lo, any = 0;
  for (int t = t_lo + lane; t < t_hi; t += 64) {
    any |= commit_out[t];
    const float c = conf[t];
    if (c > best_conf) { best_conf = c; best_t = t; }   // strict: first on ties
  }
  if (__builtin_amdgcn_ballot_w64(any != 0) != 0) return;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float oc = __shfl_xor(best_conf, off, 64);
    const int ot = __shfl_xor(best_t, off, 64);
    if (oc > best_conf || (oc == best_conf && ot < best_t)) { best_conf = oc; best_t = ot; }
  }
  // lanes without a token kept (-1, t_lo), so best_t is a token of this request
  if (lane == 0) commit_out[best_t] = 1;
}

static bool commit_params_ok(const optimus_commit_params_t* p) {
  return p && p->num_tokens >= 0 && p->num_tokens <= (1 << 24) && p->vocab >= 1 && p->row_stride % 8 == 0 &&
         p->row_stride >= ((int64_t)p->vocab + 7) / 8 * 8 && p->batch >= 0 &&
         (p->min_commit == 0 || p->min_commit == 1);
}

}  // namespace optimus

using namespace optimus;

extern "C" int optimus_commit_forward(const optimus_commit_params_t* params, int device,
                                      const void* logits, const int32_t* cu_q, int32_t* token_out,
                                      float* conf_out, int32_t* commit_out, void* hip_stream) {
  if (!commit_params_ok(params) || device < 0) return OPTIMUS_ERR_INVALID_ARGUMENT;
  const optimus_commit_params_t& p = *params;
  if (p.num_tokens == 0) return OPTIMUS_OK;
  if (!logits || !token_out || !conf_out || !commit_out) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (p.batch > 0 && !cu_q) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if ((uintptr_t)logits & 15) return OPTIMUS_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(device);   // the caller's current device is put back on return
  if (guard.status() != OPTIMUS_OK) return guard.status();
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  hipLaunchKernelGGL(commit_row_kernel, dim3(p.num_tokens), dim3(kRowThreads), 0, s,
                     (const uint16_t*)logits, p.vocab, p.row_stride, p.threshold, token_out, conf_out,
                     commit_out);
  if (p.batch > 0 && p.min_commit >= 1)
    hipLaunchKernelGGL(commit_progress_kernel, dim3((p.batch + 3) / 4), dim3(256), 0, s, conf_out, cu_q,
                       p.batch, commit_out);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error((int)e, "commit kernel launch"); return OPTIMUS_ERR_HIP; }
  return OPTIMUS_OK;
}
