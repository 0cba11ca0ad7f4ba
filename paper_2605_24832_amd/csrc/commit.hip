// Commit step of block-diffusion decoding on gfx950 (Optimus Sec. 2.3 / 4.1:
// positions whose confidence exceeds a threshold are committed each iteration).
// Confidence = largest softmax probability of the position's logit row, token = first index
// attaining it; -inf and NaN logits are entries that cannot be chosen.
//
// HBM-bound scan of the logits with a co-critical exponential per entry.  One workgroup of
// 1024 threads owns one row (no partial results leave the workgroup): every thread walks
// its 16-byte pieces with eight loads in flight and keeps an online (max, sum of exp, first
// argmax); the threads are joined through the wave and LDS and the row's token, confidence
// and commit flag are stored directly.  A second, tiny kernel applies the per-request progress rule.
//
// Arithmetic per entry: unpack, max (v_max3 over a piece), one fma, one exp2, one add.  The
// exponent is fma(x, log2 e, -r) with r = fl(m * log2 e) the reference in log2 units, which
// the joins carry along, so no rounding of m * log2 e enters the result: the confidence is
// 2^(fma(M, log2 e, -R)) / S for the row's maximum M and the final reference R.
// -inf entries add exp2(-inf) = 0; a piece whose sum comes out NaN (a NaN entry) is summed
// again with NaN entries read as -inf.  +inf entries are outside the definition (no access
// depends on a value, so they cannot cause one out of bounds).
#include <hip/hip_runtime.h>

#include <cmath>

#include "optimus_attn.h"
#include "plan_internal.h"

namespace optimus {

typedef unsigned int u32x4c __attribute__((ext_vector_type(4)));
constexpr int kRowThreads = 1024;
constexpr int kPiece = 8;                       // bf16 per 16-byte load
constexpr int kInflight = 8;                    // 16-byte loads in flight per thread
constexpr float kLog2e = 1.4426950408889634f;
constexpr uint32_t kNegInfPair = 0xff80ff80u;   // two bf16 -inf

struct RowState { float m, r, s; int32_t idx; };   // LDS record of one wave's result

__device__ __forceinline__ bool is_nan_bits(float x) {   // the build assumes no NaN: compare bit patterns
  return (__float_as_uint(x) & 0x7fffffffu) > 0x7f800000u;
}

// Join with the state of lane (lane ^ off); plain scalars so that everything stays in registers.
__device__ __forceinline__ void join_xor(float& m, float& r, float& s, int32_t& idx, int off) {
  const float bm = __shfl_xor(m, off, 64), br = __shfl_xor(r, off, 64), bs = __shfl_xor(s, off, 64);
  const int32_t bi = __shfl_xor(idx, off, 64);
  const bool b_wins = bm > m || (bm == m && bi < idx);
  const float R = fmaxf(r, br);
  // r = -inf on both sides: nothing summed yet (the difference would be NaN)
  s = R == -INFINITY ? 0.f : s * __builtin_amdgcn_exp2f(r - R) + bs * __builtin_amdgcn_exp2f(br - R);
  m = b_wins ? bm : m;
  idx = b_wins ? bi : idx;
  r = R;
}

// 8 waves per SIMD: two rows resident per compute unit (at most 64 vector registers)
__global__ __launch_bounds__(kRowThreads, 8) void commit_row_kernel(
    const uint16_t* __restrict__ logits, int vocab, int64_t row_stride, float threshold,
    int32_t* __restrict__ token_out, float* __restrict__ conf_out, int32_t* __restrict__ commit_out) {
  const int t = blockIdx.x;
  const uint16_t* row = logits + (int64_t)t * row_stride;
  const int n_pieces = (vocab + kPiece - 1) / kPiece;
  // m: largest entry so far (-inf: none), r = fl(m * log2 e), s = sum of 2^(x log2 e - r),
  // idx = first index attaining m
  float pm = -INFINITY, pr = -INFINITY, ps = 0.f;
  int32_t pidx = 0x7fffffff;
  for (int p0 = threadIdx.x; p0 < n_pieces; p0 += kInflight * kRowThreads) {
    // rows are padded to a multiple of 8 entries, so a piece that starts inside the row is
    // readable as a whole; pieces past the row read as -inf and change nothing
    u32x4c raw[kInflight];
#pragma unroll
    for (int u = 0; u < kInflight; ++u) {
      const int pc = p0 + u * kRowThreads;
      raw[u] = pc < n_pieces ? __builtin_nontemporal_load(reinterpret_cast<const u32x4c*>(row) + pc)   // read once
                             : u32x4c{kNegInfPair, kNegInfPair, kNegInfPair, kNegInfPair};
    }
#pragma unroll
    for (int u = 0; u < kInflight; ++u) {
      const int base = (p0 + u * kRowThreads) * kPiece;
      if (__builtin_amdgcn_ballot_w64(base < vocab) == 0) continue;   // the whole wave is past the row
      uint32_t xb[kPiece];
      float x[kPiece];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        xb[2 * e] = raw[u][e] << 16;
        xb[2 * e + 1] = raw[u][e] & 0xffff0000u;
      }
      if (base + kPiece > vocab) {   // the row's last piece (or one past the row)
#pragma unroll
        for (int e = 0; e < kPiece; ++e)
          if (base + e >= vocab) xb[e] = 0xff800000u;
      }
#pragma unroll
      for (int e = 0; e < kPiece; ++e) x[e] = __uint_as_float(xb[e]);
      // v_max returns the other operand when one is NaN, so cm is the largest non-NaN entry
      // (NaN only if all eight are)
      const float cm = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
      const bool raise = cm > pm && !is_nan_bits(cm);   // strict: the earlier piece keeps a tie
      if (__builtin_amdgcn_ballot_w64(raise) != 0) {   // rare after the first pieces of a row
        // first entry equal to cm, compared as bit patterns (+0 and -0 are equal)
        const uint32_t cmb = __float_as_uint(cm);
        int ci = kPiece - 1;
#pragma unroll
        for (int e = kPiece - 2; e >= 0; --e)
          ci = (xb[e] == cmb || ((xb[e] | cmb) & 0x7fffffffu) == 0u) ? e : ci;
        const float r_new = raise ? cm * kLog2e : pr;
        ps = pr == -INFINITY ? 0.f : ps * __builtin_amdgcn_exp2f(pr - r_new);
        pidx = raise ? base + ci : pidx;
        pm = raise ? cm : pm;
        pr = r_new;
      }
      const float ref = pr == -INFINITY ? 0.f : -pr;   // nothing finite yet: exp2(-inf + 0) = 0
      float add = 0.f;
#pragma unroll
      for (int e = 0; e < kPiece; ++e) add += __builtin_amdgcn_exp2f(fmaf(x[e], kLog2e, ref));
      if (__builtin_amdgcn_ballot_w64(is_nan_bits(add)) != 0) {   // some entry is NaN: it counts as -inf
        add = 0.f;
#pragma unroll
        for (int e = 0; e < kPiece; ++e)
          add += is_nan_bits(x[e]) ? 0.f : __builtin_amdgcn_exp2f(fmaf(x[e], kLog2e, ref));
      }
      ps += add;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) join_xor(pm, pr, ps, pidx, off);
  __shared__ RowState sm[kRowThreads / 64];
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = RowState{pm, pr, ps, pidx};
  __syncthreads();
  if (threadIdx.x < 64) {
    const RowState w = sm[threadIdx.x & (kRowThreads / 64 - 1)];
    pm = w.m; pr = w.r; ps = w.s; pidx = w.idx;
#pragma unroll
    for (int off = kRowThreads / 128; off >= 1; off >>= 1) join_xor(pm, pr, ps, pidx, off);
    if (threadIdx.x == 0) {
      const bool none = pm == -INFINITY;   // every entry masked
      const float conf = none ? 0.f : __builtin_amdgcn_exp2f(fmaf(pm, kLog2e, -pr)) / ps;
      token_out[t] = none ? 0 : pidx;
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
