// Commit step of block-diffusion decoding on gfx950 (Optimus Sec. 2.3 / 4.1:
// positions whose confidence exceeds a threshold are committed each iteration).
//
// HBM-bound scan of the logits: every row is cut into segments, one workgroup
// per (segment, row) keeps a running (max, sum of exp, first argmax) per thread
// over 16-byte pieces and reduces it through the wave and LDS; a second small
// kernel joins the segments of a row (confidence = 1 / sum of exp(x - max)),
// applies the threshold and the per-request progress rule.
#include <hip/hip_runtime.h>

#include <cmath>

#include "optimus_attn.h"
#include "plan_internal.h"

namespace optimus {

typedef unsigned int u32x4c __attribute__((ext_vector_type(4)));
constexpr int kScanThreads = 256;
constexpr int kPiece = 8;                       // bf16 per 16-byte load
constexpr int kStep = kScanThreads * kPiece;    // columns one block covers per load round
constexpr int kUnroll = 4;                      // load rounds in flight per thread
constexpr float kLog2e = 1.4426950408889634f;

struct Partial { float m, s; int32_t idx, pad; };   // max, sum of exp(x - m), first argmax

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ Partial join(const Partial& a, const Partial& b) {
  // an empty partial has m = -inf, s = 0
  if (b.m == -INFINITY) return a;
  if (a.m == -INFINITY) return b;
  Partial r;
  r.m = fmaxf(a.m, b.m);
  r.s = a.s * __builtin_amdgcn_exp2f((a.m - r.m) * kLog2e) + b.s * __builtin_amdgcn_exp2f((b.m - r.m) * kLog2e);
  r.idx = (a.m > b.m || (a.m == b.m && a.idx < b.idx)) ? a.idx : b.idx;
  r.pad = 0;
  return r;
}

__global__ __launch_bounds__(kScanThreads) void commit_scan_kernel(
    const uint16_t* __restrict__ logits, int vocab, int64_t row_stride, int seg_len, Partial* __restrict__ part) {
  const int seg = blockIdx.x, t = blockIdx.y, n_seg = gridDim.x;
  const uint16_t* row = logits + (int64_t)t * row_stride;
  const int lo = seg * seg_len, hi = min(vocab, lo + seg_len);
  Partial p{-INFINITY, 0.f, 0x7fffffff, 0};
  for (int base0 = lo + threadIdx.x * kPiece; base0 < hi; base0 += kUnroll * kStep) {
    // kUnroll independent 16-byte loads in flight per thread (rows are padded to a multiple
    // of 8 elements, so a piece that starts inside the row is readable as a whole)
    u32x4c raw[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int base = base0 + u * kStep;
      raw[u] = base < hi ? __builtin_nontemporal_load(reinterpret_cast<const u32x4c*>(row + base))   // read once
                        : u32x4c{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int base = base0 + u * kStep;
      if (base >= hi) break;
      float x[kPiece];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        x[2 * e] = bf16_bits_to_float(raw[u][e] & 0xffffu);
        x[2 * e + 1] = bf16_bits_to_float(raw[u][e] >> 16);
      }
      if (base + kPiece > hi) {
#pragma unroll
        for (int e = 0; e < kPiece; ++e)
          if (base + e >= hi) x[e] = -INFINITY;
      }
      float cm = x[0];
      int ci = 0;
#pragma unroll
      for (int e = 1; e < kPiece; ++e)
        if (x[e] > cm) { cm = x[e]; ci = e; }
      if (cm > p.m) {   // strict: the earlier index keeps a tie
        p.s *= __builtin_amdgcn_exp2f((p.m - cm) * kLog2e);
        p.m = cm;
        p.idx = base + ci;
      }
      float add = 0.f;
#pragma unroll
      for (int e = 0; e < kPiece; ++e) add += __builtin_amdgcn_exp2f((x[e] - p.m) * kLog2e);
      p.s += add;
    }
  }
  // wave reduction, then across the 4 waves through LDS
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    Partial o;
    o.m = __shfl_xor(p.m, off, 64);
    o.s = __shfl_xor(p.s, off, 64);
    o.idx = __shfl_xor(p.idx, off, 64);
    o.pad = 0;
    p = join(p, o);
  }
  __shared__ Partial sm[kScanThreads / 64];
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = p;
  __syncthreads();
  if (threadIdx.x == 0) {
    Partial r = sm[0];
#pragma unroll
    for (int w = 1; w < kScanThreads / 64; ++w) r = join(r, sm[w]);
    part[(int64_t)t * n_seg + seg] = r;
  }
}

// One wave per request (4 requests per block), or one wave per 64 tokens when there is no
// per-request rule.  Lane l joins the segments of tokens l, l+64, ... of the request.
__global__ __launch_bounds__(256) void commit_decide_kernel(
    const Partial* __restrict__ part, int n_seg, int num_tokens, int n_units, float threshold,
    const int32_t* __restrict__ cu_q, int min_commit, int32_t* __restrict__ token_out,
    float* __restrict__ conf_out, int32_t* __restrict__ commit_out) {
  const int lane = threadIdx.x & 63;
  const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (unit >= n_units) return;   // whole wave
  int t_lo, t_hi;
  if (cu_q) { t_lo = cu_q[unit]; t_hi = cu_q[unit + 1]; }
  else { t_lo = unit * 64; t_hi = min(num_tokens, t_lo + 64); }
  float best_conf = -1.f;
  int best_t = 0x7fffffff, any = 0;
  for (int t = t_lo + lane; t < t_hi; t += 64) {
    Partial r = part[(int64_t)t * n_seg];
    for (int s = 1; s < n_seg; ++s) r = join(r, part[(int64_t)t * n_seg + s]);
    const float conf = 1.f / r.s;   // exp(max - max) / sum
    const int com = conf > threshold ? 1 : 0;
    token_out[t] = r.idx;
    conf_out[t] = conf;
    commit_out[t] = com;
    any |= com;
    if (conf > best_conf) { best_conf = conf; best_t = t; }   // strict: first on ties
  }
  if (!cu_q || min_commit < 1) return;
  // progress rule: nothing above the threshold -> commit the most confident token (first on ties)
  if (__builtin_amdgcn_ballot_w64(any != 0) != 0 || t_hi <= t_lo) return;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float oc = __shfl_xor(best_conf, off, 64);
    const int ot = __shfl_xor(best_t, off, 64);
    if (oc > best_conf || (oc == best_conf && ot < best_t)) { best_conf = oc; best_t = ot; }
  }
  // the store follows this wave's own stores to commit_out in program order
  if (lane == 0) commit_out[best_t] = 1;
}

static int commit_segments(const optimus_commit_params_t& p, int* seg_len_out) {
  // enough blocks to fill the chip, segments a multiple of one block iteration
  // about 8192 blocks: several rounds over the chip's 2048 resident blocks, so that the last,
  // partly filled round costs little
  int n_seg = (8192 + p.num_tokens - 1) / (p.num_tokens > 0 ? p.num_tokens : 1);
  n_seg = n_seg < 1 ? 1 : (n_seg > 64 ? 64 : n_seg);
  int seg_len = ((p.vocab + n_seg - 1) / n_seg + kStep - 1) / kStep * kStep;  // a multiple of 8: pieces stay aligned
  n_seg = (p.vocab + seg_len - 1) / seg_len;
  *seg_len_out = seg_len;
  return n_seg;
}

static bool commit_params_ok(const optimus_commit_params_t* p) {
  return p && p->num_tokens >= 0 && p->num_tokens <= 65535 && p->vocab >= 1 && p->row_stride % 8 == 0 &&
         p->row_stride >= ((int64_t)p->vocab + 7) / 8 * 8 && p->batch >= 0 &&
         (p->min_commit == 0 || p->min_commit == 1);
}

}  // namespace optimus

using namespace optimus;

extern "C" size_t optimus_commit_workspace_bytes(const optimus_commit_params_t* params) {
  if (!commit_params_ok(params)) return 0;
  int seg_len;
  const int n_seg = commit_segments(*params, &seg_len);
  return (size_t)params->num_tokens * n_seg * sizeof(Partial) + 16;
}

extern "C" int optimus_commit_forward(const optimus_commit_params_t* params, int device,
                                      const void* logits, const int32_t* cu_q, int32_t* token_out,
                                      float* conf_out, int32_t* commit_out, void* workspace,
                                      size_t workspace_bytes, void* hip_stream) {
  if (!commit_params_ok(params) || device < 0) return OPTIMUS_ERR_INVALID_ARGUMENT;
  const optimus_commit_params_t& p = *params;
  if (p.num_tokens == 0) return OPTIMUS_OK;
  if (!logits || !token_out || !conf_out || !commit_out || !workspace) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (p.batch > 0 && !cu_q) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (((uintptr_t)logits | (uintptr_t)workspace) & 15) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (workspace_bytes < optimus_commit_workspace_bytes(params)) return OPTIMUS_ERR_WORKSPACE_TOO_SMALL;
  hipError_t e = hipSetDevice(device);
  if (e != hipSuccess) { set_hip_error((int)e, "hipSetDevice"); return OPTIMUS_ERR_HIP; }
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  int seg_len;
  const int n_seg = commit_segments(p, &seg_len);
  Partial* part = reinterpret_cast<Partial*>(workspace);
  hipLaunchKernelGGL(commit_scan_kernel, dim3(n_seg, p.num_tokens), dim3(kScanThreads), 0, s,
                     (const uint16_t*)logits, p.vocab, p.row_stride, seg_len, part);
  const bool per_req = p.batch > 0;
  const int units = per_req ? p.batch : (p.num_tokens + 63) / 64;
  hipLaunchKernelGGL(commit_decide_kernel, dim3((units + 3) / 4), dim3(256), 0, s, part, n_seg,
                     p.num_tokens, units, p.threshold, per_req ? cu_q : nullptr, p.min_commit, token_out, conf_out,
                     commit_out);
  e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error((int)e, "commit kernel launch"); return OPTIMUS_ERR_HIP; }
  return OPTIMUS_OK;
}
