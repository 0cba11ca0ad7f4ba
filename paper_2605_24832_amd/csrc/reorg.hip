// Step-wise reorganisation of streaming chunked decoding on gfx950 (Optimus
// Sec. 4.4): from the decoded flags of every request's current block and the
// chunk size the scheduler asked for, build this step's chunk: the first c
// undecoded positions of the block, the ragged offsets cu_q, the cached length
// and, per chunk token, its sequence position, its KV slot and its request.
// Integer work only: results are exact.
#include <hip/hip_runtime.h>

#include "optimus_attn.h"
#include "plan_internal.h"

namespace optimus {

// One block: chunk sizes, cached lengths and the exclusive scan cu_q over all requests.
__global__ __launch_bounds__(1024) void reorg_count_kernel(
    const uint8_t* __restrict__ decoded, const int32_t* __restrict__ block_start,
    const int32_t* __restrict__ chunk_req, int batch, int block_size, int32_t* __restrict__ chunk_out,
    int32_t* __restrict__ cu_q_out, int32_t* __restrict__ prefix_len_out) {
  __shared__ int32_t sm[1024];
  __shared__ int32_t carry;
  if (threadIdx.x == 0) { carry = 0; cu_q_out[0] = 0; }
  __syncthreads();
  for (int base = 0; base < batch; base += 1024) {
    const int i = base + threadIdx.x;
    int c = 0;
    if (i < batch) {
      int n_dec = 0;
      const uint8_t* row = decoded + (int64_t)i * block_size;
      for (int b = 0; b < block_size; ++b) n_dec += row[b] != 0;
      c = min(max(chunk_req[i], 0), block_size - n_dec);
      chunk_out[i] = c;
      prefix_len_out[i] = block_start[i] + n_dec;
    }
    // inclusive scan of c over the block (Hillis-Steele in LDS)
    sm[threadIdx.x] = c;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
      const int v = threadIdx.x >= off ? sm[threadIdx.x - off] : 0;
      __syncthreads();
      sm[threadIdx.x] += v;
      __syncthreads();
    }
    if (i < batch) cu_q_out[i + 1] = carry + sm[threadIdx.x];
    __syncthreads();
    if (threadIdx.x == 1023) carry += sm[1023];
    __syncthreads();
  }
}

// One wave per request: lane l looks at block positions l, l+64, ...; the rank of an
// undecoded position among the undecoded ones comes from a ballot and a prefix popcount.
__global__ __launch_bounds__(256) void reorg_emit_kernel(
    const uint8_t* __restrict__ decoded, const int32_t* __restrict__ block_start,
    const int32_t* __restrict__ chunk, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ prefix_len, int batch, int block_size, int32_t* __restrict__ q_pos,
    int32_t* __restrict__ kv_slot, int32_t* __restrict__ token_req) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= batch) return;   // whole wave
  const int c = chunk[i], t0 = cu_q[i], L = prefix_len[i], s = block_start[i];
  const uint8_t* row = decoded + (int64_t)i * block_size;
  int taken = 0;   // undecoded positions before this group of 64
  for (int b0 = 0; b0 < block_size && taken < c; b0 += 64) {
    const int b = b0 + lane;
    const bool undec = b < block_size && row[b] == 0;
    const unsigned long long mask = __builtin_amdgcn_ballot_w64(undec);
    const int rank = taken + __popcll(mask & ((1ull << lane) - 1ull));
    if (undec && rank < c) {
      q_pos[t0 + rank] = s + b;
      kv_slot[t0 + rank] = L + rank;
      token_req[t0 + rank] = i;
    }
    taken += __popcll(mask);
  }
}

}  // namespace optimus

using namespace optimus;

extern "C" int optimus_reorg_forward(int device, int32_t batch, int32_t block_size,
                                     const uint8_t* decoded, const int32_t* block_start,
                                     const int32_t* chunk_req, int32_t* chunk_out,
                                     int32_t* cu_q_out, int32_t* prefix_len_out, int32_t* q_pos_out,
                                     int32_t* kv_slot_out, int32_t* token_req_out,
                                     void* hip_stream) {
  if (device < 0 || batch < 0 || block_size < 1 || block_size > 4096) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (!cu_q_out) return OPTIMUS_ERR_INVALID_ARGUMENT;
  if (batch > 0 && (!decoded || !block_start || !chunk_req || !chunk_out || !prefix_len_out ||
                    !q_pos_out || !kv_slot_out || !token_req_out))
    return OPTIMUS_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(device);   // the caller's current device is put back on return
  if (guard.status() != OPTIMUS_OK) return guard.status();
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  hipLaunchKernelGGL(reorg_count_kernel, dim3(1), dim3(1024), 0, s, decoded, block_start, chunk_req,
                     batch, block_size, chunk_out, cu_q_out, prefix_len_out);
  if (batch > 0)
    hipLaunchKernelGGL(reorg_emit_kernel, dim3((batch + 3) / 4), dim3(256), 0, s, decoded,
                       block_start, chunk_out, cu_q_out, prefix_len_out, batch, block_size,
                       q_pos_out, kv_slot_out, token_req_out);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_hip_error((int)e, "reorg kernel launch"); return OPTIMUS_ERR_HIP; }
  return OPTIMUS_OK;
}
