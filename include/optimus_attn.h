/*
 * optimus_attn.h - C ABI of the MI355X (gfx950) chunked block-diffusion
 * attention library.
 *
 * The operation is the attention step of Optimus's elastic diffusion decoding
 * (Sec. 4 "Streaming Chunked Decoding", Sec. 6 "Implementation"): in one
 * decoding iteration each request i of a continuously batched set contributes
 * a chunk of c_i query tokens (c_i is re-chosen every iteration by the elastic
 * scheduler, Sec. 5); the chunk's K/V are mapped into the paged KV cache and
 * the chunk attends to the request's cached tokens (all visible: earlier
 * blocks and committed tokens of the current block, Sec. 2.3 / 4.2) and to
 * itself bidirectionally (in-block streaming, Sec. 7.2).
 *
 * Conventions
 *   - All pointers named *_host are host memory, all others are device memory
 *     on the plan's device.  The caller owns every buffer; the plan owns only
 *     its private descriptor copies and work list.
 *   - bf16 tensors are raw 16-bit patterns.  q/out: [T, Hq, D]; k_new/v_new:
 *     [T, Hkv, D]; T = cu_q[batch]; token t of request i, chunk index j is
 *     t = cu_q[i] + j.  Query head h reads kv head h / (Hq/Hkv).
 *   - Paged pool: the tile of (page, kv head) starts at element
 *     page*stride_page + head*stride_head and holds P*D elements in the
 *     "grouped-K / slot-contiguous-V" layout
 *         K[slot][d] at ((d/8)*P + slot)*8 + d%8
 *         V[slot][d] at d*P + slot
 *     (8-element = 16-byte groups of the head dim: one 16x16x32 MFMA operand
 *     register set per lane; a wave-wide load of a page tile is contiguous).
 *     Logical slot n of request i lives in page block_table[i][n / P], in-page
 *     slot n % P.  Slots at or beyond L_i + c_i and unreferenced pages are
 *     never read into a result, whatever they hold (NaN included).
 *   - How K/V get into that layout: only through this library.  The K/V of
 *     a prompt or of any other already computed tokens (prefix caching, Sec.
 *     4.2) are written with optimus_kv_write from plain [n, Hkv, D] rows;
 *     the K/V of the chunk of a decoding iteration with optimus_kv_append.
 *     Both take the same rows and produce the same bytes for the same slots.
 *   - Every call returns an optimus_status_t (0 = OK, negative = error) and
 *     never throws.  Kernel launches are asynchronous on the given stream.
 *     Device calls run on the device they are given (the plan's) and put the
 *     calling thread's current device back before they return.
 */
#ifndef OPTIMUS_ATTN_H_
#define OPTIMUS_ATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  OPTIMUS_OK = 0,
  OPTIMUS_ERR_INVALID_ARGUMENT = -1,   /* null pointer, negative size, bad enum       */
  OPTIMUS_ERR_UNSUPPORTED_SHAPE = -2,  /* head_dim, page_size, Hq % Hkv, layout        */
  OPTIMUS_ERR_BAD_CU_Q = -3,           /* cu_q[0] != 0 or decreasing                   */
  OPTIMUS_ERR_BAD_PREFIX = -4,         /* L_i < 0, s_i < 0 or s_i > L_i                */
  OPTIMUS_ERR_CHUNK_EXCEEDS_BLOCK = -5,/* in-block mode: (L_i - s_i) + c_i > B         */
  OPTIMUS_ERR_BLOCK_TABLE_TOO_SHORT = -6, /* ceil((L_i+c_i)/P) > max_pages_per_req     */
  OPTIMUS_ERR_PAGE_OUT_OF_RANGE = -7,  /* a referenced block-table entry not in [0,num_pages) */
  OPTIMUS_ERR_WORKSPACE_TOO_SMALL = -8,
  OPTIMUS_ERR_NOT_PLANNED = -9,        /* forward/append before a successful plan_update */
  OPTIMUS_ERR_NO_DEVICE = -10,         /* device call on a host-only plan              */
  OPTIMUS_ERR_HIP = -11                /* a HIP runtime call failed; see optimus_last_hip_error */
} optimus_status_t;

typedef struct optimus_attn_plan optimus_attn_plan_t; /* opaque */

/* Problem geometry, fixed for the life of a plan. */
typedef struct {
  int32_t num_q_heads;       /* Hq                                              */
  int32_t num_kv_heads;      /* Hkv, Hq % Hkv == 0                              */
  int32_t head_dim;          /* D in {64, 128}                                  */
  int32_t page_size;         /* P in {16, 32, 64, 128}                          */
  int32_t block_size;        /* B, diffusion block (32 in the paper's models)   */
  int32_t mask_mode;         /* 0 in-block streaming (Sec. 7.2 default): chunk
                                bidirectional.  1 out-block streaming read as
                                block-causal inside the chunk: chunk key k is
                                visible to chunk query j iff
                                (d_i+k)/B <= (d_i+j)/B, d_i = L_i - s_i.        */
  int32_t out_dtype;         /* 0 bf16, 1 fp32                                  */
  int32_t kv_layout;         /* must be 1 (layout described above)              */
  float   softmax_scale;     /* <= 0 -> 1/sqrt(D)                               */
  int32_t num_pages;         /* pool size, for block-table validation           */
  int32_t max_pages_per_req; /* row stride of the block table                   */
  int32_t reserved0;
  int64_t k_stride_page, k_stride_head; /* elements; multiples of 8; page strides
                                           below 2^31                            */
  int64_t v_stride_page, v_stride_head; /* elements; multiples of 8             */
} optimus_attn_params_t;

/* One unit of device work, exposed so that host tests can check that the plan
 * covers every (request, kv head, query row, key) exactly once.  The rows of
 * a (request, kv head) pair are r = j*G + u for chunk token j and head u of
 * the group (G = Hq/Hkv), r in [0, c_i*G).                                    */
typedef struct {
  int32_t req;         /* request index i                                       */
  int32_t kv_head;     /* g                                                     */
  int32_t row_begin;   /* first row of this q tile                              */
  int32_t row_count;   /* rows in this q tile (1..128)                          */
  int32_t kv_begin;    /* first logical key slot, multiple of 32                */
  int32_t kv_end;      /* one past the last key slot, <= L_i + c_i              */
  int32_t part_row;    /* -1: writes final output; else first row of its partial
                          in the workspace                                      */
  int32_t q_token0;    /* cu_q[i]                                               */
} optimus_work_item_t;

/* Create a plan.  device >= 0: HIP device ordinal that all later device calls
 * of this plan use.  device == -1: host-only plan (validation and planning
 * work; kv_append / forward return OPTIMUS_ERR_NO_DEVICE).                     */
int optimus_attn_plan_create(const optimus_attn_params_t* params, int device,
                             optimus_attn_plan_t** plan_out);

/* Per-iteration planning (host).  Validates the descriptors, tiles the query
 * rows, chooses the KV split of every (request, kv head) so the launch fills
 * the chip, builds the work list and uploads it.  Arrays are host memory and
 * are copied; they may be freed on return.
 *   cu_q_host        [batch+1], cu_q[0] == 0, non-decreasing (c_i = 0 allowed)
 *   prefix_len_host  [batch]   L_i >= 0 cached tokens
 *   block_start_host [batch]   s_i, 0 <= s_i <= L_i, origin of the current block
 *   block_table_host [batch, max_pages_per_req] or NULL (skips page-id checks)
 *   workspace_bytes_out  bytes of scratch that optimus_attn_forward needs
 * The upload of the work list is enqueued by the next kv_append / forward on
 * that call's stream, behind the kernels of earlier iterations, so updates may
 * run ahead of the device as long as one plan is used on one stream at a time
 * (the host blocks only when it is four updates ahead).  batch == 0 is a valid
 * no-op plan.                                                                  */
int optimus_attn_plan_update(optimus_attn_plan_t* plan, int32_t batch,
                             const int32_t* cu_q_host, const int32_t* prefix_len_host,
                             const int32_t* block_start_host,
                             const int32_t* block_table_host,
                             size_t* workspace_bytes_out);

/* Sec. 6: map the chunk's K/V into the paged cache.  Chunk token j of request
 * i is written to logical slot L_i + j, overwriting the slot (chunk KV is
 * provisional until commit, Sec. 4.1).  k_new, v_new: bf16 [T, Hkv, D].
 * Index arithmetic is exact; the payload is a bit copy.                        */
int optimus_kv_append(optimus_attn_plan_t* plan, void* k_pool, void* v_pool,
                      const void* k_new, const void* v_new,
                      const int32_t* block_table, void* hip_stream);

/* Sec. 4.2 (cached prefix) / Sec. 6 (K/V states mapped into the paged cache), without a
 * plan: tokens 0..n-1 of k_src / v_src (bf16 [n, Hkv, D], device memory, 16-byte aligned)
 * are written to the logical slots first_slot .. first_slot+n-1 of request `req`, i.e. to
 * page block_table[req][slot / P], in the pool layout described at the top; whatever the
 * slots held is overwritten.  This is how a prompt's K/V (prefill) or recomputed K/V of
 * committed tokens reach the pool; there is no limit on n other than the block-table row.
 * `params` gives the geometry (same validation as optimus_attn_plan_create; mask_mode,
 * out_dtype and softmax_scale are not used).  block_table is device memory
 * [*, max_pages_per_req]; entries outside [0, num_pages) make the kernel skip that page's
 * tokens.  Nothing is allocated; asynchronous on the stream; the caller's current device
 * is left unchanged.  Errors: OPTIMUS_ERR_INVALID_ARGUMENT (null / misaligned pointers,
 * negative req / first_slot / n), OPTIMUS_ERR_UNSUPPORTED_SHAPE,
 * OPTIMUS_ERR_BLOCK_TABLE_TOO_SHORT (ceil((first_slot+n)/P) > max_pages_per_req).         */
int optimus_kv_write(const optimus_attn_params_t* params, int device, void* k_pool, void* v_pool,
                     const void* k_src, const void* v_src, const int32_t* block_table,
                     int32_t req, int32_t first_slot, int32_t n, void* hip_stream);

/* Sec. 6: attention of every chunk over its cached prefix and itself.  The
 * chunk's K/V must already be in the pool (optimus_kv_append on the same
 * stream).  out: [T, Hq, D] in params.out_dtype.  workspace: device scratch
 * of at least the size plan_update reported (may be NULL if that was 0); it
 * holds split-KV partials and is fully overwritten before it is read.          */
int optimus_attn_forward(optimus_attn_plan_t* plan, const void* q, const void* k_pool,
                         const void* v_pool, const int32_t* block_table, void* out,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* optimus_attn_forward with the sequence positions of the chunk tokens (Sec. 4.4: the chunk is
 * rebuilt every step from the positions not yet decoded, which need not be contiguous; Sec. 7.2
 * out-block streaming lets it cross a block boundary).  q_pos: int32 [T] device memory, e.g.
 * q_pos_out of optimus_reorg_forward, or NULL (= optimus_attn_forward).  Only mask_mode 1 looks
 * at it: chunk key k is visible to chunk query j iff
 * (q_pos[k] - s_i) / B <= (q_pos[j] - s_i) / B.  Preconditions: q_pos >= s_i and non-decreasing
 * within a request's chunk (the order optimus_reorg_forward emits); for other orders the
 * visible keys are taken to be the first n chunk keys, n = number of chunk keys whose position
 * lies before the end of the query's block.  No memory access depends on a position value.  */
int optimus_attn_forward_pos(optimus_attn_plan_t* plan, const void* q, const void* k_pool,
                             const void* v_pool, const int32_t* block_table, const int32_t* q_pos,
                             void* out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* One decoding iteration in one call: optimus_attn_plan_update, optimus_kv_append and
 * optimus_attn_forward_pos (Sec. 4.4: chunk sizes and cached lengths change every iteration, so
 * planning is part of every step; Sec. 6 for the other two).  Same arguments, same launches and
 * same results as the three calls; what it saves is two library calls and their argument
 * marshalling, which count next to kernels of a few microseconds.  workspace_bytes is the
 * capacity of `workspace`: if the new plan needs more, OPTIMUS_ERR_WORKSPACE_TOO_SMALL is
 * returned after planning and nothing is launched (the split-KV partials need
 * 4 x (D+2) bytes per query row and split).  q_pos may be NULL.                             */
int optimus_attn_step(optimus_attn_plan_t* plan, int32_t batch, const int32_t* cu_q_host,
                      const int32_t* prefix_len_host, const int32_t* block_start_host,
                      const int32_t* block_table_host, const void* q, const void* k_new, const void* v_new,
                      void* k_pool, void* v_pool, const int32_t* block_table, const int32_t* q_pos,
                      void* out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* optimus_attn_forward for callers that cannot allocate or provide scratch memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments,
 * same kernels and same results as optimus_attn_forward, except that the split-KV partials go
 * to a static device array of the library instead of a workspace
 * (optimus_attn_static_scratch_bytes() = 64 MiB, held by every GPU the library runs on until
 * the process ends; its address on the plan's device is looked up in
 * optimus_attn_plan_create).  The call itself allocates nothing (no hipMalloc / hipFree, no
 * event creation: it records no timing for optimus_attn_timing_read).  A plan whose
 * plan_update reported more workspace than that returns OPTIMUS_ERR_WORKSPACE_TOO_SMALL and
 * nothing is launched.  The scratch is fully overwritten before it is read, so nothing has to
 * be cleared between calls; but all calls on one GPU share it: two calls that may overlap in
 * time (different streams, different plans or threads) race on it and must be serialised by
 * the caller.  Planning still happens in optimus_attn_plan_update, which may allocate when a
 * work list outgrows the plan's buffers: under graph capture, update the plan beforehand.   */
int optimus_attn_forward_static(optimus_attn_plan_t* plan, const void* q, const void* k_pool,
                                const void* v_pool, const int32_t* block_table, void* out,
                                void* hip_stream);
size_t optimus_attn_static_scratch_bytes(void);

void optimus_attn_plan_destroy(optimus_attn_plan_t* plan);

/* Introspection of the current work list (host). */
int32_t optimus_attn_plan_num_work_items(const optimus_attn_plan_t* plan);
int32_t optimus_attn_plan_num_merge_items(const optimus_attn_plan_t* plan);
/* Copies up to capacity items; returns the number copied or a negative status. */
int32_t optimus_attn_plan_get_work_items(const optimus_attn_plan_t* plan,
                                         optimus_work_item_t* items_out, int32_t capacity);

/* Planner knobs (host).  target_items: aim for at least this many work items
 * (0 = default: the list is fitted to whole rounds of the workgroups that are
 * resident at once, two per compute unit).
 * min_split_tokens / max_split_tokens: bounds on the keys one work item scans
 * (multiples of 32; 0 = default).                                               */
int optimus_attn_plan_set_tuning(optimus_attn_plan_t* plan, int32_t target_items,
                                 int32_t min_split_tokens, int32_t max_split_tokens);

/* Optional timing of the attention main kernel with HIP events recorded on the
 * caller's stream around its launch.  set_timing(every): 0 turns recording off;
 * n >= 1 clears the record and times the kernel of every n-th forward from now
 * on (two event records cost the host about 3 us per timed forward, which
 * shows in a step of 25 us: sample).  timing_read synchronises on the recorded
 * events and returns the summed milliseconds and the number of forwards timed
 * since then (at most 4096 are kept; later ones are dropped).                   */
int optimus_attn_set_timing(optimus_attn_plan_t* plan, int32_t every);
int optimus_attn_timing_read(optimus_attn_plan_t* plan, float* total_ms_out,
                             int32_t* forwards_out);

/* ---------------------------------------------------------------------------
 * Commit step (Sec. 2.3, Sec. 4.1; threshold 0.9 in Sec. 7.1): every chunk
 * position gets a confidence and the positions whose confidence exceeds the
 * threshold are committed.  Reading: confidence = largest softmax probability
 * of the position's logit row, token = first index attaining it.  A logit
 * that is -inf or NaN is an entry that cannot be chosen and adds nothing to
 * the softmax; a row without any other entry gets token 0, confidence 0.
 * With min_commit = 1 a request that has chunk tokens but none above the
 * threshold commits its most confident one (first on ties), so decoding
 * always advances.
 * All pointers are device memory; nothing is allocated and no scratch is
 * needed; asynchronous on the stream.                                          */
typedef struct {
  int32_t num_tokens;   /* T = rows of logits, <= 2^24                           */
  int32_t vocab;        /* V >= 1 used entries per row                           */
  int64_t row_stride;   /* elements between rows: multiple of 8, >= V rounded up
                           to a multiple of 8 (rows are read in 16-byte pieces)  */
  float   threshold;    /* commit iff confidence > threshold                     */
  int32_t batch;        /* requests described by cu_q; 0 = no per-request rule   */
  int32_t min_commit;   /* 0 or 1                                                */
  int32_t reserved0;
} optimus_commit_params_t;

/* logits: bf16 [T, row_stride], 16-byte aligned.  cu_q: int32 [batch+1] (ignored if
 * batch == 0).  token_out int32 [T], conf_out fp32 [T], commit_out int32 [T] (0/1).
 * Returns OPTIMUS_ERR_INVALID_ARGUMENT for parameters outside the ranges above or
 * null / misaligned pointers.                                                   */
int optimus_commit_forward(const optimus_commit_params_t* params, int device, const void* logits,
                           const int32_t* cu_q, int32_t* token_out, float* conf_out,
                           int32_t* commit_out, void* hip_stream);

/* ---------------------------------------------------------------------------
 * Step-wise reorganisation (Sec. 4.4): rebuild every request's chunk for this
 * step from the tokens decoded so far.  Reading: the chunk is the first
 * min(chunk_req_i, undecoded_i) not yet decoded positions of the current block
 * (in-block streaming, Sec. 7.2), in sequence order; the decoded positions of
 * the block are cached, so the cached length is block_start_i + decoded_i and
 * chunk token j uses KV slot cached length + j.
 * All pointers are device memory; nothing is allocated; asynchronous.
 *   decoded       uint8 [batch, block_size], non-zero = decoded
 *   block_start   int32 [batch]  sequence position of the block's first token
 *   chunk_req     int32 [batch]  chunk size asked for (negative counts as 0)
 *   chunk_out     int32 [batch]; cu_q_out int32 [batch+1]; prefix_len_out int32 [batch]
 *   q_pos_out, kv_slot_out, token_req_out  int32 [>= sum of chunk_out] (at most
 *       sum of min(chunk_req, block_size)): sequence position, KV slot and
 *       request of every chunk token, ordered by request then position.       */
int optimus_reorg_forward(int device, int32_t batch, int32_t block_size, const uint8_t* decoded,
                          const int32_t* block_start, const int32_t* chunk_req,
                          int32_t* chunk_out, int32_t* cu_q_out, int32_t* prefix_len_out,
                          int32_t* q_pos_out, int32_t* kv_slot_out, int32_t* token_req_out,
                          void* hip_stream);

/* ---------------------------------------------------------------------------
 * Saturation-aware chunk-size selection (Sec. 5).  Host memory only, no GPU.
 *
 * Latency model (Sec. 5.2): one continuous curve over the step's token count
 * x = batch * chunk with three affine regimes: memory-bound, transition, compute-bound.
 *   T(x) = beta1[k] * x + beta0[k],  k = 0 if x < x_break[0], 1 if x < x_break[1], else 2,
 * and neighbouring regimes take the same value at the boundary between them.               */
typedef struct optimus_latency_model {
  double x_break[2];
  double beta1[3];
  double beta0[3];
} optimus_latency_model_t;

/* Fit the model to profiled samples (x_i, latency_i), 6 <= num_samples <= 2048, in any order.
 * Reading (the paper says only that the coefficients come from offline profiling): the curve is
 *   T(x) = alpha + beta x + gamma0 max(0, x - b0) + gamma1 max(0, x - b1),
 * the boundaries b0 < b1 are profiled loads strictly between the smallest and the largest one,
 * for a pair of boundaries the four parameters are the least-squares solution, and the pair
 * with the smallest squared error is kept (the first such pair in (b0, b1) order).  sse_out
 * (may be NULL) receives the squared error of the returned model.
 * Returns OPTIMUS_ERR_INVALID_ARGUMENT for null pointers, non-finite or negative samples, or
 * fewer than four distinct loads.                                                          */
int optimus_latency_fit(int32_t num_samples, const double* x, const double* latency,
                        optimus_latency_model_t* model_out, double* sse_out);
/* T(x) of the model (NaN for a null model). */
double optimus_latency_eval(const optimus_latency_model_t* model, double x);

/* Sec. 5.1: best_index_out = argmax_i n_commit[i] * batch / T(batch * chunk_sizes[i]) over the
 * num_candidates candidate chunk sizes (first index on ties); n_commit[i] is the caller's
 * estimate of tokens committed per request and step at chunk_sizes[i] (Sec. 5.3).  rate_out
 * (may be NULL) receives the num_candidates objective values (tokens per latency unit).
 * Returns OPTIMUS_ERR_INVALID_ARGUMENT for null pointers, batch < 1, a chunk size < 1, a
 * negative or NaN n_commit, or a model latency that is not positive at a candidate.          */
int optimus_select_chunk(const optimus_latency_model_t* model, int32_t batch,
                         int32_t num_candidates, const int32_t* chunk_sizes,
                         const double* n_commit, int32_t* best_index_out, double* rate_out);

const char* optimus_status_string(int status);
/* Text of the last HIP error seen by this thread inside the library ("" if none). */
const char* optimus_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* OPTIMUS_ATTN_H_ */
