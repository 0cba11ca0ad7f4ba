/*
 * CPU oracle for the chunked block-diffusion attention step of elastic
 * diffusion decoding (Optimus, Sec. 4 "Streaming Chunked Decoding" and
 * Sec. 6 "Implementation": a paged-attention kernel that maps per-chunk KV
 * into the paged cache and attends over variable-length query chunks).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the plain definition written out
 * in fp64, slow on purpose, and shares nothing with the HIP path: only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What it computes, for request i with c_i chunk (query) tokens, L_i cached
 * tokens and block origin s_i (d_i = L_i - s_i cached tokens already inside
 * the current block), query head h, kv head g = h / (Hq/Hkv):
 *
 *   key set   = cached slots 0..L_i-1, read through the block table from the
 *               paged pool, followed by the c_i chunk tokens (taken from
 *               k_new / v_new, i.e. independent of the append step);
 *               every cached token is visible: it lies in an earlier block or
 *               is a committed token of the current block (Sec. 2.3 block
 *               diffusion; Sec. 4.2 prefix caching);  the not-yet-computed
 *               suffix of the block is not a key at all (Sec. 4.3);
 *   mask      = mode 0 (in-block streaming, Sec. 7.2, the default): the chunk
 *               is bidirectional, all c_i chunk keys visible to all c_i
 *               queries;  mode 1 (out-block streaming, Sec. 7.2, read as
 *               block-causal): chunk key k visible to chunk query j iff
 *               floor((d_i+k)/B) <= floor((d_i+j)/B); with explicit sequence
 *               positions pos[] of the chunk tokens (Sec. 4.4: the chunk is
 *               the not yet decoded positions, which need not be contiguous)
 *               iff floor((pos[k]-s_i)/B) <= floor((pos[j]-s_i)/B);
 *   scores    = scale * <q, K_n>,  softmax over the visible keys,
 *   output    = sum_n p_n V_n.
 *
 * Inputs are bf16 bit patterns (uint16_t); all arithmetic is fp64.
 *
 * Pool layouts (kv_layout), element offsets inside one (page, kv head) tile:
 *   0: K[slot][d] -> slot*D + d            V[slot][d] -> slot*D + d
 *   1: K[slot][d] -> ((d/8)*P + slot)*8 + d%8      (8-element d groups)
 *      V[slot][d] -> d*P + slot                    (slot-contiguous)
 * The tile of (page, head) starts at page*stride_page + head*stride_head.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t num_q_heads;   /* Hq  */
  int32_t num_kv_heads;  /* Hkv */
  int32_t head_dim;      /* D   */
  int32_t page_size;     /* P   */
  int32_t block_size;    /* B   */
  int32_t mask_mode;     /* 0 in-block bidirectional, 1 block-causal inside chunk */
  int32_t kv_layout;     /* 0 plain, 1 grouped-K / slot-contiguous-V */
  int32_t max_pages_per_req; /* row stride of block_table */
  int64_t k_stride_page, k_stride_head; /* elements */
  int64_t v_stride_page, v_stride_head; /* elements */
  double scale;          /* <=0 -> 1/sqrt(D) */
} oracle_params_t;

static double bf16_to_double(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

static int64_t k_offset(const oracle_params_t *p, int64_t page, int head, int slot, int d) {
  int64_t base = page * p->k_stride_page + (int64_t)head * p->k_stride_head;
  if (p->kv_layout == 0) return base + (int64_t)slot * p->head_dim + d;
  return base + ((int64_t)(d / 8) * p->page_size + slot) * 8 + d % 8;
}

static int64_t v_offset(const oracle_params_t *p, int64_t page, int head, int slot, int d) {
  int64_t base = page * p->v_stride_page + (int64_t)head * p->v_stride_head;
  if (p->kv_layout == 0) return base + (int64_t)slot * p->head_dim + d;
  return base + (int64_t)d * p->page_size + slot;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Step "KV append" (Sec. 6: per-chunk KV states are mapped into the paged
 * cache): chunk token j of request i goes to logical slot L_i + j, i.e. page
 * block_table[i][(L_i+j)/P], in-page slot (L_i+j)%P, overwriting what is there
 * (chunk KV is provisional and rewritten after commit, Sec. 4.1).            */
int oracle_kv_append(const oracle_params_t *p, int32_t batch, const int32_t *cu_q,
                     const int32_t *prefix_len, const int32_t *block_table,
                     const uint16_t *k_new, const uint16_t *v_new,
                     uint16_t *k_pool, uint16_t *v_pool) {
  const int D = p->head_dim, P = p->page_size, Hkv = p->num_kv_heads;
  for (int i = 0; i < batch; ++i) {
    int c = cu_q[i + 1] - cu_q[i];
    for (int j = 0; j < c; ++j) {
      int n = prefix_len[i] + j;
      int32_t page = block_table[(int64_t)i * p->max_pages_per_req + n / P];
      if (page < 0) return -1;
      int slot = n % P;
      int64_t t = cu_q[i] + j;
      for (int g = 0; g < Hkv; ++g)
        for (int d = 0; d < D; ++d) {
          k_pool[k_offset(p, page, g, slot, d)] = k_new[(t * Hkv + g) * D + d];
          v_pool[v_offset(p, page, g, slot, d)] = v_new[(t * Hkv + g) * D + d];
        }
    }
  }
  return 0;
}

/* Gather the key set of (request i, kv head g) into dense fp64 rows:
 * cached slots from the pool through the block table, then the chunk rows.   */
static int gather_keys(const oracle_params_t *p, int i, int g, const int32_t *cu_q,
                       const int32_t *prefix_len, const int32_t *block_table,
                       const uint16_t *k_new, const uint16_t *v_new,
                       const uint16_t *k_pool, const uint16_t *v_pool,
                       double *K, double *V) {
  const int D = p->head_dim, P = p->page_size, Hkv = p->num_kv_heads;
  const int L = prefix_len[i], c = cu_q[i + 1] - cu_q[i];
  for (int n = 0; n < L; ++n) {
    int32_t page = block_table[(int64_t)i * p->max_pages_per_req + n / P];
    if (page < 0) return -1;
    int slot = n % P;
    for (int d = 0; d < D; ++d) {
      K[(int64_t)n * D + d] = bf16_to_double(k_pool[k_offset(p, page, g, slot, d)]);
      V[(int64_t)n * D + d] = bf16_to_double(v_pool[v_offset(p, page, g, slot, d)]);
    }
  }
  for (int k = 0; k < c; ++k) {
    int64_t t = cu_q[i] + k;
    for (int d = 0; d < D; ++d) {
      K[(int64_t)(L + k) * D + d] = bf16_to_double(k_new[(t * Hkv + g) * D + d]);
      V[(int64_t)(L + k) * D + d] = bf16_to_double(v_new[(t * Hkv + g) * D + d]);
    }
  }
  return 0;
}

/* Is logical key n (0..L+c-1) visible to chunk query j of a request with
 * L cached tokens and d cached tokens inside the current block?  pos: NULL, or
 * the sequence positions of the request's chunk tokens (block origin s = L - d). */
static int key_visible(const oracle_params_t *p, int L, int d, int j, int n, const int32_t *pos) {
  if (n < L) return 1;                 /* cached prefix: always */
  if (p->mask_mode == 0) return 1;     /* in-block: bidirectional chunk */
  int k = n - L;
  if (pos) {
    int s = L - d;
    return (pos[k] - s) / p->block_size <= (pos[j] - s) / p->block_size;
  }
  return (d + k) / p->block_size <= (d + j) / p->block_size;
}

/* One query row: scores over keys [lo,hi), masked two-pass softmax pieces.
 * Writes the row maximum *m, the sum of exp(s-m) *l and, in o[D], the
 * un-normalised sum_n exp(s_n-m) V_n.  p_out (optional) gets exp(s_n-m) or 0.
 * If no key in range is visible: m=-inf, l=0, o=0.                            */
static void attend_row(const oracle_params_t *p, const double *q, const double *K,
                       const double *V, int L, int dblk, int j, int lo, int hi,
                       double scale, double *s, double *m, double *l, double *o,
                       double *p_out, const int32_t *pos) {
  const int D = p->head_dim;
  double mx = -INFINITY;
  for (int n = lo; n < hi; ++n) {
    if (!key_visible(p, L, dblk, j, n, pos)) { s[n - lo] = -INFINITY; continue; }
    double acc = 0.0;
    for (int d = 0; d < D; ++d) acc += q[d] * K[(int64_t)n * D + d];
    s[n - lo] = acc * scale;
    if (s[n - lo] > mx) mx = s[n - lo];
  }
  for (int d = 0; d < D; ++d) o[d] = 0.0;
  double z = 0.0;
  for (int n = lo; n < hi; ++n) {
    double e = (s[n - lo] == -INFINITY) ? 0.0 : exp(s[n - lo] - mx);
    if (p_out) p_out[n - lo] = e;
    if (e == 0.0) continue;
    z += e;
    for (int d = 0; d < D; ++d) o[d] += e * V[(int64_t)n * D + d];
  }
  *m = mx;
  *l = z;
}

/* Step "attention forward", whole batch.  out is fp64 [T, Hq, D].  q_pos: NULL, or the
 * sequence position of every chunk token (only looked at in mask mode 1).
 * q bf16 [T,Hq,D]; k_new, v_new bf16 [T,Hkv,D].  Returns 0, or -1 on a bad
 * descriptor (negative page id inside the cached range, Hq % Hkv != 0).      */
int oracle_chunked_attention_pos(const oracle_params_t *p, int32_t batch,
                                 const int32_t *cu_q, const int32_t *prefix_len,
                                 const int32_t *block_start, const int32_t *block_table,
                                 const uint16_t *q, const uint16_t *k_new,
                                 const uint16_t *v_new, const uint16_t *k_pool,
                                 const uint16_t *v_pool, const int32_t *q_pos /* [T] or NULL */,
                                 double *out) {
  const int D = p->head_dim, Hq = p->num_q_heads, Hkv = p->num_kv_heads;
  if (Hkv <= 0 || Hq % Hkv != 0) return -1;
  const int G = Hq / Hkv;
  const double scale = p->scale > 0.0 ? p->scale : 1.0 / sqrt((double)D);
  int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int i = 0; i < batch; ++i) {
    for (int h = 0; h < Hq; ++h) {
      const int L = prefix_len[i], c = cu_q[i + 1] - cu_q[i];
      if (c <= 0) continue;
      const int g = h / G, n_keys = L + c, dblk = L - block_start[i];
      double *K = (double *)malloc(sizeof(double) * (size_t)n_keys * D);
      double *V = (double *)malloc(sizeof(double) * (size_t)n_keys * D);
      double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
      double *qrow = (double *)malloc(sizeof(double) * (size_t)D);
      double *o = (double *)malloc(sizeof(double) * (size_t)D);
      if (gather_keys(p, i, g, cu_q, prefix_len, block_table, k_new, v_new, k_pool,
                      v_pool, K, V) != 0) {
#pragma omp atomic write
        err = -1;
      } else {
        for (int j = 0; j < c; ++j) {
          int64_t t = cu_q[i] + j;
          for (int d = 0; d < D; ++d) qrow[d] = bf16_to_double(q[(t * Hq + h) * D + d]);
          double m, l;
          attend_row(p, qrow, K, V, L, dblk, j, 0, n_keys, scale, s, &m, &l, o, NULL,
                     q_pos ? q_pos + cu_q[i] : NULL);
          for (int d = 0; d < D; ++d) out[(t * Hq + h) * D + d] = o[d] / l;
        }
      }
      free(K); free(V); free(s); free(qrow); free(o);
    }
  }
  return err;
}

/* The same with the chunk taken as contiguous after the cached tokens of the block. */
int oracle_chunked_attention(const oracle_params_t *p, int32_t batch,
                             const int32_t *cu_q, const int32_t *prefix_len,
                             const int32_t *block_start, const int32_t *block_table,
                             const uint16_t *q, const uint16_t *k_new,
                             const uint16_t *v_new, const uint16_t *k_pool,
                             const uint16_t *v_pool, double *out) {
  return oracle_chunked_attention_pos(p, batch, cu_q, prefix_len, block_start, block_table, q,
                                      k_new, v_new, k_pool, v_pool, NULL, out);
}

/* Softmax probabilities of one query row (token t of request i, head h) over
 * its full key set, normalised: probs[0..L_i+c_i).  For the sum-to-one and
 * brute-force pins.                                                           */
int oracle_attention_probs(const oracle_params_t *p, int32_t batch, const int32_t *cu_q,
                           const int32_t *prefix_len, const int32_t *block_start,
                           const int32_t *block_table, const uint16_t *q,
                           const uint16_t *k_new, const uint16_t *v_new,
                           const uint16_t *k_pool, const uint16_t *v_pool, int32_t i,
                           int32_t j, int32_t h, double *probs) {
  const int D = p->head_dim, Hq = p->num_q_heads, Hkv = p->num_kv_heads;
  if (i < 0 || i >= batch || Hq % Hkv != 0) return -1;
  const int G = Hq / Hkv, L = prefix_len[i], c = cu_q[i + 1] - cu_q[i];
  if (j < 0 || j >= c || h < 0 || h >= Hq) return -1;
  const double scale = p->scale > 0.0 ? p->scale : 1.0 / sqrt((double)D);
  const int n_keys = L + c;
  double *K = (double *)malloc(sizeof(double) * (size_t)n_keys * D);
  double *V = (double *)malloc(sizeof(double) * (size_t)n_keys * D);
  double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
  double *qrow = (double *)malloc(sizeof(double) * (size_t)D);
  double *o = (double *)malloc(sizeof(double) * (size_t)D);
  int rc = gather_keys(p, i, h / G, cu_q, prefix_len, block_table, k_new, v_new, k_pool,
                       v_pool, K, V);
  if (rc == 0) {
    int64_t t = cu_q[i] + j;
    for (int d = 0; d < D; ++d) qrow[d] = bf16_to_double(q[(t * Hq + h) * D + d]);
    double m, l;
    attend_row(p, qrow, K, V, L, L - block_start[i], j, 0, n_keys, scale, s, &m, &l, o,
               probs, NULL);
    for (int n = 0; n < n_keys; ++n) probs[n] /= l;
  }
  free(K); free(V); free(s); free(qrow); free(o);
  return rc;
}

/* Split-KV partial (the quantity the merge step consumes): one query row
 * restricted to keys [lo,hi): un-normalised o_part[D], its maximum m and its
 * sum l, natural-log domain.                                                  */
int oracle_partial_row(const oracle_params_t *p, int32_t batch, const int32_t *cu_q,
                       const int32_t *prefix_len, const int32_t *block_start,
                       const int32_t *block_table, const uint16_t *q,
                       const uint16_t *k_new, const uint16_t *v_new,
                       const uint16_t *k_pool, const uint16_t *v_pool, int32_t i,
                       int32_t j, int32_t h, int32_t lo, int32_t hi, double *o_part,
                       double *m_out, double *l_out) {
  const int D = p->head_dim, Hq = p->num_q_heads, Hkv = p->num_kv_heads;
  if (i < 0 || i >= batch || Hq % Hkv != 0) return -1;
  const int G = Hq / Hkv, L = prefix_len[i], c = cu_q[i + 1] - cu_q[i];
  const int n_keys = L + c;
  if (j < 0 || j >= c || h < 0 || h >= Hq || lo < 0 || hi > n_keys || lo > hi) return -1;
  const double scale = p->scale > 0.0 ? p->scale : 1.0 / sqrt((double)D);
  double *K = (double *)malloc(sizeof(double) * (size_t)n_keys * D);
  double *V = (double *)malloc(sizeof(double) * (size_t)n_keys * D);
  double *s = (double *)malloc(sizeof(double) * (size_t)(n_keys + 1));
  double *qrow = (double *)malloc(sizeof(double) * (size_t)D);
  int rc = gather_keys(p, i, h / G, cu_q, prefix_len, block_table, k_new, v_new, k_pool,
                       v_pool, K, V);
  if (rc == 0) {
    int64_t t = cu_q[i] + j;
    for (int d = 0; d < D; ++d) qrow[d] = bf16_to_double(q[(t * Hq + h) * D + d]);
    attend_row(p, qrow, K, V, L, L - block_start[i], j, lo, hi, scale, s, m_out, l_out,
               o_part, NULL, NULL);
  }
  free(K); free(V); free(s); free(qrow);
  return rc;
}

/* Step "merge": combine S partials of one row.  With M = max_s m_s,
 *   o = sum_s exp(m_s-M) o_part_s / sum_s exp(m_s-M) l_s.
 * A partial with m_s = -inf (no visible key in its range) contributes nothing. */
void oracle_merge_partials(int32_t S, int32_t D, const double *o_part /*[S,D]*/,
                           const double *m /*[S]*/, const double *l /*[S]*/,
                           double *o /*[D]*/) {
  double M = -INFINITY;
  for (int s = 0; s < S; ++s) if (m[s] > M) M = m[s];
  double z = 0.0;
  for (int d = 0; d < D; ++d) o[d] = 0.0;
  for (int s = 0; s < S; ++s) {
    if (m[s] == -INFINITY) continue;
    double w = exp(m[s] - M);
    z += w * l[s];
    for (int d = 0; d < D; ++d) o[d] += w * o_part[(int64_t)s * D + d];
  }
  for (int d = 0; d < D; ++d) o[d] /= z;
}
