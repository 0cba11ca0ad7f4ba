/*
 * CPU oracle of the commit step of block-diffusion decoding (Optimus Sec. 2.3
 * and Sec. 4.1: in every iteration the model assigns each chunk position a
 * confidence, and positions whose confidence exceeds a threshold are
 * committed; Sec. 7.1 uses the threshold 0.9).
 *
 * TEST INFRASTRUCTURE ONLY: plain definition in fp64, shares nothing with the
 * HIP path.
 *
 * Reading (the paper gives no formula): the confidence of a position is the
 * largest softmax probability of its logit row, its token the first index that
 * attains it.  A position is committed iff confidence > threshold.  Optional
 * progress rule: a request that has chunk tokens but none above the threshold
 * commits its single most confident one (first on ties) when min_commit = 1.
 * A logit that is -inf or NaN stands for a vocabulary entry that cannot be
 * chosen (a masked entry): it can never be the token and adds nothing to the
 * softmax sum.  A row without any other entry has confidence 0 and token 0.
 * +inf logits are outside the definition.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static double bf16_to_double_c(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* value of a logit; masked entries (NaN, -inf) read as -inf */
static double logit_value(uint16_t b) {
  const double x = bf16_to_double_c(b);
  return isnan(x) ? -INFINITY : x;
}

/* logits: bf16 [T, row_stride], first `vocab` entries of a row are used.
 * cu_q: [batch+1] or NULL (then no per-request rule).                        */
int oracle_commit(int32_t num_tokens, int32_t vocab, int64_t row_stride, const uint16_t *logits,
                  double threshold, int32_t batch, const int32_t *cu_q, int32_t min_commit,
                  int32_t *token_out, double *conf_out, int32_t *commit_out) {
  if (num_tokens < 0 || vocab < 1 || row_stride < vocab) return -1;
#pragma omp parallel for schedule(static)
  for (int t = 0; t < num_tokens; ++t) {
    const uint16_t *row = logits + (int64_t)t * row_stride;
    double mx = -INFINITY;
    int arg = 0;
    for (int v = 0; v < vocab; ++v) {
      double x = logit_value(row[v]);
      if (x > mx) { mx = x; arg = v; }
    }
    if (mx == -INFINITY) {          /* every entry masked */
      token_out[t] = 0;
      conf_out[t] = 0.0;
      commit_out[t] = 0;
      continue;
    }
    double z = 0.0;
    for (int v = 0; v < vocab; ++v) {
      const double x = logit_value(row[v]);
      if (x != -INFINITY) z += exp(x - mx);
    }
    token_out[t] = arg;
    conf_out[t] = 1.0 / z;          /* exp(mx - mx) / z */
    commit_out[t] = conf_out[t] > threshold ? 1 : 0;
  }
  if (cu_q && min_commit >= 1) {
    for (int i = 0; i < batch; ++i) {
      int any = 0, best = -1;
      for (int t = cu_q[i]; t < cu_q[i + 1]; ++t) {
        any |= commit_out[t];
        if (best < 0 || conf_out[t] > conf_out[best]) best = t;
      }
      if (!any && best >= 0) commit_out[best] = 1;
    }
  }
  return 0;
}
