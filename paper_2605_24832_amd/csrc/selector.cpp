// Saturation-aware chunk-size selection (Optimus Sec. 5): a three-regime
// piecewise-affine latency model over x = batch * chunk (Sec. 5.2), fitted to
// profiled samples as ONE continuous curve by least squares with the two regime
// boundaries searched over the profiled loads, and the per-step choice
// c* = argmax_c N_commit(c) * b / T(c * b) (Sec. 5.1).  Host code only.
//
// Fit.  T(x) = alpha + beta x + gamma0 max(0, x - b0) + gamma1 max(0, x - b1).  For a pair
// of boundaries the normal equations of the four parameters need only sums of 1, x, x^2, t,
// x t over the samples above a boundary, so with suffix sums over the sorted samples every
// pair costs O(1); all pairs of interior distinct loads are tried.  Loads are scaled to
// [0, 1] and latencies centred, sums and the 4 x 4 solves are in long double, and the
// reported squared error is recomputed from the residuals of the chosen model.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <numeric>
#include <vector>

#include "optimus_attn.h"

namespace {

typedef long double ld;
constexpr int kMaxSamples = 2048;

// Finite test on the bit pattern: the library is built with NaN-free floating-point
// assumptions, under which an ordinary comparison against NaN may be folded away.
bool finite_bits(double v) {
  uint64_t u;
  std::memcpy(&u, &v, sizeof u);
  return ((u >> 52) & 0x7ff) != 0x7ff;
}

// Solves the symmetric 4 x 4 system m p = r by Gaussian elimination with partial pivoting.
// Returns false if a pivot vanishes (cannot happen for boundaries strictly between the
// smallest and the largest load).
bool solve4(ld m[4][4], ld r[4], ld p[4]) {
  int perm[4] = {0, 1, 2, 3};
  for (int c = 0; c < 4; ++c) {
    int piv = c;
    for (int k = c + 1; k < 4; ++k)
      if (std::fabs(m[perm[k]][c]) > std::fabs(m[perm[piv]][c])) piv = k;
    std::swap(perm[c], perm[piv]);
    const ld d = m[perm[c]][c];
    if (d == 0) return false;
    for (int k = c + 1; k < 4; ++k) {
      const ld f = m[perm[k]][c] / d;
      for (int j = c; j < 4; ++j) m[perm[k]][j] -= f * m[perm[c]][j];
      r[perm[k]] -= f * r[perm[c]];
    }
  }
  for (int c = 3; c >= 0; --c) {
    ld v = r[perm[c]];
    for (int j = c + 1; j < 4; ++j) v -= m[perm[c]][j] * p[j];
    p[c] = v / m[perm[c]][c];
  }
  return true;
}

struct Sums { ld n, x, xx, t, xt; };

}  // namespace

extern "C" int optimus_latency_fit(int32_t num_samples, const double* x, const double* latency,
                                   optimus_latency_model_t* model_out, double* sse_out) {
  if (!x || !latency || !model_out || num_samples < 6 || num_samples > kMaxSamples)
    return OPTIMUS_ERR_INVALID_ARGUMENT;
  const int n = num_samples;
  for (int i = 0; i < n; ++i)
    if (!finite_bits(x[i]) || !finite_bits(latency[i]) || x[i] < 0) return OPTIMUS_ERR_INVALID_ARGUMENT;
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return x[a] < x[b]; });
  const double x_max = x[order[n - 1]];
  if (!(x_max > 0)) return OPTIMUS_ERR_INVALID_ARGUMENT;
  ld t_mean = 0;
  for (int i = 0; i < n; ++i) t_mean += latency[i];
  t_mean /= n;
  std::vector<ld> u(n), tc(n);
  for (int i = 0; i < n; ++i) { u[i] = (ld)x[order[i]] / x_max; tc[i] = latency[order[i]] - t_mean; }

  // suf[i]: sums over the sorted samples i .. n-1
  std::vector<Sums> suf(n + 1, Sums{0, 0, 0, 0, 0});
  ld tt = 0;
  for (int i = n - 1; i >= 0; --i) {
    suf[i] = Sums{suf[i + 1].n + 1, suf[i + 1].x + u[i], suf[i + 1].xx + u[i] * u[i], suf[i + 1].t + tc[i],
                  suf[i + 1].xt + u[i] * tc[i]};
    tt += tc[i] * tc[i];
  }
  // distinct loads: first[g] = index of the first sample of the g-th distinct load
  std::vector<int> first;
  for (int i = 0; i < n; ++i)
    if (i == 0 || x[order[i]] != x[order[i - 1]]) first.push_back(i);
  const int d = (int)first.size();
  if (d < 4) return OPTIMUS_ERR_INVALID_ARGUMENT;   // no room for two boundaries between the extreme loads
  first.push_back(n);

  const Sums& all = suf[0];
  ld best = std::numeric_limits<ld>::infinity();
  int best0 = -1, best1 = -1;
  ld best_p[4] = {0, 0, 0, 0};
  for (int g0 = 1; g0 + 1 < d - 1; ++g0) {
    const ld b0 = u[first[g0]];
    const Sums& a0 = suf[first[g0 + 1]];            // samples above b0
    // hinge h0 = max(0, u - b0): sums of h0, h0 u, h0^2, h0 t
    const ld h0 = a0.x - b0 * a0.n, h0x = a0.xx - b0 * a0.x, h0h0 = a0.xx - 2 * b0 * a0.x + b0 * b0 * a0.n;
    const ld h0t = a0.xt - b0 * a0.t;
    for (int g1 = g0 + 1; g1 < d - 1; ++g1) {
      const ld b1 = u[first[g1]];
      const Sums& a1 = suf[first[g1 + 1]];          // samples above b1
      const ld h1 = a1.x - b1 * a1.n, h1x = a1.xx - b1 * a1.x, h1h1 = a1.xx - 2 * b1 * a1.x + b1 * b1 * a1.n;
      const ld h1t = a1.xt - b1 * a1.t;
      const ld h0h1 = a1.xx - (b0 + b1) * a1.x + b0 * b1 * a1.n;
      ld m[4][4] = {{all.n, all.x, h0, h1}, {all.x, all.xx, h0x, h1x}, {h0, h0x, h0h0, h0h1}, {h1, h1x, h0h1, h1h1}};
      ld r[4] = {all.t, all.xt, h0t, h1t};
      const ld r0[4] = {all.t, all.xt, h0t, h1t};
      ld p[4];
      if (!solve4(m, r, p)) continue;
      const ld sse = tt - (p[0] * r0[0] + p[1] * r0[1] + p[2] * r0[2] + p[3] * r0[3]);
      if (sse < best) {
        best = sse; best0 = g0; best1 = g1;
        for (int k = 0; k < 4; ++k) best_p[k] = p[k];
      }
    }
  }
  if (best0 < 0) return OPTIMUS_ERR_INVALID_ARGUMENT;
  const ld b0 = u[first[best0]], b1 = u[first[best1]];
  const ld alpha = best_p[0] + t_mean, beta = best_p[1], g0 = best_p[2], g1 = best_p[3];
  model_out->x_break[0] = x[order[first[best0]]];
  model_out->x_break[1] = x[order[first[best1]]];
  model_out->beta1[0] = (double)(beta / x_max);
  model_out->beta1[1] = (double)((beta + g0) / x_max);
  model_out->beta1[2] = (double)((beta + g0 + g1) / x_max);
  model_out->beta0[0] = (double)alpha;
  model_out->beta0[1] = (double)(alpha - g0 * b0);
  model_out->beta0[2] = (double)(alpha - g0 * b0 - g1 * b1);
  if (sse_out) {
    ld sse = 0;
    for (int i = 0; i < n; ++i) {
      const ld ui = u[i];
      const ld fit = best_p[0] + beta * ui + g0 * std::max<ld>(0, ui - b0) + g1 * std::max<ld>(0, ui - b1);
      sse += (tc[i] - fit) * (tc[i] - fit);
    }
    *sse_out = (double)sse;
  }
  return OPTIMUS_OK;
}

extern "C" double optimus_latency_eval(const optimus_latency_model_t* model, double x) {
  if (!model) return std::numeric_limits<double>::quiet_NaN();
  const int k = x < model->x_break[0] ? 0 : (x < model->x_break[1] ? 1 : 2);
  return model->beta1[k] * x + model->beta0[k];
}

extern "C" int optimus_select_chunk(const optimus_latency_model_t* model, int32_t batch,
                                    int32_t num_candidates, const int32_t* chunk_sizes,
                                    const double* n_commit, int32_t* best_index_out,
                                    double* rate_out) {
  if (!model || !chunk_sizes || !n_commit || !best_index_out || batch < 1 || num_candidates < 1)
    return OPTIMUS_ERR_INVALID_ARGUMENT;
  int best = -1;
  double best_rate = -1;
  for (int i = 0; i < num_candidates; ++i) {
    if (chunk_sizes[i] < 1 || !finite_bits(n_commit[i]) || n_commit[i] < 0) return OPTIMUS_ERR_INVALID_ARGUMENT;
    const double t = optimus_latency_eval(model, (double)batch * chunk_sizes[i]);
    if (!finite_bits(t) || t <= 0) return OPTIMUS_ERR_INVALID_ARGUMENT;  // a latency model must stay positive
    const double rate = n_commit[i] * batch / t;
    if (rate_out) rate_out[i] = rate;
    if (rate > best_rate) { best_rate = rate; best = i; }
  }
  *best_index_out = best;
  return OPTIMUS_OK;
}
