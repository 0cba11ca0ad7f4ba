// Saturation-aware chunk-size selection (Optimus Sec. 5): a three-regime
// piecewise-affine latency model over x = batch * chunk (Sec. 5.2), fitted to
// profiled samples by least squares with the two regime boundaries chosen to
// minimise the total squared error, and the per-step choice
// c* = argmax_c N_commit(c) * b / T(c * b) (Sec. 5.1).  Host code only.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <numeric>
#include <vector>

#include "optimus_attn.h"

namespace {

// Running least-squares sums of one segment, updated one sample at a time
// (Welford's recurrences: no cancellation between large sums).
struct Segment {
  double n = 0, mx = 0, mt = 0, sxx = 0, sxt = 0, stt = 0;
  void add(double x, double t) {
    n += 1;
    const double dx = x - mx, dt = t - mt;
    mx += dx / n;
    mt += dt / n;
    sxx += dx * (x - mx);
    sxt += dx * (t - mt);
    stt += dt * (t - mt);
  }
  bool has_slope() const { return sxx > 0; }
  double slope() const { return sxt / sxx; }
  double intercept() const { return mt - slope() * mx; }
  double sse() const { return std::max(0.0, stt - sxt * sxt / sxx); }
};

constexpr int kMaxSamples = 2048;

// Finite test on the bit pattern: the library is built with NaN-free floating-point
// assumptions, under which an ordinary comparison against NaN may be folded away.
bool finite_bits(double v) {
  uint64_t u;
  std::memcpy(&u, &v, sizeof u);
  return ((u >> 52) & 0x7ff) != 0x7ff;
}

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
  std::vector<double> xs(n), ts(n);
  for (int i = 0; i < n; ++i) { xs[i] = x[order[i]]; ts[i] = latency[order[i]]; }

  // cost[i * (n + 1) + j] = squared error of the best line through samples [i, j); inf where the
  // segment has fewer than two distinct x
  const double inf = std::numeric_limits<double>::infinity();
  std::vector<double> cost((size_t)(n + 1) * (n + 1), inf);
  for (int i = 0; i < n; ++i) {
    Segment s;
    for (int j = i; j < n; ++j) {
      s.add(xs[j], ts[j]);
      if (s.has_slope()) cost[(size_t)i * (n + 1) + j + 1] = s.sse();
    }
  }
  // a boundary may only fall between two different x: equal loads belong to one regime
  double best = inf;
  int best_a = -1, best_b = -1;
  for (int a = 1; a < n; ++a) {
    if (xs[a] == xs[a - 1]) continue;
    const double c0 = cost[a];
    if (c0 == inf) continue;
    for (int b = a + 1; b < n; ++b) {
      if (xs[b] == xs[b - 1]) continue;
      const double total = c0 + cost[(size_t)a * (n + 1) + b] + cost[(size_t)b * (n + 1) + n];
      if (total < best) { best = total; best_a = a; best_b = b; }
    }
  }
  if (best_a < 0) return OPTIMUS_ERR_INVALID_ARGUMENT;  // fewer than six usable distinct loads
  const int lo[3] = {0, best_a, best_b}, hi[3] = {best_a, best_b, n};
  for (int k = 0; k < 3; ++k) {
    Segment s;
    for (int j = lo[k]; j < hi[k]; ++j) s.add(xs[j], ts[j]);
    model_out->beta1[k] = s.slope();
    model_out->beta0[k] = s.intercept();
  }
  model_out->x_break[0] = 0.5 * (xs[best_a - 1] + xs[best_a]);
  model_out->x_break[1] = 0.5 * (xs[best_b - 1] + xs[best_b]);
  if (sse_out) *sse_out = best;
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
