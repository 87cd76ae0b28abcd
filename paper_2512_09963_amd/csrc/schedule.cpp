// Estimator updates and the per-round scheduling problem of GoodSpeed
// (paper Section III-C: the exponential smoothing of alpha-hat and of X, then
// GoodSpeed-sched with log utility).  Host code.
//
// The objective sum_i (1/X_i) * (1 + a_i + ... + a_i^{S_i}) is separable and each term is
// concave in S_i (the S-th extra slot of server i adds (1/X_i) a_i^S, a decreasing sequence),
// so handing out the capacity one slot at a time to the largest next gain is exact.  A
// max-heap keyed by (gain, lowest index first) makes that O((N + C) log N).
#include <algorithm>
#include <cmath>
#include <queue>
#include <vector>
#include "common.h"

namespace gs {

char* error_buffer() {
  static thread_local char buf[512] = "";
  return buf;
}

}  // namespace gs

extern "C" const char* gs_last_error(void) { return gs::error_buffer(); }

namespace {

struct Slot {
  double gain;   // value of the next slot of this server
  int server;
};
struct SlotLess {
  bool operator()(const Slot& a, const Slot& b) const {
    if (a.gain != b.gain) return a.gain < b.gain;
    return a.server > b.server;   // equal gains: the lower index is served first
  }
};

}  // namespace

extern "C" gs_status gs_schedule_gamma(int n, const int* accepted_len, const float* accept_stat,
                                       const int* gamma_prev, double* alpha_hat, double* x_smooth, double eta,
                                       double beta, int capacity, int gamma_min, int gamma_max, int* gamma_next) {
  if (n <= 0) return gs::fail(GS_EINVAL, "n must be positive");
  if (!accepted_len || !accept_stat || !gamma_prev || !alpha_hat || !x_smooth || !gamma_next)
    return gs::fail(GS_EINVAL, "null argument");
  if (!(eta >= 0.0 && eta <= 1.0) || !(beta >= 0.0 && beta <= 1.0))
    return gs::fail(GS_EINVAL, "eta and beta must lie in [0, 1]");
  if (gamma_min < 0) return gs::fail(GS_EINVAL, "gamma_min must be non-negative");
  if (gamma_max >= 0 && gamma_max < gamma_min) return gs::fail(GS_EINVAL, "gamma_max below gamma_min");
  if ((long)capacity < (long)n * gamma_min)
    return gs::fail(GS_EINVAL, "capacity %d cannot give every server gamma_min = %d", capacity, gamma_min);
  for (int i = 0; i < n; ++i) {
    if (accepted_len[i] < 0 || gamma_prev[i] < 0 || accepted_len[i] > gamma_prev[i])
      return gs::fail(GS_EINVAL, "accepted_len[%d] = %d outside [0, gamma_prev = %d]", i, accepted_len[i],
                      gamma_prev[i]);
    const double x_new = (1.0 - beta) * x_smooth[i] + beta * ((double)accepted_len[i] + 1.0);
    if (!(x_new > 0.0) || !std::isfinite(x_new))
      return gs::fail(GS_EINVAL, "smoothed goodput of server %d is not positive", i);
  }

  // estimator updates first: the solve uses alpha_hat(t) and X(t)
  for (int i = 0; i < n; ++i) {
    if (gamma_prev[i] > 0) alpha_hat[i] = (1.0 - eta) * alpha_hat[i] + eta * (double)accept_stat[i];
    x_smooth[i] = (1.0 - beta) * x_smooth[i] + beta * ((double)accepted_len[i] + 1.0);
  }

  std::vector<double> a(n);
  std::priority_queue<Slot, std::vector<Slot>, SlotLess> heap;
  long left = capacity;
  for (int i = 0; i < n; ++i) {
    a[i] = std::min(std::max(alpha_hat[i], 1e-6), 1.0 - 1e-6);
    gamma_next[i] = gamma_min;
    left -= gamma_min;
    if (gamma_max < 0 || gamma_min < gamma_max) {
      heap.push({(1.0 / x_smooth[i]) * std::pow(a[i], (double)(gamma_min + 1)), i});
    }
  }
  while (left > 0 && !heap.empty()) {
    Slot s = heap.top();
    heap.pop();
    gamma_next[s.server] += 1;
    --left;
    // next gain formed from scratch as (1/X) a^(S + 1): the same expression for every S, so that two servers
    // with equal (alpha_hat, X) always tie exactly (a running product would depend on the path)
    if (gamma_max < 0 || gamma_next[s.server] < gamma_max)
      heap.push({(1.0 / x_smooth[s.server]) * std::pow(a[s.server], (double)(gamma_next[s.server] + 1)), s.server});
  }
  return GS_OK;
}

// Baseline allocation policies of the paper's comparison (Section IV-A): Fixed-S and Random-S.
extern "C" gs_status gs_allocate_fixed(int n, int capacity, int* gamma_next) {
  if (n <= 0 || capacity < 0 || !gamma_next) return gs::fail(GS_EINVAL, "n must be positive, capacity non-negative");
  for (int i = 0; i < n; ++i) gamma_next[i] = capacity / n + (i < capacity % n ? 1 : 0);
  return GS_OK;
}

extern "C" gs_status gs_allocate_random(int n, int capacity, const float* uniforms, int* gamma_next) {
  if (n <= 0 || capacity < 0 || !gamma_next || (capacity > 0 && !uniforms))
    return gs::fail(GS_EINVAL, "n must be positive, capacity non-negative, uniforms given");
  for (int k = 0; k < capacity; ++k)
    if (!(uniforms[k] >= 0.f && uniforms[k] < 1.f)) return gs::fail(GS_EINVAL, "uniforms[%d] is outside [0, 1)", k);
  for (int i = 0; i < n; ++i) gamma_next[i] = 0;
  for (int k = 0; k < capacity; ++k) {
    int i = (int)((double)uniforms[k] * (double)n);
    gamma_next[i < n ? i : n - 1] += 1;
  }
  return GS_OK;
}
