// Offline layer-range profiler (Section 4.2, Eq. 2-4; Appendix table "Hyperparameters for Critical Layer
// Selection"): host-side post-processing of the per-layer deviation scores that rc_vdev_score produces.
// Plain C++ on host memory; nothing here touches the GPU.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "common.h"

namespace rc {
namespace {

// ranks 1..n, equal values share the mean of the ranks they occupy
void average_ranks(const float* x, int n, std::vector<int>& order, std::vector<double>& ranks) {
  order.resize(n);
  ranks.resize(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [x](int a, int b) { return x[a] < x[b]; });
  for (int i = 0; i < n;) {
    int j = i;
    while (j + 1 < n && x[order[j + 1]] == x[order[i]]) ++j;
    const double r = 0.5 * (i + j) + 1.0;
    for (int t = i; t <= j; ++t) ranks[order[t]] = r;
    i = j + 1;
  }
}

double pearson(const std::vector<double>& a, const std::vector<double>& b) {
  const int n = (int)a.size();
  double ma = 0.0, mb = 0.0;
  for (int i = 0; i < n; ++i) { ma += a[i]; mb += b[i]; }
  ma /= n; mb /= n;
  double sab = 0.0, saa = 0.0, sbb = 0.0;
  for (int i = 0; i < n; ++i) {
    const double u = a[i] - ma, v = b[i] - mb;
    sab += u * v; saa += u * u; sbb += v * v;
  }
  const double den = std::sqrt(saa * sbb);
  return den > 0.0 ? sab / den : 0.0;
}

}  // namespace
}  // namespace rc

extern "C" rc_status rc_layer_profile(const float* d, int32_t n_layers, int32_t n_tokens,
                                      const rc_layer_profile_params* params, rc_layer_triple* out, double* s_out,
                                      double* rho_out) {
  using namespace rc;
  if (!d || !params || !out || n_layers < 2 || n_tokens < 1) return RC_E_INVALID_ARG;
  if (n_layers > RC_MAX_LAYERS) return RC_E_CAPACITY;
  if (params->tail < 1 || params->consecutive < 1 || !(params->lambda >= 0.f)) return RC_E_INVALID_ARG;
  const int L = n_layers, n = n_tokens;
  // Eq. (2)
  std::vector<double> s(L);
  for (int l = 0; l < L; ++l) {
    double acc = 0.0;
    for (int j = 0; j < n; ++j) acc += 1.0 - (double)d[(size_t)l * n + j];
    s[l] = acc / n;
  }
  int l_min = 0;
  for (int l = 1; l < L; ++l)
    if (s[l] < s[l_min]) l_min = l;
  // start layer: deepest layer up to the minimum whose similarity is still above the threshold
  int l_start = 0;
  for (int l = 0; l <= l_min; ++l)
    if (s[l] >= (double)params->tau_st) l_start = l;
  // end layer: onset of the stable tail regime
  const int t0 = std::max(0, L - params->tail);
  double mu = 0.0;
  for (int l = t0; l < L; ++l) mu += s[l];
  mu /= (L - t0);
  double var = 0.0;
  for (int l = t0; l < L; ++l) var += (s[l] - mu) * (s[l] - mu);
  const double sigma = std::sqrt(var / (L - t0));
  const double b = mu - sigma, step = (double)params->lambda * sigma;
  int l_end = L - 1;
  for (int l = l_min; l + params->consecutive < L; ++l) {
    bool ok = true;
    for (int l2 = l + 1; l2 <= l + params->consecutive && ok; ++l2)
      ok = s[l2] >= b && std::fabs(s[l2] - s[l2 - 1]) < step;
    if (ok) { l_end = l; break; }
  }
  l_end = std::max(l_end, std::min(l_start + 1, L - 1));
  // detection layer: first positive-to-negative change of the second difference of the rank correlation
  std::vector<double> rho(L, 0.0), alpha(L, 0.0), prev, cur;
  std::vector<int> order;
  average_ranks(d, n, order, prev);
  for (int l = 1; l < L; ++l) {
    average_ranks(d + (size_t)l * n, n, order, cur);
    rho[l] = pearson(prev, cur);
    prev.swap(cur);
  }
  for (int l = 3; l < L; ++l) alpha[l] = rho[l] - 2.0 * rho[l - 1] + rho[l - 2];
  int l_det = std::min(l_start + 1, l_end);
  for (int l = 4; l < L; ++l) {
    if (alpha[l - 1] > 0.0 && alpha[l] < 0.0 && l_start < l + 1 && l + 1 <= l_end) { l_det = l + 1; break; }
  }
  out->l_start = l_start;
  out->l_det = l_det;
  out->l_end = l_end;
  if (s_out) std::copy(s.begin(), s.end(), s_out);
  if (rho_out) std::copy(rho.begin(), rho.end(), rho_out);
  return RC_OK;
}
