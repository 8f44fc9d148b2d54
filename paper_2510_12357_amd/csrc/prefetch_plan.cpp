// Prefetch plan (Sec. III-B): request lists from router logits, and the layers due at a point of
// a pass.  Host only; see prefetch_plan.h.
#include "prefetch_plan.h"

#include <cmath>
#include <limits>

namespace mm {

void plan_select(const float* logits, int E, int k, int32_t* out) {
  std::vector<char> taken((size_t)E, 0);
  for (int j = 0; j < k; ++j) {
    int best = -1;
    float bv = 0.f;
    for (int e = 0; e < E; ++e) {
      if (taken[e]) continue;
      const float v = std::isnan(logits[e]) ? -std::numeric_limits<float>::infinity() : logits[e];
      if (best < 0 || v > bv) { best = e; bv = v; }      // strict: the lowest id among equals stays
    }
    out[j] = best;
    if (best >= 0) taken[best] = 1;
  }
}

PrefetchPlan::PrefetchPlan(int n_layers, int n_experts, int k)
    : L_(n_layers), E_(n_experts), k_(k), lists_((size_t)n_layers) {}

void PrefetchPlan::clear() {
  for (auto& l : lists_) l.clear();
}

bool PrefetchPlan::predict(const float* logits, int T, const int32_t* rejected, int n) {
  for (int i = 0; i < n; ++i)
    if (rejected[i] < 0 || rejected[i] >= T) return false;
  clear();
  if (n == 0) return true;
  std::vector<int32_t> sel((size_t)n * k_);
  std::vector<char> seen((size_t)E_);
  for (int l = 0; l < L_; ++l) {
    const float* base = logits + (size_t)l * T * E_;
    for (int i = 0; i < n; ++i) plan_select(base + (size_t)rejected[i] * E_, E_, k_, sel.data() + (size_t)i * k_);
    seen.assign((size_t)E_, 0);
    for (int j = 0; j < k_; ++j)
      for (int i = 0; i < n; ++i) {
        const int e = sel[(size_t)i * k_ + j];
        if (e >= 0 && !seen[e]) { seen[e] = 1; lists_[l].push_back(e); }
      }
  }
  return true;
}

int PrefetchPlan::due(int layer, int d, int32_t* out) const {
  if (d <= 0) return 0;
  int n = 0;
  if (layer < 0) {
    for (int l = 0; l < d && l < L_; ++l) out[n++] = l;
  } else if (layer + d < L_) {
    out[n++] = layer + d;
  }
  return n;
}

}  // namespace mm
