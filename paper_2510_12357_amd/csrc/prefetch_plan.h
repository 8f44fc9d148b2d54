// What to prefetch and when (Sec. III-B): plain host C++ (no HIP).
//
// When a token's little pass is rejected, the router outputs of that pass are known for every
// layer; the big pass that follows will most likely select the same experts, so they are
// requested ahead of the layer that needs them.  How far ahead is adjustable (Sec. III-B: one
// layer on a fast link, two or three on a slow one).  This unit turns router logits into the
// per-layer request lists and says which layers' requests are due at which point of a pass.
#pragma once

#include <stdint.h>

#include <vector>

namespace mm {

// The k experts a row of router logits selects, in the layer's own order: logit descending,
// expert id ascending among equals, NaN counted as -infinity.  out[k].
void plan_select(const float* logits, int E, int k, int32_t* out);

class PrefetchPlan {
 public:
  PrefetchPlan(int n_layers, int n_experts, int k);

  // logits: [n_layers][T][n_experts] router logits of one pass; rejected[n]: the tokens whose
  // little result was dropped (each in [0, T)).  Replaces the previous prediction.  The list of
  // a layer holds the rejected tokens' selections rank by rank (every token's most likely expert
  // first), each expert once.  n == 0 clears the prediction.  Returns false on a token index
  // outside [0, T).
  bool predict(const float* logits, int T, const int32_t* rejected, int n);
  void clear();

  const std::vector<int32_t>& layer(int l) const { return lists_[l]; }

  // Layers whose requests are issued now, at distance d: layer == -1 is the start of a pass
  // (layers 0 .. d-1), layer == l >= 0 is "layer l is about to run" (layer l + d).  d == 0:
  // nothing is prefetched.  Returns how many were written to out (capacity n_layers).
  int due(int layer, int d, int32_t* out) const;

  int n_layers() const { return L_; }
  int n_experts() const { return E_; }
  int k() const { return k_; }

 private:
  int L_, E_, k_;
  std::vector<std::vector<int32_t>> lists_;
};

}  // namespace mm
