// Replacement policy of the HBM expert cache (see cache_policy.h): least recently named slot
// first, DEMAND before PREFETCH, nothing queued.
#include "cache_policy.h"

namespace mm {

CachePolicy::CachePolicy(int n_experts, int n_slots)
    : E_(n_experts), S_(n_slots), slot_expert_(n_slots, -1), expert_slot_(n_experts, -1),
      stamp_(n_slots, 0), demand_epoch_(n_slots, 0) {}

// least recently stamped slot that holds no expert named by the call (and, for PREFETCH, none of
// the most recent DEMAND call); lowest slot id among equals; empty slots carry stamp 0
int CachePolicy::victim(const std::vector<char>& named, bool protect_last_demand) const {
  int best = -1;
  for (int s = 0; s < S_; ++s) {
    const int e = slot_expert_[s];
    if (e >= 0 && named[e]) continue;
    if (protect_last_demand && in_last_demand(s)) continue;
    if (best < 0 || stamp_[s] < stamp_[best]) best = s;
  }
  return best;
}

void CachePolicy::place(int expert, int slot) {
  const int old = slot_expert_[slot];
  if (old >= 0) expert_slot_[old] = -1;
  slot_expert_[slot] = expert;
  expert_slot_[expert] = slot;
}

int CachePolicy::fetch(const int32_t* ids, int n, int mode, int max_copies, int32_t* slot_of,
                       std::vector<PolicyCopy>* copies, PolicyCounts* counts) {
  if (mode != kPolicyDemand && mode != kPolicyPrefetch) return kPolicyBadMode;
  std::vector<char> named(E_, 0);
  for (int i = 0; i < n; ++i) {
    if (ids[i] < 0 || ids[i] >= E_) return kPolicyBadId;
    if (named[ids[i]]) return kPolicyDuplicate;
    named[ids[i]] = 1;
  }
  if (mode == kPolicyDemand && n > S_) return kPolicyTooMany;

  PolicyCounts c = {0, 0, 0};
  if (copies) copies->clear();
  ++clock_;
  if (mode == kPolicyDemand) {
    ++epoch_;
    for (int e = 0; e < E_; ++e) {                 // residents: hits
      if (!named[e] || expert_slot_[e] < 0) continue;
      const int s = expert_slot_[e];
      stamp_[s] = clock_; demand_epoch_[s] = epoch_;
      ++c.hits;
    }
    for (int e = 0; e < E_; ++e) {                 // misses, ascending expert id
      if (!named[e] || expert_slot_[e] >= 0) continue;
      const int v = victim(named, false);          // exists: n <= n_slots and the ids are distinct
      place(e, v);
      stamp_[v] = clock_; demand_epoch_[v] = epoch_;
      if (copies) copies->push_back({e, v});
      ++c.misses;
    }
    for (int i = 0; i < n; ++i) slot_of[i] = expert_slot_[ids[i]];
  } else {
    for (int i = 0; i < n; ++i) {                  // the caller's priority order
      const int e = ids[i];
      if (expert_slot_[e] >= 0) {
        stamp_[expert_slot_[e]] = clock_;
        slot_of[i] = expert_slot_[e];
        ++c.hits;
        continue;
      }
      const int v = victim(named, true);
      if (v < 0 || (max_copies >= 0 && c.misses >= max_copies)) {
        slot_of[i] = -1;
        ++c.dropped;
        continue;
      }
      place(e, v);
      stamp_[v] = clock_;
      if (copies) copies->push_back({e, v});
      slot_of[i] = v;
      ++c.misses;
    }
  }
  if (counts) *counts = c;
  return kPolicyOk;
}

void CachePolicy::wave_order(const std::vector<int32_t>& needed, std::vector<int32_t>* order) const {
  order->clear();
  for (int pass = 0; pass < 2; ++pass)
    for (int32_t e : needed) {
      if (e < 0 || e >= E_) continue;
      const bool resident = expert_slot_[e] >= 0;
      if ((pass == 0) == resident) order->push_back(e);
    }
}

}  // namespace mm
