// Replacement policy of the HBM expert cache: plain host C++ (no HIP), integers only.
//
// The paper keeps inactive experts in host DRAM and loads what the router selects (Sec. II-B);
// for a token that falls back to the big model the router outputs of its discarded little pass
// name the experts to prefetch (Sec. III-B).  It fixes no replacement policy; this is the one the
// library documents (mobile_moe.h, expert_cache_fetch).  Every decision depends on the sequence
// of calls alone, never on timing, so the unit can be replayed and checked without a GPU.
#pragma once

#include <stdint.h>

#include <vector>

namespace mm {

enum { kPolicyDemand = 0, kPolicyPrefetch = 1 };
enum { kPolicyOk = 0, kPolicyBadId = 1, kPolicyDuplicate = 2, kPolicyTooMany = 3, kPolicyBadMode = 4 };

struct PolicyCopy { int expert, slot; };          // load `expert` into `slot`
struct PolicyCounts { int hits, misses, dropped; };

class CachePolicy {
 public:
  CachePolicy(int n_experts, int n_slots);

  // One fetch call.  ids[n]: distinct experts (DEMAND: at most n_slots of them; PREFETCH: any
  // number, most wanted first).  slot_of[n]: slot of each id afterwards, -1 for a dropped
  // PREFETCH miss.  copies: the loads this call starts, in the order they are to be issued.
  // max_copies (PREFETCH): loads this call may start at most, negative = no bound.
  // A call that returns an error has changed nothing.
  int fetch(const int32_t* ids, int n, int mode, int max_copies, int32_t* slot_of,
            std::vector<PolicyCopy>* copies, PolicyCounts* counts);

  // The experts a step needs (ascending ids in `needed`), put in the order in which waves of at
  // most n_slots experts are fetched: those resident now first, then the others, ascending id
  // within each part.
  void wave_order(const std::vector<int32_t>& needed, std::vector<int32_t>* order) const;

  int n_experts() const { return E_; }
  int n_slots() const { return S_; }
  int expert_in_slot(int s) const { return slot_expert_[s]; }
  int slot_of_expert(int e) const { return expert_slot_[e]; }
  // the slot was named by the most recent DEMAND call
  bool in_last_demand(int s) const { return epoch_ > 0 && demand_epoch_[s] == epoch_; }

 private:
  int victim(const std::vector<char>& named, bool protect_last_demand) const;
  void place(int expert, int slot);

  int E_, S_;
  std::vector<int> slot_expert_, expert_slot_;
  std::vector<uint64_t> stamp_, demand_epoch_;
  uint64_t clock_ = 0, epoch_ = 0;
};

}  // namespace mm
