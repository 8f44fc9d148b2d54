// Replays a trace of fetch calls through the library's cache policy unit (cache_policy.cpp, no HIP)
// and prints every decision.  Built by tests/test_cache_policy_host.py with the host compiler and
// -fsanitize=address,undefined.
//
// stdin:   E n_slots
//          mode n max_copies id_0 ... id_{n-1}          (one line per call; mode 0 DEMAND, 1 PREFETCH)
//          w n id_0 ... id_{n-1}                        (wave order of the named experts)
// stdout:  per call:  rc | slot_of ... | hits misses dropped | expert:slot copies ... | occupancy ...
//          per w:     order ...
#include <stdio.h>
#include <stdlib.h>

#include <string>
#include <vector>

#include "cache_policy.h"

int main() {
  int E, S;
  if (scanf("%d %d", &E, &S) != 2) return 2;
  mm::CachePolicy pol(E, S);
  char tag[8];
  while (scanf("%7s", tag) == 1) {
    if (tag[0] == 'w') {
      int n;
      if (scanf("%d", &n) != 1) return 2;
      std::vector<int32_t> ids(n), order;
      for (int i = 0; i < n; ++i) if (scanf("%d", &ids[i]) != 1) return 2;
      pol.wave_order(ids, &order);
      printf("order");
      for (int32_t e : order) printf(" %d", e);
      printf("\n");
      continue;
    }
    const int mode = atoi(tag);
    int n, lim;
    if (scanf("%d %d", &n, &lim) != 2) return 2;
    std::vector<int32_t> ids(n > 0 ? n : 1), slots(n > 0 ? n : 1, -7);
    for (int i = 0; i < n; ++i) if (scanf("%d", &ids[i]) != 1) return 2;
    std::vector<mm::PolicyCopy> copies;
    mm::PolicyCounts c = {0, 0, 0};
    const int rc = pol.fetch(ids.data(), n, mode, lim, slots.data(), &copies, &c);
    printf("%d |", rc);
    if (rc == 0) for (int i = 0; i < n; ++i) printf(" %d", slots[i]);
    printf(" | %d %d %d |", c.hits, c.misses, c.dropped);
    for (const auto& cp : copies) printf(" %d:%d", cp.expert, cp.slot);
    printf(" |");
    for (int s = 0; s < S; ++s) printf(" %d", pol.expert_in_slot(s));
    printf("\n");
  }
  return 0;
}
