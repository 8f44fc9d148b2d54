// Runs the library's prefetch plan unit (prefetch_plan.cpp, no HIP) on inputs from stdin and prints
// what it decides.  Built by tests/test_prefetch_plan_host.py with the host compiler and
// -fsanitize=address,undefined.
//
// stdin:   L E k T n
//          rejected_0 ... rejected_{n-1}
//          L*T*E logits as hexadecimal bit patterns of fp32 (so that NaN and -0 survive)
//          then any number of lines "layer d"
// stdout:  "ok" or "bad" (the return of predict), then per layer: its request list,
//          then per "layer d" line: the layers due
#include <stdio.h>
#include <string.h>

#include <vector>

#include "prefetch_plan.h"

int main() {
  int L, E, k, T, n;
  if (scanf("%d %d %d %d %d", &L, &E, &k, &T, &n) != 5) return 2;
  std::vector<int32_t> rej(n > 0 ? n : 1);
  for (int i = 0; i < n; ++i) if (scanf("%d", &rej[i]) != 1) return 2;
  std::vector<float> logits((size_t)L * T * E);
  for (float& v : logits) {
    unsigned bits;
    if (scanf("%x", &bits) != 1) return 2;
    memcpy(&v, &bits, 4);
  }
  mm::PrefetchPlan plan(L, E, k);
  const bool ok = plan.predict(logits.data(), T, rej.data(), n);
  printf(ok ? "ok\n" : "bad\n");
  for (int l = 0; l < L; ++l) {
    printf("list");
    for (int32_t e : plan.layer(l)) printf(" %d", e);
    printf("\n");
  }
  int layer, d;
  std::vector<int32_t> due(L);
  while (scanf("%d %d", &layer, &d) == 2) {
    const int m = plan.due(layer, d, due.data());
    printf("due");
    for (int i = 0; i < m; ++i) printf(" %d", due[i]);
    printf("\n");
  }
  return 0;
}
