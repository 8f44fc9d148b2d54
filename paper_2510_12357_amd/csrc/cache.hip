// HBM expert cache: on-demand fetch and prefetch of expert blobs from pinned host DRAM
// (Sec. II-B: experts are loaded over the host link when the router selects them; Sec. III-B:
// the router outputs of a token's discarded little pass name the experts of its big pass ahead
// of time, so their copies can overlap with compute).
//
// Which expert goes to which slot is decided by the host-only policy unit (cache_policy.h); this
// file moves the bytes and orders them against the compute stream.  Data movement is
// hipMemcpyAsync on two side streams of default priority, one for DEMAND copies and one for
// PREFETCH copies, so that a copy the step is waiting for never queues behind copies that were
// only started on a prediction.  Per slot:
//   ready[s]     recorded behind the latest copy into slot s (on the stream that carried it); the
//                compute stream waits for it before kernels read the slot, and a later copy into
//                the slot waits for it as well (the two copy streams are not ordered otherwise)
//   released[s]  recorded on the compute stream at the start of the first DEMAND call after the
//                slot was handed out by a DEMAND call, i.e. after every kernel that may read the
//                slot has been enqueued; a later copy into the slot waits for it.  PREFETCH calls
//                record nothing: the only slots still waiting for their release then belong to
//                the most recent DEMAND call, which a PREFETCH never evicts.
#include <algorithm>
#include <mutex>
#include <vector>

#include "cache_policy.h"
#include "internal.h"
#include "prefetch_plan.h"

struct moe_cache {
  mm::CachePolicy policy;
  size_t blob_bytes = 0;
  const char* host = nullptr;
  char* dev = nullptr;
  hipStream_t demand_stream = nullptr, prefetch_stream = nullptr;
  const void** d_table = nullptr;          // device, [E]
  std::vector<char> pending_release, has_ready, has_released;
  std::vector<hipEvent_t> ready, released;
  std::vector<int> prefetched;             // slots whose latest copy was a PREFETCH that may still be in flight
  int prefetch_limit = -1;                 // copies one PREFETCH call may start; < 0: no bound
  double link_gbps = 0.0;                  // > 0: every copy is followed by a timed hold of its stream (slower link)
  int32_t* h_offsets = nullptr;            // pinned host, [E+1]: landing zone of expert_offsets
  moe_cache(int E, int n_slots) : policy(E, n_slots) {}
};

namespace mm {
namespace {

struct TableImage { const void* p[MOE_MAX_EXPERTS]; };

__global__ void table_update_kernel(const void** table, int E, const TableImage img) {
  for (int e = threadIdx.x; e < E; e += blockDim.x) table[e] = img.p[e];
}

// Holds the stream it runs on for `ticks` of the 100 MHz wall clock (one wave; bounded both by
// the clock and by an iteration count, so it always ends).
__global__ void hold_stream_kernel(long long ticks) {
  const long long t0 = wall_clock64();
  for (int i = 0; i < (1 << 22) && wall_clock64() - t0 < ticks; ++i) __builtin_amdgcn_s_sleep(32);
}

// The emulated link is one queue for the whole device: every emulated copy, whichever cache and
// stream carries it, starts when the one issued before it is over (its hold included).
std::mutex g_link_mutex;
hipEvent_t g_link_free[16];
bool g_link_has[16];

int issue_copy(moe_cache& c, int expert, int slot, hipStream_t cs) {
  if (c.has_released[slot]) MM_HIP(hipStreamWaitEvent(cs, c.released[slot], 0));
  if (c.has_ready[slot]) MM_HIP(hipStreamWaitEvent(cs, c.ready[slot], 0));   // an earlier copy into the slot
  if (c.link_gbps > 0.0) {
    // a hold of blob / link_gbps behind the copy: the link then delivers 1 / (1/link + 1/link_gbps)
    int dev = 0;
    MM_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 16) return fail(MOE_E_UNSUPPORTED, "link emulation: device %d", dev);
    const long long ticks = (long long)((double)c.blob_bytes / (c.link_gbps * 1e9) * 1e8);
    std::lock_guard<std::mutex> lock(g_link_mutex);
    if (!g_link_has[dev]) {
      MM_HIP(hipEventCreateWithFlags(&g_link_free[dev], hipEventDisableTiming));
    } else {
      MM_HIP(hipStreamWaitEvent(cs, g_link_free[dev], 0));
    }
    MM_HIP(hipMemcpyAsync(c.dev + (size_t)slot * c.blob_bytes, c.host + (size_t)expert * c.blob_bytes,
                          c.blob_bytes, hipMemcpyHostToDevice, cs));
    if (ticks > 0) {
      hipLaunchKernelGGL(hold_stream_kernel, dim3(1), dim3(64), 0, cs, ticks);
      MM_HIP(hipGetLastError());
    }
    MM_HIP(hipEventRecord(g_link_free[dev], cs));
    g_link_has[dev] = true;
  } else {
    MM_HIP(hipMemcpyAsync(c.dev + (size_t)slot * c.blob_bytes, c.host + (size_t)expert * c.blob_bytes,
                          c.blob_bytes, hipMemcpyHostToDevice, cs));
  }
  MM_HIP(hipEventRecord(c.ready[slot], cs));
  c.has_ready[slot] = 1;
  return MOE_OK;
}

// PREFETCH copies of this cache that have not landed yet (the list is pruned on the way).
int prefetch_in_flight(moe_cache& c) {
  size_t keep = 0;
  for (size_t i = 0; i < c.prefetched.size(); ++i) {
    const int s = c.prefetched[i];
    if (hipEventQuery(c.ready[s]) == hipErrorNotReady) c.prefetched[keep++] = s;
  }
  (void)hipGetLastError();                                // hipErrorNotReady is not a failure
  c.prefetched.resize(keep);
  return (int)keep;
}

// Points the device table at the slots of `ids` (all other experts NULL) on the compute stream,
// after making that stream wait for the copies into those slots.
int publish(moe_cache& c, const int32_t* ids, int n, hipStream_t cs) {
  TableImage img;
  for (int e = 0; e < MOE_MAX_EXPERTS; ++e) img.p[e] = nullptr;
  for (int i = 0; i < n; ++i) {
    const int s = c.policy.slot_of_expert(ids[i]);
    if (c.has_ready[s]) MM_HIP(hipStreamWaitEvent(cs, c.ready[s], 0));
    img.p[ids[i]] = c.dev + (size_t)s * c.blob_bytes;
  }
  hipLaunchKernelGGL(table_update_kernel, dim3(1), dim3(256), 0, cs, c.d_table, c.policy.n_experts(), img);
  return hip_fail(hipGetLastError(), "table_update_kernel launch");
}

// The policy decision of one call plus its copies.  With `publish_now` (DEMAND) the compute
// stream is made to wait for all of the call's slots and the pointer table is rewritten.
int fetch_impl(moe_cache& c, const int32_t* ids, int n, int mode, int32_t* slot_of, moe_fetch_stats* stats,
               hipStream_t cs, bool publish_now, int max_copies) {
  std::vector<PolicyCopy> copies;
  PolicyCounts counts = {0, 0, 0};
  std::vector<int32_t> slots_local((size_t)std::max(n, 1));
  int32_t* so = slot_of ? slot_of : slots_local.data();
  const int prc = c.policy.fetch(ids, n, mode == MOE_FETCH_DEMAND ? kPolicyDemand : kPolicyPrefetch,
                                 max_copies, so, &copies, &counts);
  switch (prc) {
    case kPolicyOk: break;
    case kPolicyBadId: return fail(MOE_E_BADARG, "expert_cache_fetch: expert id outside [0,%d)", c.policy.n_experts());
    case kPolicyDuplicate: return fail(MOE_E_BADARG, "expert_cache_fetch: an expert id is named twice");
    case kPolicyTooMany:
      return fail(MOE_E_CACHE_FULL, "expert_cache_fetch: DEMAND of %d experts exceeds the %d slots; split the step into waves",
                  n, c.policy.n_slots());
    default: return fail(MOE_E_BADARG, "expert_cache_fetch: mode %d", mode);
  }
  if (mode == MOE_FETCH_DEMAND) {
    // everything enqueued so far on the compute stream may still read the slots of the previous DEMAND
    for (int s = 0; s < c.policy.n_slots(); ++s)
      if (c.pending_release[s]) {
        MM_HIP(hipEventRecord(c.released[s], cs));
        c.has_released[s] = 1;
        c.pending_release[s] = 0;
      }
  }
  hipStream_t copy_stream = mode == MOE_FETCH_DEMAND ? c.demand_stream : c.prefetch_stream;
  for (const PolicyCopy& cp : copies) {
    const int rc = issue_copy(c, cp.expert, cp.slot, copy_stream);
    if (rc) return rc;
    if (mode == MOE_FETCH_PREFETCH && std::find(c.prefetched.begin(), c.prefetched.end(), cp.slot) == c.prefetched.end())
      c.prefetched.push_back(cp.slot);
  }
  if (mode == MOE_FETCH_DEMAND) {
    for (int i = 0; i < n; ++i) c.pending_release[so[i]] = 1;
    if (publish_now) {
      const int rc = publish(c, ids, n, cs);
      if (rc) return rc;
    }
  }
  if (stats) {
    stats->hits = counts.hits; stats->misses = counts.misses; stats->dropped = counts.dropped;
    stats->reserved = 0;
    stats->bytes_h2d = (uint64_t)counts.misses * c.blob_bytes;
  }
  return MOE_OK;
}

}  // namespace
}  // namespace mm

using namespace mm;

extern "C" moe_cache_t* moe_cache_create(int32_t E, size_t blob_bytes, int32_t n_slots,
                                         const void* host_blobs, void* device_slots) {
  if (E <= 0 || E > MOE_MAX_EXPERTS || n_slots <= 0 || blob_bytes == 0 || !host_blobs || !device_slots) {
    fail(MOE_E_BADARG, "moe_cache_create: E=%d n_slots=%d blob_bytes=%zu host=%p dev=%p", E, n_slots,
         blob_bytes, host_blobs, device_slots);
    return nullptr;
  }
  if (((uintptr_t)device_slots & 255) || (blob_bytes & 15)) {
    fail(MOE_E_BADARG, "moe_cache_create: device_slots must be 256-byte aligned, blob_bytes a multiple of 16");
    return nullptr;
  }
  moe_cache* c = new moe_cache(E, n_slots);
  c->blob_bytes = blob_bytes;
  c->host = static_cast<const char*>(host_blobs);
  c->dev = static_cast<char*>(device_slots);
  c->pending_release.assign(n_slots, 0);
  c->has_ready.assign(n_slots, 0);
  c->has_released.assign(n_slots, 0);
  bool ok = hipStreamCreateWithFlags(&c->demand_stream, hipStreamNonBlocking) == hipSuccess;
  ok = ok && hipStreamCreateWithFlags(&c->prefetch_stream, hipStreamNonBlocking) == hipSuccess;
  ok = ok && hipMalloc((void**)&c->d_table, sizeof(void*) * E) == hipSuccess;
  ok = ok && hipMemset((void*)c->d_table, 0, sizeof(void*) * E) == hipSuccess;
  ok = ok && hipHostMalloc((void**)&c->h_offsets, sizeof(int32_t) * (E + 1), hipHostMallocDefault) == hipSuccess;
  for (int s = 0; ok && s < n_slots; ++s) {
    hipEvent_t a, b;
    ok = hipEventCreateWithFlags(&a, hipEventDisableTiming) == hipSuccess &&
         hipEventCreateWithFlags(&b, hipEventDisableTiming) == hipSuccess;
    if (ok) { c->ready.push_back(a); c->released.push_back(b); }
  }
  if (!ok) {
    hip_fail(hipGetLastError(), "moe_cache_create");
    moe_cache_destroy(c);
    return nullptr;
  }
  return c;
}

extern "C" void moe_cache_destroy(moe_cache_t* c) {
  if (!c) return;
  for (hipStream_t s : {c->demand_stream, c->prefetch_stream})
    if (s) { (void)hipStreamSynchronize(s); (void)hipStreamDestroy(s); }
  for (hipEvent_t e : c->ready) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->released) (void)hipEventDestroy(e);
  if (c->d_table) (void)hipFree((void*)c->d_table);
  if (c->h_offsets) (void)hipHostFree(c->h_offsets);
  delete c;
}

extern "C" const void* const* moe_cache_expert_table(moe_cache_t* c) { return c ? c->d_table : nullptr; }

extern "C" int moe_cache_snapshot(moe_cache_t* c, int32_t* resident_expert) {
  if (!c || !resident_expert) return fail(MOE_E_BADARG, "moe_cache_snapshot: null argument");
  for (int s = 0; s < c->policy.n_slots(); ++s) resident_expert[s] = c->policy.expert_in_slot(s);
  return c->policy.n_slots();
}

extern "C" int moe_cache_sync(moe_cache_t* c) {
  if (!c) return fail(MOE_E_BADARG, "moe_cache_sync: null cache");
  MM_HIP(hipStreamSynchronize(c->demand_stream));
  MM_HIP(hipStreamSynchronize(c->prefetch_stream));
  return MOE_OK;
}

extern "C" int moe_cache_set_prefetch_limit(moe_cache_t* c, int32_t max_copies_per_call) {
  if (!c) return fail(MOE_E_BADARG, "moe_cache_set_prefetch_limit: null cache");
  c->prefetch_limit = max_copies_per_call < 0 ? -1 : max_copies_per_call;
  return MOE_OK;
}

extern "C" int moe_cache_emulate_link(moe_cache_t* c, double gb_per_s) {
  if (!c || !(gb_per_s >= 0.0)) return fail(MOE_E_BADARG, "moe_cache_emulate_link: null cache or negative rate");
  c->link_gbps = gb_per_s;
  return MOE_OK;
}

extern "C" int expert_cache_fetch(moe_cache_t* c, const int32_t* ids, int32_t n, int32_t mode,
                                  int32_t* slot_of, moe_fetch_stats* stats, void* compute_stream) {
  if (!c || n < 0 || (n > 0 && (!ids || !slot_of)))
    return fail(MOE_E_BADARG, "expert_cache_fetch: null argument or n < 0");
  if (mode != MOE_FETCH_DEMAND && mode != MOE_FETCH_PREFETCH)
    return fail(MOE_E_BADARG, "expert_cache_fetch: mode %d", mode);
  return fetch_impl(*c, ids, n, mode, slot_of, stats, static_cast<hipStream_t>(compute_stream), true,
                    c->prefetch_limit);
}

// One step's execution stage with offloaded experts: the router's decision is brought to the
// host (the only host synchronisation of a step), the needed experts are fetched in waves of at
// most n_slots (resident ones first), and within a wave the grouped FFN is launched for the
// experts that were resident at once and then for the missing ones a few at a time, each launch
// waiting only for its own experts' copies, so that computing overlaps the copies that follow.
extern "C" int moe_expert_ffn_cached(const moe_config* cfg, moe_cache_t* c, const void* x,
                                     const int32_t* expert_offsets, const int32_t* sorted_token,
                                     const void* const* shared_w, float* y, float* shared_out, void* ws,
                                     size_t ws_bytes, moe_fetch_stats* total, int32_t* n_waves,
                                     void* stream) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  if (!c) return fail(MOE_E_BADARG, "moe_expert_ffn_cached: cache is NULL");
  const int E = c->policy.n_experts(), S = c->policy.n_slots();
  if (cfg->E != E) return fail(MOE_E_SHAPE, "moe_expert_ffn_cached: cache holds %d experts, layer has %d", E, cfg->E);
  const size_t need = expert_blob_bytes(cfg->dtype, cfg->H, cfg->I);
  if (need != c->blob_bytes) return fail(MOE_E_SHAPE, "moe_expert_ffn_cached: blob of %zu bytes, layer needs %zu", c->blob_bytes, need);
  moe_fetch_stats sum = {0, 0, 0, 0, 0};
  if (n_waves) *n_waves = 0;
  if (total) *total = sum;
  if (cfg->T == 0) return MOE_OK;
  if (!expert_offsets) return fail(MOE_E_BADARG, "moe_expert_ffn_cached: expert_offsets is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  MM_HIP(hipMemcpyAsync(c->h_offsets, expert_offsets, sizeof(int32_t) * (E + 1), hipMemcpyDeviceToHost, s));
  // shared experts do not depend on the router: enqueue them before waiting for it
  if (cfg->n_shared > 0) {
    rc = moe_expert_ffn(cfg, x, expert_offsets, sorted_token, nullptr, shared_w, 0, 1, y, shared_out, ws, ws_bytes, stream);
    if (rc) return rc;
  }
  MM_HIP(hipStreamSynchronize(s));
  std::vector<int32_t> needed, order;
  for (int e = 0; e < E; ++e)
    if (c->h_offsets[e + 1] > c->h_offsets[e]) needed.push_back(e);
  c->policy.wave_order(needed, &order);
  // missing experts per FFN launch: about 32 MB of copies, so that a launch's fixed cost stays
  // small next to the copy time it hides under
  const int per_launch = (int)std::max<size_t>(1, ((size_t)32 << 20) / c->blob_bytes);
  std::vector<int32_t> slots(S), part;
  int waves = 0;
  for (size_t i = 0; i < order.size(); i += S) {
    const int n = (int)std::min<size_t>(S, order.size() - i);
    const int32_t* ids = order.data() + i;
    std::vector<char> was_resident(n);
    for (int k = 0; k < n; ++k) was_resident[k] = c->policy.slot_of_expert(ids[k]) >= 0;
    moe_fetch_stats st;
    rc = fetch_impl(*c, ids, n, MOE_FETCH_DEMAND, slots.data(), &st, s, false, -1);
    if (rc) return rc;
    sum.hits += st.hits; sum.misses += st.misses; sum.bytes_h2d += st.bytes_h2d;
    // residents of the wave in one launch, then the misses in copy order (ascending id)
    for (int pass = 0; pass < 2; ++pass) {
      part.clear();
      for (int k = 0; k <= n; ++k) {
        if (k < n && (pass == 0) == (bool)was_resident[k]) part.push_back(ids[k]);
        const bool flush = k == n || (pass == 1 && (int)part.size() == per_launch);
        if (!flush || part.empty()) continue;
        rc = publish(*c, part.data(), (int)part.size(), s);
        if (rc) return rc;
        rc = moe_expert_ffn(cfg, x, expert_offsets, sorted_token, moe_cache_expert_table(c), nullptr, 1, 0, y,
                            shared_out, ws, ws_bytes, stream);
        if (rc) return rc;
        part.clear();
      }
    }
    ++waves;
  }
  if (n_waves) *n_waves = waves;
  if (total) *total = sum;
  return MOE_OK;
}

// ---------------------------------------------------------------------------------------------
// Prefetch scheduler over the caches of a stack of layers (Sec. III-B).
struct moe_prefetcher {
  mm::PrefetchPlan plan;
  std::vector<moe_cache*> caches;
  float* h_logits = nullptr;               // pinned host staging, [n_layers][T][E]
  size_t h_floats = 0;
  int in_flight_limit = -1;                // PREFETCH copies in flight over all layers; < 0: no bound
  bool yield_to_demand = false;            // start no copy while a DEMAND copy of any layer is in flight
  moe_prefetcher(int L, int E, int k) : plan(L, E, k) {}
};

extern "C" moe_prefetcher_t* moe_prefetcher_create(int32_t n_layers, moe_cache_t* const* caches, int32_t k_big) {
  if (n_layers <= 0 || !caches || !caches[0]) {
    fail(MOE_E_BADARG, "moe_prefetcher_create: n_layers=%d caches=%p", n_layers, (const void*)caches);
    return nullptr;
  }
  const int E = caches[0]->policy.n_experts();
  for (int l = 0; l < n_layers; ++l)
    if (!caches[l] || caches[l]->policy.n_experts() != E) {
      fail(MOE_E_BADARG, "moe_prefetcher_create: cache of layer %d is NULL or holds another number of experts", l);
      return nullptr;
    }
  if (k_big < 1 || k_big > E) {
    fail(MOE_E_BADARG, "moe_prefetcher_create: k_big=%d with %d experts", k_big, E);
    return nullptr;
  }
  moe_prefetcher* p = new moe_prefetcher(n_layers, E, k_big);
  p->caches.assign(caches, caches + n_layers);
  return p;
}

extern "C" void moe_prefetcher_destroy(moe_prefetcher_t* p) {
  if (!p) return;
  if (p->h_logits) (void)hipHostFree(p->h_logits);
  delete p;
}

extern "C" int moe_prefetcher_set_in_flight_limit(moe_prefetcher_t* p, int32_t max_copies_in_flight) {
  if (!p) return fail(MOE_E_BADARG, "moe_prefetcher_set_in_flight_limit: null scheduler");
  p->in_flight_limit = max_copies_in_flight < 0 ? -1 : max_copies_in_flight;
  return MOE_OK;
}

extern "C" int moe_prefetcher_set_yield_to_demand(moe_prefetcher_t* p, int32_t on) {
  if (!p) return fail(MOE_E_BADARG, "moe_prefetcher_set_yield_to_demand: null scheduler");
  p->yield_to_demand = on != 0;
  return MOE_OK;
}

extern "C" int moe_prefetcher_predict(moe_prefetcher_t* p, const float* const* layer_logits, int32_t T,
                                      const int32_t* rejected, int32_t n_rejected, void* stream) {
  if (!p || n_rejected < 0 || T < 0) return fail(MOE_E_BADARG, "moe_prefetcher_predict: null scheduler or negative count");
  if (n_rejected == 0) { p->plan.clear(); return MOE_OK; }
  if (!layer_logits || !rejected) return fail(MOE_E_BADARG, "moe_prefetcher_predict: null argument");
  const int L = p->plan.n_layers(), E = p->plan.n_experts();
  for (int i = 0; i < n_rejected; ++i)
    if (rejected[i] < 0 || rejected[i] >= T)
      return fail(MOE_E_BADARG, "moe_prefetcher_predict: token %d outside [0,%d)", rejected[i], T);
  for (int l = 0; l < L; ++l)
    if (!layer_logits[l]) return fail(MOE_E_BADARG, "moe_prefetcher_predict: logits of layer %d are NULL", l);
  const size_t per_layer = (size_t)T * E, need = per_layer * L;
  if (need > p->h_floats) {
    if (p->h_logits) MM_HIP(hipHostFree(p->h_logits));
    p->h_logits = nullptr;
    p->h_floats = 0;
    MM_HIP(hipHostMalloc((void**)&p->h_logits, need * sizeof(float), hipHostMallocDefault));
    p->h_floats = need;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  for (int l = 0; l < L; ++l)
    MM_HIP(hipMemcpyAsync(p->h_logits + per_layer * l, layer_logits[l], per_layer * sizeof(float),
                          hipMemcpyDeviceToHost, s));
  MM_HIP(hipStreamSynchronize(s));
  p->plan.predict(p->h_logits, T, rejected, n_rejected);
  return MOE_OK;
}

extern "C" int moe_prefetcher_predicted(moe_prefetcher_t* p, int32_t layer, int32_t* ids) {
  if (!p || !ids || layer < 0 || layer >= p->plan.n_layers())
    return fail(MOE_E_BADARG, "moe_prefetcher_predicted: null argument or layer %d", layer);
  const std::vector<int32_t>& v = p->plan.layer(layer);
  std::copy(v.begin(), v.end(), ids);
  return (int)v.size();
}

extern "C" int moe_prefetcher_advance(moe_prefetcher_t* p, int32_t layer, int32_t distance, int32_t* issued_layers,
                                      int32_t* limits_used, moe_fetch_stats* issued_stats, void* compute_stream) {
  if (!p || distance < 0 || layer < -1 || layer >= p->plan.n_layers())
    return fail(MOE_E_BADARG, "moe_prefetcher_advance: null scheduler, layer %d or distance %d", layer, distance);
  std::vector<int32_t> due((size_t)p->plan.n_layers());
  const int n_due = p->plan.due(layer, distance, due.data());
  int n_issued = 0;
  for (int i = 0; i < n_due; ++i) {
    const int l = due[i];
    const std::vector<int32_t>& ids = p->plan.layer(l);
    if (ids.empty()) continue;
    moe_cache& c = *p->caches[l];
    int limit = c.prefetch_limit;
    if (p->in_flight_limit >= 0) {
      int flying = 0;
      for (moe_cache* q : p->caches) flying += prefetch_in_flight(*q);
      const int room = std::max(0, p->in_flight_limit - flying);
      limit = limit < 0 ? room : std::min(limit, room);
    }
    if (p->yield_to_demand) {
      bool busy = false;
      for (moe_cache* q : p->caches) busy = busy || hipStreamQuery(q->demand_stream) == hipErrorNotReady;
      (void)hipGetLastError();                            // hipErrorNotReady is not a failure
      if (busy) limit = 0;
    }
    moe_fetch_stats st;
    const int rc = fetch_impl(c, ids.data(), (int)ids.size(), MOE_FETCH_PREFETCH, nullptr, &st,
                              static_cast<hipStream_t>(compute_stream), false, limit);
    if (rc) return rc;
    if (issued_layers) issued_layers[n_issued] = l;
    if (limits_used) limits_used[n_issued] = limit;
    if (issued_stats) issued_stats[n_issued] = st;
    ++n_issued;
  }
  return n_issued;
}
