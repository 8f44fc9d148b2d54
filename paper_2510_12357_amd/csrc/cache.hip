// HBM expert cache: on-demand fetch and prefetch of expert blobs from pinned host DRAM
// (Sec. II-B: experts are loaded over the host link when the router selects them; Sec. III-B:
// the router outputs of a token's discarded little pass name the experts of its big pass ahead
// of time, so their copies can overlap with compute).
//
// All policy decisions are host-side integer bookkeeping and depend only on the sequence of
// calls, never on timing.  Data movement is hipMemcpyAsync on one side stream of default
// priority; ordering against the compute stream uses two events per slot:
//   ready[s]     recorded on the copy stream after the copy into slot s; the compute stream waits
//   released[s]  recorded on the compute stream at the start of the first fetch call after the
//                slot was handed out by a DEMAND call, i.e. after every kernel that may read the
//                slot has been enqueued; a later copy into the slot waits for it
#include <algorithm>
#include <vector>

#include "internal.h"

struct moe_cache {
  int E = 0, n_slots = 0;
  size_t blob_bytes = 0;
  const char* host = nullptr;
  char* dev = nullptr;
  hipStream_t copy_stream = nullptr;
  const void** d_table = nullptr;          // device, [E]
  std::vector<int> slot_expert, expert_slot;
  std::vector<uint64_t> stamp, demand_epoch;
  std::vector<char> pending_release, has_ready, has_released;
  std::vector<hipEvent_t> ready, released;
  uint64_t clock = 0, epoch = 0;
  int32_t* h_offsets = nullptr;            // pinned host, [E+1]: landing zone of expert_offsets
};

namespace mm {
namespace {

constexpr uint64_t kNever = ~0ull;

struct TableImage { const void* p[MOE_MAX_EXPERTS]; };

__global__ void table_update_kernel(const void** table, int E, const TableImage img) {
  for (int e = threadIdx.x; e < E; e += blockDim.x) table[e] = img.p[e];
}

// least recently stamped slot among those the predicate admits; lowest id among equals
template <typename Pred>
int pick_victim(const moe_cache& c, Pred admissible) {
  int best = -1;
  for (int s = 0; s < c.n_slots; ++s) {
    if (!admissible(s)) continue;
    if (best < 0 || c.stamp[s] < c.stamp[best]) best = s;
  }
  return best;
}

int issue_copy(moe_cache& c, int expert, int slot) {
  if (c.has_released[slot]) MM_HIP(hipStreamWaitEvent(c.copy_stream, c.released[slot], 0));
  MM_HIP(hipMemcpyAsync(c.dev + (size_t)slot * c.blob_bytes, c.host + (size_t)expert * c.blob_bytes,
                        c.blob_bytes, hipMemcpyHostToDevice, c.copy_stream));
  MM_HIP(hipEventRecord(c.ready[slot], c.copy_stream));
  c.has_ready[slot] = 1;
  return MOE_OK;
}

void assign(moe_cache& c, int expert, int slot) {
  const int old = c.slot_expert[slot];
  if (old >= 0) c.expert_slot[old] = -1;
  c.slot_expert[slot] = expert;
  c.expert_slot[expert] = slot;
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
  moe_cache* c = new moe_cache();
  c->E = E; c->n_slots = n_slots; c->blob_bytes = blob_bytes;
  c->host = static_cast<const char*>(host_blobs);
  c->dev = static_cast<char*>(device_slots);
  c->slot_expert.assign(n_slots, -1);
  c->expert_slot.assign(E, -1);
  c->stamp.assign(n_slots, 0);
  c->demand_epoch.assign(n_slots, kNever);
  c->pending_release.assign(n_slots, 0);
  c->has_ready.assign(n_slots, 0);
  c->has_released.assign(n_slots, 0);
  bool ok = hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking) == hipSuccess;
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
  if (c->copy_stream) { (void)hipStreamSynchronize(c->copy_stream); (void)hipStreamDestroy(c->copy_stream); }
  for (hipEvent_t e : c->ready) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->released) (void)hipEventDestroy(e);
  if (c->d_table) (void)hipFree((void*)c->d_table);
  if (c->h_offsets) (void)hipHostFree(c->h_offsets);
  delete c;
}

extern "C" const void* const* moe_cache_expert_table(moe_cache_t* c) { return c ? c->d_table : nullptr; }

extern "C" int moe_cache_snapshot(moe_cache_t* c, int32_t* resident_expert) {
  if (!c || !resident_expert) return fail(MOE_E_BADARG, "moe_cache_snapshot: null argument");
  for (int s = 0; s < c->n_slots; ++s) resident_expert[s] = c->slot_expert[s];
  return c->n_slots;
}

extern "C" int moe_cache_sync(moe_cache_t* c) {
  if (!c) return fail(MOE_E_BADARG, "moe_cache_sync: null cache");
  MM_HIP(hipStreamSynchronize(c->copy_stream));
  return MOE_OK;
}

extern "C" int expert_cache_fetch(moe_cache_t* c, const int32_t* ids, int32_t n, int32_t mode,
                                  int32_t* slot_of, moe_fetch_stats* stats, void* compute_stream) {
  if (!c || n < 0 || (n > 0 && (!ids || !slot_of)))
    return fail(MOE_E_BADARG, "expert_cache_fetch: null argument or n < 0");
  if (mode != MOE_FETCH_DEMAND && mode != MOE_FETCH_PREFETCH)
    return fail(MOE_E_BADARG, "expert_cache_fetch: mode %d", mode);
  std::vector<char> needed(c->E, 0);
  for (int i = 0; i < n; ++i) {
    if (ids[i] < 0 || ids[i] >= c->E) return fail(MOE_E_BADARG, "expert_cache_fetch: expert id %d outside [0,%d)", ids[i], c->E);
    if (needed[ids[i]]) return fail(MOE_E_BADARG, "expert_cache_fetch: expert id %d named twice", ids[i]);
    needed[ids[i]] = 1;
  }
  if (mode == MOE_FETCH_DEMAND && n > c->n_slots)
    return fail(MOE_E_CACHE_FULL, "expert_cache_fetch: DEMAND of %d experts exceeds the %d slots; split the step into waves", n, c->n_slots);

  hipStream_t cs = static_cast<hipStream_t>(compute_stream);
  // everything enqueued so far on the compute stream may still read the slots of earlier DEMANDs
  for (int s = 0; s < c->n_slots; ++s)
    if (c->pending_release[s]) {
      MM_HIP(hipEventRecord(c->released[s], cs));
      c->has_released[s] = 1;
      c->pending_release[s] = 0;
    }

  moe_fetch_stats st = {0, 0, 0, 0, 0};
  c->clock++;
  if (mode == MOE_FETCH_DEMAND) {
    c->epoch++;
    for (int e = 0; e < c->E; ++e) {              // residents first, ascending id
      if (!needed[e] || c->expert_slot[e] < 0) continue;
      const int s = c->expert_slot[e];
      c->stamp[s] = c->clock; c->demand_epoch[s] = c->epoch;
      st.hits++;
    }
    for (int e = 0; e < c->E; ++e) {              // then the misses, ascending id
      if (!needed[e] || c->expert_slot[e] >= 0) continue;
      const int v = pick_victim(*c, [&](int s) { return c->slot_expert[s] < 0 || !needed[c->slot_expert[s]]; });
      if (v < 0) return fail(MOE_E_CACHE_FULL, "expert_cache_fetch: no evictable slot (internal)");
      assign(*c, e, v);
      c->stamp[v] = c->clock; c->demand_epoch[v] = c->epoch;
      int rc = issue_copy(*c, e, v);
      if (rc) return rc;
      st.misses++;
    }
    TableImage img;
    for (int e = 0; e < MOE_MAX_EXPERTS; ++e) img.p[e] = nullptr;
    for (int i = 0; i < n; ++i) {
      const int s = c->expert_slot[ids[i]];
      slot_of[i] = s;
      if (c->has_ready[s]) MM_HIP(hipStreamWaitEvent(cs, c->ready[s], 0));
      c->pending_release[s] = 1;
      img.p[ids[i]] = c->dev + (size_t)s * c->blob_bytes;
    }
    hipLaunchKernelGGL(table_update_kernel, dim3(1), dim3(256), 0, cs, c->d_table, c->E, img);
    MM_HIP(hipGetLastError());
  } else {
    for (int i = 0; i < n; ++i) {                 // priority order as given
      const int e = ids[i];
      if (c->expert_slot[e] >= 0) {
        const int s = c->expert_slot[e];
        c->stamp[s] = c->clock;
        slot_of[i] = s;
        st.hits++;
        continue;
      }
      const int v = pick_victim(*c, [&](int s) {
        if (c->demand_epoch[s] != kNever && c->demand_epoch[s] == c->epoch) return false;
        return c->slot_expert[s] < 0 || !needed[c->slot_expert[s]];
      });
      if (v < 0) { slot_of[i] = -1; st.dropped++; continue; }
      assign(*c, e, v);
      c->stamp[v] = c->clock;
      int rc = issue_copy(*c, e, v);
      if (rc) return rc;
      slot_of[i] = v;
      st.misses++;
    }
  }
  st.bytes_h2d = (uint64_t)st.misses * c->blob_bytes;
  if (stats) *stats = st;
  return MOE_OK;
}

// One step's execution stage with offloaded experts: the router's decision is brought to the
// host (the only host synchronisation of a step), the needed experts are fetched in waves of at
// most n_slots (resident ones first, so their compute overlaps the first copies), and each wave
// runs the grouped FFN on exactly its experts through the cache's pointer table.
extern "C" int moe_expert_ffn_cached(const moe_config* cfg, moe_cache_t* c, const void* x,
                                     const int32_t* expert_offsets, const int32_t* sorted_token,
                                     const void* const* shared_w, float* y, float* shared_out, void* ws,
                                     size_t ws_bytes, moe_fetch_stats* total, int32_t* n_waves,
                                     void* stream) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  if (!c) return fail(MOE_E_BADARG, "moe_expert_ffn_cached: cache is NULL");
  if (cfg->E != c->E) return fail(MOE_E_SHAPE, "moe_expert_ffn_cached: cache holds %d experts, layer has %d", c->E, cfg->E);
  const size_t need = expert_blob_bytes(cfg->dtype, cfg->H, cfg->I);
  if (need != c->blob_bytes) return fail(MOE_E_SHAPE, "moe_expert_ffn_cached: blob of %zu bytes, layer needs %zu", c->blob_bytes, need);
  moe_fetch_stats sum = {0, 0, 0, 0, 0};
  if (n_waves) *n_waves = 0;
  if (total) *total = sum;
  if (cfg->T == 0) return MOE_OK;
  if (!expert_offsets) return fail(MOE_E_BADARG, "moe_expert_ffn_cached: expert_offsets is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  MM_HIP(hipMemcpyAsync(c->h_offsets, expert_offsets, sizeof(int32_t) * (c->E + 1), hipMemcpyDeviceToHost, s));
  // shared experts do not depend on the router: enqueue them before waiting for it
  if (cfg->n_shared > 0) {
    rc = moe_expert_ffn(cfg, x, expert_offsets, sorted_token, nullptr, shared_w, 0, 1, y, shared_out, ws, ws_bytes, stream);
    if (rc) return rc;
  }
  MM_HIP(hipStreamSynchronize(s));
  std::vector<int32_t> order;                      // resident experts first, then the misses
  for (int pass = 0; pass < 2; ++pass)
    for (int e = 0; e < c->E; ++e) {
      if (c->h_offsets[e + 1] <= c->h_offsets[e]) continue;
      const bool resident = c->expert_slot[e] >= 0;
      if ((pass == 0) == resident) order.push_back(e);
    }
  std::vector<int32_t> slots(c->n_slots);
  int waves = 0;
  for (size_t i = 0; i < order.size(); i += c->n_slots) {
    const int n = (int)std::min<size_t>(c->n_slots, order.size() - i);
    moe_fetch_stats st;
    rc = expert_cache_fetch(c, order.data() + i, n, MOE_FETCH_DEMAND, slots.data(), &st, stream);
    if (rc) return rc;
    sum.hits += st.hits; sum.misses += st.misses; sum.bytes_h2d += st.bytes_h2d;
    rc = moe_expert_ffn(cfg, x, expert_offsets, sorted_token, moe_cache_expert_table(c), nullptr, 1, 0, y,
                        shared_out, ws, ws_bytes, stream);
    if (rc) return rc;
    ++waves;
  }
  if (n_waves) *n_waves = waves;
  if (total) *total = sum;
  return MOE_OK;
}
