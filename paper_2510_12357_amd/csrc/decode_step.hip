// One decode step of the layer (at most 64 tokens) in ONE kernel launch: selection stage, dispatch,
// grouped SwiGLU feed-forward and the final weighted sum (Sec. II-A), with the per-token number of
// experts of the big-little rule (Sec. III-A, Alg. 1).
//
// Why one kernel: a decode step moves 0.1 .. 1 GB of expert weights, i.e. 15 .. 130 us of HBM
// time, and five dependent launches (router, dispatch, gate/up, down, combine) each pay a launch
// gap, a prologue and a pipeline ramp that the weight stream cannot hide.  Here the weight stream
// never stops: the workgroups are persistent (exactly as many as are resident), all work items of
// the step form one list, and what a later item needs from an earlier one is handed over through
// global memory with counters inside the kernel.
//
//   * item list (every workgroup derives the same list; workgroup b takes items b, b + G, ...):
//       A  gate/up items of the shared experts        - need nothing from the router
//       B  gate/up items of the routed experts        - need the selection
//       C  down items: shared experts' K chunks, then the routed experts
//     An item is 32 weight rows x all of K for up to 32 token rows, streamed through the LDS ring
//     of stream_lds.hip (4 loader waves issue global->LDS loads, 4 computer waves run the MFMAs).
//   * selection: workgroups 0..T-1 first compute the router logits and the selection of token b
//     (same code and bits as the stand-alone router kernels) while the others already stream the
//     shared experts; they publish through the counter `route_done`.
//   * dispatch: with at most 64 tokens, the tokens of an expert are a 64-bit mask.  When a
//     workgroup reaches its first item behind segment A (an iteration both kinds of waves can compute
//     in advance), all its waves build the E masks in LDS from the published selection (LDS atomic
//     OR: the result does not depend on the order), the offsets and the item list of B and C.
//     Position of pair (t, e) = offset[e] + popcount(mask[e] below bit t): the (expert ascending,
//     token ascending) order of the stand-alone dispatch.  Workgroup 0 also writes the dispatch
//     arrays of the C ABI.
//   * gate/up -> down: the wave that stored a tile of SwiGLU activations bumps `h_done` of the
//     down group (routed expert, or K chunk of a shared expert) the tile belongs to; a computer wave
//     that starts a down item first waits until that group's counter has reached the number of tiles
//     the group has.  The loaders never wait: the down weights are already in the ring by then.
//   * down -> sum: the wave that stored a tile of y bumps `col_done` of its 32 output columns; the
//     workgroup whose wave brings it to the number of tiles of the step notes the columns and, when
//     it has run out of items, sums them for all tokens with all its waves (ascending rank, then
//     the shared slabs: the order of the stand-alone combine).
//   * hand-over through memory: producers store with the device-coherent cache policy (sc1:
//     written through), and one iteration later, when the stores have long been acknowledged
//     (s_waitcnt vmcnt(0) then costs nothing), bump the counter with a device-scope atomic;
//     consumers poll the counter with device-scope atomic loads and read the data with sc1 loads.
//     (Plain accesses are not enough: the eight XCDs have separate L2 caches; plain stores stay
//     in the writer's L2 and plain loads are served stale lines, as a probe on the box showed.)
//   * no deadlock: an item only ever waits for items that precede it in the list, every workgroup
//     walks its items in list order, and all workgroups are resident.  Every wait is bounded all the
//     same: after `spin_limit` polls it gives up, records the fact in the error word and goes on.
//   * the last workgroup to leave resets the counters, so the next step starts from zero.
#include <atomic>

#include "internal.h"
#include "groups.h"
#include "route_device.h"

namespace mm {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int kRowBytes = 512;               // bytes of one weight row per chunk
constexpr int kRows = 32;                    // weight rows per item
constexpr int kStageBytes = kRows * kRowBytes;
constexpr int kStages = 4;
constexpr int kWorkers = 4;                  // loader waves = computer waves
constexpr int kThreadsD = 2 * kWorkers * 64;
constexpr int kTok = 32;                     // token rows per item, at most
constexpr int kKParts = 2;
constexpr int kReads = kRowBytes / 16 / 4 / kKParts;
#ifndef MOE_DECODE_LD_AUX
#define MOE_DECODE_LD_AUX 16
#endif
#ifndef MOE_DECODE_ST_AUX
#define MOE_DECODE_ST_AUX 16
#endif
#ifndef MOE_DECODE_POLL_SLEEP
#define MOE_DECODE_POLL_SLEEP 16
#endif
constexpr int kCoherent = 16;                // cache policy bit sc1 of buffer loads / stores: coherent across the device
constexpr int kCoherentLd = MOE_DECODE_LD_AUX, kCoherentSt = MOE_DECODE_ST_AUX;   // the bulk data: activations, y
constexpr unsigned kWholeBuffer = 0x7ffffff0u;

#define MM_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0f70 | ((n) & 15) | (((n) >> 4) << 14))
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ void compiler_fence() { asm volatile("" ::: "memory"); }

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ unsigned uni(unsigned v) { return (unsigned)__builtin_amdgcn_readfirstlane((int)v); }
template <typename P>
__device__ __forceinline__ P* uni(P* p) {
  const uint64_t v = (uint64_t)p;
  const uint64_t lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)v);
  const uint64_t hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(v >> 32));
  return (P*)((hi << 32) | lo);
}

// ---- counters of a step (ints, in the caller's workspace; zero between steps) ------------------
constexpr int kMaxColTiles = 1024;                            // H <= 32768
// A counter that many workgroups bump within a short time (the activations of one group: one bump
// per 16 x 16 tile) is cut into kShards counters; the tile picks its shard, a reader adds them up.
constexpr int kShards = 8;
enum {
  kSyncRouteDone = 0, kSyncExit = 1, kSyncErr = 2,
  kSyncExitSub = 4,                                           // [kShards] first level of the exit ticket
  kSyncHDone = kSyncExitSub + kShards,                        // [(kMaxSlabs + MOE_MAX_EXPERTS) * kShards]
  kSyncColDone = kSyncHDone + (kMaxSlabs + MOE_MAX_EXPERTS) * kShards,   // [kMaxColTiles]
  kSyncToken = kSyncColDone + kMaxColTiles,                   // [kDecodeMaxTokens] router parts of a token that are done
  kSyncInts = kSyncToken + kDecodeMaxTokens
};

#ifdef MOE_DECODE_TRACE
// Timeline of a step for analysis builds: 16 time stamps (100 MHz wall clock) per workgroup behind the counters.
constexpr int kTraceSlots = 16;
#define MM_TRACE(slot) do { if (tid == 4 * 64 && (slot) < kTraceSlots) \
  reinterpret_cast<long long*>(a.sync + kSyncInts * kCtrStride)[(size_t)blockIdx.x * kTraceSlots + (slot)] = wall_clock64(); } while (0)
#else
#define MM_TRACE(slot) do { } while (0)
#endif
#if defined(MOE_DECODE_TRACE) && MOE_DECODE_TRACE == 2
// per-iteration stamps: loader wave 0 in slots 0..15 of the upper half, computer wave 4 in the lower half
#define MM_TRACE_IT(who, it) do { if ((it) < 16 && lane == 0 && wave == (who)) \
  reinterpret_cast<long long*>(a.sync + kSyncInts * kCtrStride)[(size_t)(512 + ((who) ? 512 : 0) + blockIdx.x) * kTraceSlots + (it)] = wall_clock64(); } while (0)
#else
#define MM_TRACE_IT(who, it) do { } while (0)
#endif

// Every counter sits in a block of its own: device-scope atomics on one address are served one
// after the other at the memory side, and counters that shared a cache line made all their updates
// queue on one memory channel, in front of the weight stream.
#ifndef MOE_DECODE_CTR_STRIDE
#define MOE_DECODE_CTR_STRIDE 64
#endif
constexpr int kCtrStride = MOE_DECODE_CTR_STRIDE;             // ints between counters (256 bytes)
__device__ __forceinline__ int* ctr(int* sync, int index) { return sync + (size_t)index * kCtrStride; }

__device__ __forceinline__ int counter_load(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int counter_bump(int* p) {
  return __hip_atomic_fetch_add(p, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Sum of the kShards counters behind `index`: lane s < kShards loads shard s.  The loads are issued
// here; `shard_sum` turns what they brought into the sum.
__device__ __forceinline__ int shard_load(int* sync, int index, int lane) {
  return lane < kShards ? counter_load(ctr(sync, index + lane)) : 0;
}
__device__ __forceinline__ int shard_sum(int v) { return wave_reduce(v, 0, [](int x, int y) { return x + y; }); }

// One lane polls until the counter has reached `want`; bounded.  The pause between polls keeps
// the polling of many waiting workgroups (all on a few addresses, i.e. on one memory channel) from
// slowing the weight stream down.
__device__ __forceinline__ void counter_wait(int* sync, int index, int want, int spin_limit) {
  int spins = 0;
  while (counter_load(ctr(sync, index)) < want) {
    __builtin_amdgcn_s_sleep(MOE_DECODE_POLL_SLEEP);
    if (++spins > spin_limit) { atomicAdd(ctr(sync, kSyncErr), 1); break; }
  }
}
// The same for a sharded counter: the whole wave takes part.
__device__ __forceinline__ void shard_wait(int* sync, int index, int want, int spin_limit, int lane) {
  int spins = 0;
  while (shard_sum(shard_load(sync, index, lane)) < want) {
    __builtin_amdgcn_s_sleep(MOE_DECODE_POLL_SLEEP);
    if (++spins > spin_limit) { if (lane == 0) atomicAdd(ctr(sync, kSyncErr), 1); break; }
  }
}

__device__ __forceinline__ int coherent_load_i32(const void* base, unsigned byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b32(make_rsrc(base, kWholeBuffer), (int)byte_off, 0, kCoherent);
}
__device__ __forceinline__ void coherent_store_i32(void* base, unsigned byte_off, int v) {
  __builtin_amdgcn_raw_buffer_store_b32(v, make_rsrc(base, kWholeBuffer), (int)byte_off, 0, kCoherent);
}

struct DecodeArgs {
  int T, H, E, I, k_big, k_little, renorm;
  float gamma;
  int n_shared;
  int shared_I[MOE_MAX_SHARED];
  int shared_kchunk[MOE_MAX_SHARED];
  int n_slabs;
  int slab_shared[kMaxSlabs];
  int slab_chunk[kMaxSlabs];
  const void* shared_w[MOE_MAX_SHARED];
  const void* const* expert_w;        // device table [E]
  const void* x;                      // [T,H] bf16
  const void* Wg;                     // [E,H] bf16
  const float* bias;
  const float* conf;
  int logits_given;
  int route_split;                    // workgroups that share the router dot products of one token
  float* logits;                      // [T,E]
  int32_t* topk_idx;                  // [T,k_big]
  float* topk_w;
  uint8_t* important;
  int32_t* k_t;
  int32_t* expert_offsets;
  int32_t* sorted_token;
  int32_t* sorted_rank;
  int32_t* inv_pos;
  void* h_routed;                     // [T*k_big, I] bf16
  void* h_shared[MOE_MAX_SHARED];     // [T, I_s] bf16
  float* y;                           // [T*k_big, H]
  float* shared_out;                  // [n_slabs, T, H]
  void* out;                          // [T,H] bf16
  int* sync;
  int spin_limit;
};

constexpr int kMaxUGroups = MOE_MAX_SHARED + MOE_MAX_EXPERTS + kMaxSlabs + MOE_MAX_EXPERTS;

struct Smem {
  char ring[kStages * kStageBytes];
  float red[kWorkers][2][4][64];       // K-split partial sums; the router's logits before the loop
  unsigned long long mask[MOE_MAX_EXPERTS];   // tokens of each routed expert
  const void* blob[MOE_MAX_EXPERTS];   // weights of each routed expert (NULL: skipped)
  int off[MOE_MAX_EXPERTS + 1];        // first dispatch position of each expert
  int prefix[kMaxUGroups + 1];         // first item of each group of the unified list
  int col_want;                        // y tiles per 32 output columns in this step
  unsigned tile_bits[kMaxColTiles / 32];   // column tiles this workgroup sums when it has no items left
  int dep_seq;                         // 1 + ordinal of the latest item whose dependency wave 4 has seen met
  int flag;
};

struct DItem {
  // ---- same value in all lanes of the workgroup ----
  int valid;
  int down;         // 0: gate/up item, 1: down item
  int nch;          // chunks
  int K, N, m;
  int r0, n0;       // first token row / first weight row of the item
  int ntn;          // token tiles in use (1..2)
  int expert;       // routed gate/up: the expert whose token mask gives the rows; else -1
  unsigned ldwb;    // bytes between rows of W
  unsigned ldbb;    // bytes between rows of B
  const float* scale;
  unsigned wbytes, bbytes;
  const void* w0;
  const void* b;
  void* out;
  int dep, dep_want;  // down: counter (index into sync) to wait for and its target; gate/up: -1
  int sig;            // counter (index into sync) each storing wave bumps
  // ---- per lane ----
  unsigned a_row[4];  // loaders: byte offset of the weight row behind each of the wave's 4 loads
  unsigned boff;      // computers: byte offset of this lane's token row (kOob: none)
};

__device__ __forceinline__ int nth_set_bit(unsigned long long m, int n) {
  for (int i = 0; i < n; ++i) m &= m - 1;
  return m ? __ffsll((long long)m) - 1 : 0;
}
__device__ __forceinline__ unsigned long long bits_below(int t) { return t <= 0 ? 0ull : (~0ull >> (64 - t)); }

// Number of items of unified group g (needs the masks for the routed groups).
template <int WB>
__device__ __forceinline__ int group_items(const DecodeArgs& a, const Smem& sm, int g) {
  const int tg_all = (a.T + kTok - 1) / kTok;
  if (g < a.n_shared) return ((a.shared_I[g] + 15) / 16) * tg_all;
  g -= a.n_shared;
  if (g < a.E) {
    const int m = sm.blob[g] ? __popcll(sm.mask[g]) : 0;
    return ((a.I + 15) / 16) * ((m + kTok - 1) / kTok);
  }
  g -= a.E;
  if (g < a.n_slabs) return ((a.H + 31) / 32) * tg_all;
  g -= a.n_slabs;
  const int m = sm.blob[g] ? __popcll(sm.mask[g]) : 0;
  return ((a.H + 31) / 32) * ((m + kTok - 1) / kTok);
}

template <int WB>
__device__ __forceinline__ DItem decode_item(const DecodeArgs& a, const Smem& sm, int item, int total, int n_groups,
                                             int wave, int lane) {
  DItem it;
  it.valid = item < total;
  int cnt = 0;
  for (int g0 = 1; g0 <= n_groups; g0 += 64) {
    const int gg = g0 + lane;
    cnt += __popcll(__ballot(gg <= n_groups && sm.prefix[gg] <= item));
  }
  const int g = it.valid ? uni(cnt) : 0;
  const int local = item - uni(sm.prefix[g]);
  constexpr unsigned wsz = (unsigned)WB;
  constexpr int KC = kRowBytes / WB;
  // ---- the group ----
  int N, K, m, ldw, row0 = 0;
  const char* w0; const char* b; char* out; const float* scale;
  unsigned wbytes, bbytes;
  it.expert = -1; it.dep = -1; it.dep_want = 0; it.down = 0;
  int gg = g;
  if (gg < a.n_shared) {                                       // A: gate/up of shared expert gg
    const int Is = a.shared_I[gg];
    const char* blob = static_cast<const char*>(a.shared_w[gg]);
    N = Is; K = a.H; ldw = a.H; m = a.T;
    w0 = blob; wbytes = 2u * Is * a.H * wsz;
    b = static_cast<const char*>(a.x); bbytes = (unsigned)a.T * a.H * 2u;
    out = static_cast<char*>(a.h_shared[gg]);
    scale = reinterpret_cast<const float*>(blob + 3 * (size_t)Is * a.H * wsz);
    it.sig = 0;                                                // set per item below (depends on n0)
  } else if ((gg -= a.n_shared) < a.E) {                       // B: gate/up of routed expert gg
    const char* blob = static_cast<const char*>(uni(sm.blob[gg]));
    m = blob ? __popcll(sm.mask[gg]) : 0; m = uni(m);
    row0 = uni(sm.off[gg]);
    N = a.I; K = a.H; ldw = a.H;
    w0 = blob; wbytes = 2u * a.I * a.H * wsz;
    b = static_cast<const char*>(a.x); bbytes = (unsigned)a.T * a.H * 2u;
    out = static_cast<char*>(a.h_routed) + (size_t)row0 * a.I * 2u;
    scale = reinterpret_cast<const float*>(blob + 3 * (size_t)a.I * a.H * wsz);
    it.expert = gg;
    it.sig = kSyncHDone + (a.n_slabs + gg) * kShards;     // + shard, per item below
  } else if ((gg -= a.E) < a.n_slabs) {                        // C: down, K chunk of a shared expert
    const int s = a.slab_shared[gg], kb = a.slab_chunk[gg] * a.shared_kchunk[s];
    const int Is = a.shared_I[s];
    const char* blob = static_cast<const char*>(a.shared_w[s]);
    N = a.H; K = min(a.shared_kchunk[s], Is - kb); ldw = Is; m = a.T;
    w0 = blob + (2 * (size_t)Is * a.H + kb) * wsz; wbytes = ((unsigned)a.H * Is - kb) * wsz;
    b = static_cast<const char*>(a.h_shared[s]) + (size_t)kb * 2u; bbytes = ((unsigned)a.T * Is - kb) * 2u;
    out = reinterpret_cast<char*>(a.shared_out + (size_t)gg * a.T * a.H);
    scale = reinterpret_cast<const float*>(blob + 3 * (size_t)Is * a.H * wsz) + 2 * (size_t)Is;
    it.down = 1;
    it.dep = kSyncHDone + gg * kShards; it.dep_want = ((K + 15) / 16) * ((a.T + 15) / 16);
  } else {                                                     // C: down of routed expert gg
    gg -= a.n_slabs;
    const char* blob = static_cast<const char*>(uni(sm.blob[gg]));
    m = blob ? __popcll(sm.mask[gg]) : 0; m = uni(m);
    row0 = uni(sm.off[gg]);
    N = a.H; K = a.I; ldw = a.I;
    w0 = blob + 2 * (size_t)a.I * a.H * wsz; wbytes = (unsigned)a.H * a.I * wsz;
    b = static_cast<const char*>(a.h_routed) + (size_t)row0 * a.I * 2u; bbytes = (unsigned)m * a.I * 2u;
    out = reinterpret_cast<char*>(a.y + (size_t)row0 * a.H);
    scale = reinterpret_cast<const float*>(blob + 3 * (size_t)a.I * a.H * wsz) + 2 * (size_t)a.I;
    it.down = 1;
    it.dep = kSyncHDone + (a.n_slabs + gg) * kShards; it.dep_want = ((a.I + 15) / 16) * ((m + 15) / 16);
  }
  // ---- the item inside the group: blocks of 8 row tiles, the token blocks of a row tile 8 items
  // apart (on workgroups of the same XCD at the same time, so the repeated weight reads hit in L2)
  const int per = it.down ? 32 : 16;
  const int rows = (N + per - 1) / per;
  const int tgs = max(1, (m + kTok - 1) / kTok);
  int tg = 0, row_item = local;
  if (tgs > 1) {
    const int block = local / (8 * tgs);
    const int rem = local - block * 8 * tgs;
    const int nb = max(1, min(8, rows - 8 * block));
    tg = rem / nb;
    row_item = block * 8 + (rem - tg * nb);
  }
  it.r0 = tg * kTok;
  it.n0 = row_item * per;
  it.K = it.valid ? K : 0;
  it.N = N; it.m = it.valid ? m : 0;
  it.nch = (it.K + KC - 1) / KC;
  it.ntn = clampi((it.m - it.r0 + 15) >> 4, 1, kTok / 16);
  it.ldwb = (unsigned)ldw * wsz;
  it.ldbb = (unsigned)ldw * 2u;
  it.scale = scale;
  it.wbytes = it.valid ? wbytes : 0u; it.bbytes = it.valid ? bbytes : 0u;
  it.w0 = it.valid ? (const void*)w0 : a.x; it.b = it.valid ? (const void*)b : a.x; it.out = out;
  if (g < a.n_shared) {
    // the K chunk of the shared expert's down projection that these 16 activations feed
    int first_slab = 0;
    for (int s = 0; s < g; ++s) first_slab += (a.shared_I[s] + a.shared_kchunk[s] - 1) / a.shared_kchunk[s];
    it.sig = kSyncHDone + (first_slab + it.n0 / a.shared_kchunk[g]) * kShards + ((it.n0 >> 4) & (kShards - 1));
  } else if (it.expert >= 0) {
    it.sig += (it.n0 >> 4) & (kShards - 1);
  } else if (it.down) {
    it.sig = kSyncColDone + it.n0 / 32;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row_local = 2 * ((wave % kWorkers) * 4 + i) + (lane >> 5);
    unsigned off;
    int n;
    if (!it.down) {
      n = it.n0 + (row_local & 15);
      off = (unsigned)n * it.ldwb + ((row_local >> 4) ? (unsigned)N * it.ldwb : 0u);   // W_up follows W_gate
    } else {
      n = it.n0 + row_local;
      off = (unsigned)n * it.ldwb;
    }
    it.a_row[i] = (it.valid && n < N) ? off : kOob;
  }
  {
    const int r = it.r0 + (wave & 1) * 16 + (lane & 15);
    const bool val = it.valid && r < it.m;
    int row = r;
    if (it.expert >= 0) row = val ? nth_set_bit(sm.mask[it.expert], r) : 0;   // r-th token of the expert
    it.boff = val ? (unsigned)row * it.ldbb : kOob;
  }
  return it;
}


// out[t][c .. c+3] for the 32 columns of tile `tile` and all tokens, by the 8 waves of a workgroup:
// wave w takes tokens 8 w .. 8 w + 7, a lane four columns of one token.  All loads of a kind are
// issued together.  Sum order: rank ascending, then the shared slabs ascending (as the stand-alone
// combine); ranks from k_t on carry expert -1.
__device__ __forceinline__ void sum_columns(const DecodeArgs& a, const Smem& sm, int tile, int wave, int lane) {
  const int cc = tile * 32 + (lane & 7) * 4;
  const int t = wave * 8 + (lane >> 3);
  if (t >= a.T || cc >= a.H) return;
  const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, kWholeBuffer);
  const __amdgpu_buffer_rsrc_t rs = make_rsrc(a.shared_out, a.shared_out ? kWholeBuffer : 0u);
  const __amdgpu_buffer_rsrc_t ri = make_rsrc(a.topk_idx, kWholeBuffer), rw = make_rsrc(a.topk_w, kWholeBuffer);
  int e[MOE_MAX_TOPK];
  float w[MOE_MAX_TOPK];
#pragma unroll
  for (int j = 0; j < MOE_MAX_TOPK; ++j) {
    const unsigned off = j < a.k_big ? (unsigned)(t * a.k_big + j) * 4u : kOob;
    e[j] = __builtin_amdgcn_raw_buffer_load_b32(ri, (int)off, 0, kCoherent);
    w[j] = __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(rw, (int)off, 0, kCoherent));
    if (j >= a.k_big) e[j] = -1;
  }
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  static_assert(MOE_MAX_TOPK % 8 == 0 && kMaxSlabs % 4 == 0, "batches of 8 ranks and 4 slabs");
#pragma unroll
  for (int j0 = 0; j0 < MOE_MAX_TOPK; j0 += 8) {
    if (j0 >= a.k_big) break;
    i32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool ok = (unsigned)e[j0 + j] < (unsigned)a.E;
      const int ee = ok ? e[j0 + j] : 0;
      const int p = sm.off[ee] + __popcll(sm.mask[ee] & bits_below(t));
      v[j] = __builtin_amdgcn_raw_buffer_load_b128(ry, (int)(ok ? ((unsigned)p * a.H + cc) * 4u : kOob), 0, kCoherent);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if ((unsigned)e[j0 + j] < (unsigned)a.E) acc += w[j0 + j] * __builtin_bit_cast(f32x4, v[j]);
  }
#pragma unroll
  for (int s0 = 0; s0 < kMaxSlabs; s0 += 4) {
    if (s0 >= a.n_slabs) break;
    i32x4 sv[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
      sv[s] = __builtin_amdgcn_raw_buffer_load_b128(
          rs, (int)(s0 + s < a.n_slabs ? (((unsigned)(s0 + s) * a.T + t) * a.H + cc) * 4u : kOob), 0, kCoherent);
#pragma unroll
    for (int s = 0; s < 4; ++s)
      if (s0 + s < a.n_slabs) acc += __builtin_bit_cast(f32x4, sv[s]);
  }
  bf16x4 o = {(__bf16)acc[0], (__bf16)acc[1], (__bf16)acc[2], (__bf16)acc[3]};
  *reinterpret_cast<bf16x4*>(static_cast<uint16_t*>(a.out) + (size_t)t * a.H + cc) = o;
}

template <int WB>
__global__ __launch_bounds__(kThreadsD) __attribute__((amdgpu_waves_per_eu(4, 4))) void decode_step_kernel(const DecodeArgs a) {
  constexpr int KC = kRowBytes / WB;         // k per chunk
  constexpr int kHalves = 2 / WB;            // MFMA k-steps fed by one 16-byte column
  __shared__ __attribute__((aligned(1024))) Smem sm;
  char* const s_ring = sm.ring;
  float (&s_red)[kWorkers][2][4][64] = sm.red;

  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  const int q = lane >> 4, c16 = lane & 15;
  const int G = gridDim.x;
  // Place in the item list.  Workgroups b and b + G/2 of a launch of two workgroups per CU share a
  // CU (the dispatcher fills every CU once before it comes back to the first).  The router's
  // workgroups are the last of the grid; their CU-mates are put right in front of them in the order
  // the items are dealt in, i.e. they are the last to get an item of segment A: while the selection
  // is computed, the router's loads do not queue behind a weight stream on their own CU.
  // (Only when segment A leaves those workgroups without an item; with more items than that the
  // order would merely shift work between workgroups, and the plain order is the faster one.)
  int vb = (int)blockIdx.x;
  {
    const int R = min(a.T * a.route_split, G / 4), half = G / 2;
    int n_a = 0;
    for (int g = 0; g < a.n_shared; ++g) n_a += ((a.shared_I[g] + 15) / 16) * ((a.T + kTok - 1) / kTok);
    if ((G & 1) == 0 && n_a + 2 * R <= G) {
      const int b = (int)blockIdx.x;
      if (b >= half - R && b < half) vb = G - 2 * R + (b - (half - R));      // CU-mates of the router's workgroups
      else if (b >= half && b < G - R) vb = b - R;                           // the others close the gap
    }
  }
  const int n_groups = a.n_shared + a.E + a.n_slabs + a.E;
  const int gA = a.n_shared;                                  // groups of segment A

  MM_TRACE(0);
  // ---- prologue: expert pointers, segment A of the item list ----
  for (int e = tid; e < a.E; e += kThreadsD) { sm.blob[e] = a.expert_w[e]; sm.mask[e] = 0ull; }
  for (int i = tid; i < kMaxColTiles / 32; i += kThreadsD) sm.tile_bits[i] = 0u;
  if (tid == 0) {
    int run = 0;
    sm.prefix[0] = 0;
    for (int g = 0; g < gA; ++g) { run += ((a.shared_I[g] + 15) / 16) * ((a.T + kTok - 1) / kTok); sm.prefix[g + 1] = run; }
    // until the selection is known the list ends behind segment A
    for (int g = gA; g < n_groups; ++g) sm.prefix[g + 1] = run;
  }

  // ---- selection stage: `route_split` workgroups per token compute its router logits (one pass
  // of 32 experts each); the one that finishes last selects ----
  if (tid == 0) sm.dep_seq = 0;
  // (the last workgroups of the grid: they get the fewest items of segment A, i.e. they would wait
  // for the selection first of all)
  const int route_id = G - 1 - vb;
  if (route_id < a.T * a.route_split) {
    const int t = route_id / a.route_split, part = route_id - t * a.route_split;
    const __amdgpu_buffer_rsrc_t rl = make_rsrc(a.logits, kWholeBuffer);
    if (!a.logits_given) {
      const int per = (a.E + a.route_split - 1) / a.route_split;
      const int e_begin = part * per, e_end = min(a.E, e_begin + per);
      gate_logits_token<uint16_t, 2 * kWorkers>(
          static_cast<const uint16_t*>(a.x) + (size_t)t * a.H, static_cast<const uint16_t*>(a.Wg), a.bias, a.H, a.E,
          e_begin, e_end, wave, lane, [&](int e, float z) {
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_int(z), rl, (int)((unsigned)(t * a.E + e) * 4u), 0, kCoherent);
          });
      compiler_fence();
      __builtin_amdgcn_s_waitcnt(0);                          // this wave's logits are in memory
      compiler_fence();
    }
    __syncthreads();
    if (tid == 0) sm.flag = a.logits_given ? part == 0 : counter_bump(ctr(a.sync, kSyncToken + t)) == a.route_split - 1;
    __syncthreads();
    if (sm.flag && wave == 0) {
      RouteParams P;
      P.conf = a.conf; P.gamma = a.gamma; P.T = a.T; P.E = a.E; P.k_big = a.k_big; P.k_little = a.k_little;
      P.renorm = a.renorm; P.idx = nullptr; P.w = nullptr; P.important = nullptr; P.k_t = nullptr;
      float raw[kPerLane];
#pragma unroll
      for (int c = 0; c < kPerLane; ++c) {
        const int e = lane + 64 * c;
        raw[c] = __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(rl, (int)(e < a.E ? (unsigned)(t * a.E + e) * 4u : kOob), 0,
                                                                     kCoherent));
      }
      const Selection sel = select_token_values(P, t, lane, raw);
      if (lane < a.k_big) {
        coherent_store_i32(a.topk_idx, (unsigned)(t * a.k_big + lane) * 4u, sel.expert);
        coherent_store_i32(a.topk_w, (unsigned)(t * a.k_big + lane) * 4u, __float_as_int(sel.weight));
      }
      if (lane == 0) {
        a.k_t[t] = sel.k;
        a.important[t] = sel.imp ? 1 : 0;
      }
      compiler_fence();
      __builtin_amdgcn_s_waitcnt(0);                          // the stores have been acknowledged
      compiler_fence();
      if (lane == 0) counter_bump(ctr(a.sync, kSyncRouteDone));
    }
  }
  __syncthreads();
  MM_TRACE(1);
  const int total_A = sm.prefix[gA];

  // Iteration at which this workgroup's loaders issue their first chunk behind segment A: all A
  // items have K = H.  Both kinds of waves run the dispatch block at the top of that iteration.
  const int my_A = total_A > vb ? (total_A - vb + G - 1) / G : 0;
  const int s_star = my_A * ((a.H + KC - 1) / KC);
  int total = total_A;                                        // items known so far

  // ---- dispatch block: token masks, offsets, item list of segments B and C (all 8 waves) ----
  auto dispatch_block = [&]() {
    const bool reader = wave >= kWorkers;                     // only computer waves touch global memory here
    const int rt = tid - kWorkers * 64;                       // 0..255 among the readers
    MM_TRACE(2);
    if (rt == 0) counter_wait(a.sync, kSyncRouteDone, a.T, a.spin_limit);
    MM_TRACE(3);
    for (int e = tid; e < a.E; e += kThreadsD) sm.mask[e] = 0ull;
    lds_barrier();
    compiler_fence();
    const int n_ent = a.T * a.k_big;                          // <= 64 * 16
    int ent_e[4], ent_ok[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      ent_e[u] = -1; ent_ok[u] = 0;
      const int i = rt + u * 256;
      if (reader && i < n_ent) {
        const int t = i / a.k_big;
        const int e = coherent_load_i32(a.topk_idx, (unsigned)i * 4u);    // -1 from rank k_t on
        ent_e[u] = e;
        ent_ok[u] = (unsigned)e < (unsigned)a.E;
        if (ent_ok[u]) atomicOr(&sm.mask[e], 1ull << t);
      }
    }
    lds_barrier();
    if (wave == 0) {
      // expert offsets: exclusive prefix of the masks' populations
      {
        constexpr int C = MOE_MAX_EXPERTS / 64;
        int loc[C], sum = 0;
#pragma unroll
        for (int c = 0; c < C; ++c) { const int e = lane * C + c; loc[c] = e < a.E ? __popcll(sm.mask[e]) : 0; sum += loc[c]; }
        int incl = sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { const int v = __shfl_up(incl, d); if (lane >= d) incl += v; }
        int run = incl - sum;
#pragma unroll
        for (int c = 0; c < C; ++c) { const int e = lane * C + c; if (e < a.E) sm.off[e] = run; run += loc[c]; }
        if (lane == 63) sm.off[a.E] = incl;
      }
      // items of the groups behind segment A, and the y tiles per 32 output columns
      {
        const int nB = n_groups - gA;
        const int C = (nB + 63) / 64;
        const int base = gA + lane * C;
        int sum = 0;
        for (int c = 0; c < C; ++c) if (base + c < n_groups) sum += group_items<WB>(a, sm, base + c);
        int incl = sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { const int v = __shfl_up(incl, d); if (lane >= d) incl += v; }
        int run = total_A + incl - sum;
        for (int c = 0; c < C; ++c) if (base + c < n_groups) { run += group_items<WB>(a, sm, base + c); sm.prefix[base + c + 1] = run; }
        int tiles = 0;
        for (int e = lane; e < a.E; e += 64) tiles += sm.blob[e] ? (__popcll(sm.mask[e]) + 15) / 16 : 0;
        tiles = wave_reduce(tiles, 0, [](int x, int y) { return x + y; });
        if (lane == 0) sm.col_want = tiles + a.n_slabs * ((a.T + 15) / 16);
      }
    }
    lds_barrier();
    MM_TRACE(4);
    total = sm.prefix[n_groups];
    // the dispatch arrays of the C ABI (workgroup 0, computer waves)
    if (blockIdx.x == 0 && reader) {
      const int P = sm.off[a.E];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = rt + u * 256;
        if (i < n_ent) {
          int p = -1;
          if (ent_ok[u]) {
            const int t = i / a.k_big;
            p = sm.off[ent_e[u]] + __popcll(sm.mask[ent_e[u]] & bits_below(t));
            a.sorted_token[p] = t;
            a.sorted_rank[p] = i - t * a.k_big;
          }
          a.inv_pos[i] = p;
        }
        if (i >= P && i < n_ent) { a.sorted_token[i] = -1; a.sorted_rank[i] = -1; }
      }
      for (int e = rt; e <= a.E; e += 256) a.expert_offsets[e] = sm.off[e];
    }
  };
  if (s_star == 0) dispatch_block();
  bool block_done = s_star == 0;

  if (wave < kWorkers) {
    // =================================== loader ===================================
    DItem it = decode_item<WB>(a, sm, vb, total, n_groups, wave, lane);
    DItem nx = it;
    bool nx_known = false;
    int j = 0, k = 0, drain = 0, s = 0;
    unsigned a_col[4], addr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row_local = 2 * (wave * 4 + i) + (lane >> 5);
      a_col[i] = (unsigned)((lane & 31) ^ (row_local & 15));
      addr[i] = it.a_row[i] + a_col[i] * 16u;
    }
    __amdgpu_buffer_rsrc_t rs = make_rsrc(it.w0, it.wbytes);
    MM_WAIT_VMCNT(0);
    auto set_item = [&]() {
      it = nx_known ? nx : decode_item<WB>(a, sm, vb + j * G, total, n_groups, wave, lane);
      nx_known = false;
      rs = make_rsrc(it.w0, it.wbytes);
#pragma unroll
      for (int i = 0; i < 4; ++i) addr[i] = it.a_row[i] + a_col[i] * 16u;
    };
    auto issue_next = [&]() -> bool {
      const bool real = k < it.nch;
      char* stage = s_ring + (s & (kStages - 1)) * kStageBytes + wave * 4096;
      if (real && (k + 1) * KC <= it.K) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)(stage + i * 1024), 16, (int)addr[i], 0, 0, kStreamOnce);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int kk = k * KC + (int)a_col[i] * (16 / WB);
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)(stage + i * 1024), 16,
                                                   (int)((real && kk < it.K) ? addr[i] : kOob), 0, 0, kStreamOnce);
        }
      }
      if (real) {
        ++k;
#pragma unroll
        for (int i = 0; i < 4; ++i) addr[i] += kRowBytes;
        // the next item is decoded under the loads of this one's first chunk when the list is known
        // that far (LDS and registers only: nothing joins the counted loads)
        if (k == 1 && (block_done || vb + (j + 1) * G < total_A)) {
          nx = decode_item<WB>(a, sm, vb + (j + 1) * G, total, n_groups, wave, lane);
          nx_known = true;
        }
        if (k == it.nch) { ++j; k = 0; set_item(); }
      }
      ++s;
      return real;
    };
    for (;;) {
      if (!block_done && s == s_star) { dispatch_block(); block_done = true; set_item(); }
      const bool real = issue_next();
      MM_WAIT_VMCNT(12);                                    // the chunk issued three iterations ago has landed
      MM_TRACE_IT(0, s - 1);
      lds_barrier();                                        // "landed"
      lds_barrier();                                        // "free"
      if (!real && block_done && ++drain == 3) break;
    }
    MM_WAIT_VMCNT(0);
  } else {
    // =================================== computer ===================================
    const int c = wave - kWorkers, tw = c & 1, kp = c >> 1;
    DItem cur = decode_item<WB>(a, sm, vb, total, n_groups, c, lane);
    int j = 0, k = 0;
    int pending = 0, started = 0;
    int pub = -1, pub_down = 0;     // counter this wave still has to bump for outputs it stored (-1: none)
    int tick = 0, tick_tile = -1;   // a bump of a column counter whose old value has not been looked at yet
    int f_r0 = 0, f_n0 = 0, f_m = 0, f_N = 0, f_ntn = 0, f_down = 0, f_sig = 0;
    void* f_out = nullptr;
    f32x4 sc[2] = {f32x4{0, 0, 0, 0}, f32x4{0, 0, 0, 0}}, f_sc[2] = {f32x4{0, 0, 0, 0}, f32x4{0, 0, 0, 0}};
    auto load_scales = [&](const DItem& it) {
      if (WB != 1) return;
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) {
        const int n = !it.down ? it.n0 + 4 * q : it.n0 + rt * 16 + 4 * q;
        const bool ok = it.valid && n < it.N;
        const float* p = it.scale + ((!it.down && rt == 1) ? it.N + n : n);
        sc[rt] = ok ? *reinterpret_cast<const f32x4*>(p) : f32x4{0, 0, 0, 0};
      }
    };
    const unsigned ring_base = (unsigned)(size_t)s_ring;
    unsigned rd_off[kReads];
#pragma unroll
    for (int t = 0; t < kReads; ++t)
      rd_off[t] = ring_base + (unsigned)c16 * kRowBytes + (unsigned)((((kp + t * kKParts) * 4 + q) ^ c16) * 16);
    i32x4 bbuf[kReads][kHalves];
#pragma unroll
    for (int t = 0; t < kReads; ++t)
#pragma unroll
      for (int h = 0; h < kHalves; ++h) bbuf[t][h] = i32x4{0, 0, 0, 0};
    f32x4 acc[2] = {f32x4{0, 0, 0, 0}, f32x4{0, 0, 0, 0}};

    // Scale (8-bit weights), activate and store this lane's 2 x 4 sums of the item that ended, with
    // the coherent cache policy: another workgroup reads them within this kernel.
    auto store_outputs = [&](float (&val)[2][4]) {
      if (WB == 1) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int v = 0; v < 4; ++v) val[rt][v] *= f_sc[rt][v];
      }
      const int r = f_r0 + tw * 16 + c16;
      const __amdgpu_buffer_rsrc_t ro = make_rsrc(f_out, kWholeBuffer);
      if (r < f_m) {
        if (!f_down) {
          const int i = f_n0 + 4 * q;
          if (i < f_N) {
            float hv[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const float gte = val[0][v];
              hv[v] = gte / (1.f + __expf(-gte)) * val[1][v];
            }
            bf16x4 o = {(__bf16)hv[0], (__bf16)hv[1], (__bf16)hv[2], (__bf16)hv[3]};
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(i32x2, o), ro,
                                                  (int)(((unsigned)r * f_N + i) * 2u), 0, kCoherentSt);
          }
        } else {
#pragma unroll
          for (int rt = 0; rt < 2; ++rt) {
            const int col = f_n0 + rt * 16 + 4 * q;
            if (col < f_N)
              __builtin_amdgcn_raw_buffer_store_b128(
                  __builtin_bit_cast(i32x4, f32x4{val[rt][0], val[rt][1], val[rt][2], val[rt][3]}), ro,
                  (int)(((unsigned)r * a.H + col) * 4u), 0, kCoherentSt);
          }
        }
      }
    };
    auto epilogue = [&]() {
      if (kp == 0 && tw < f_ntn) {
        float val[2][4];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int v = 0; v < 4; ++v) val[rt][v] = s_red[tw][rt][v][lane] + s_red[tw + 2][rt][v][lane];
        store_outputs(val);
        pub = f_sig; pub_down = f_down;                       // published later: see publish()
      }
    };
    // Tells the other workgroups that the outputs this wave stored last are in memory.  Called an
    // iteration after the stores (their acknowledgements have arrived by then), or at once when this
    // wave is about to wait for a counter itself.
    auto publish = [&]() {
      if (tick_tile >= 0) {           // issued an iteration ago: the old value has arrived
        if (uni(tick) + 1 == sm.col_want && lane == 0)        // it was the step's last y tile of these 32 columns
          atomicOr(&sm.tile_bits[tick_tile >> 5], 1u << (tick_tile & 31));
        tick_tile = -1;
      }
      if (pub < 0) return;
      compiler_fence();
      __builtin_amdgcn_s_waitcnt(0);
      compiler_fence();
      if (!pub_down) {
        if (lane == 0) (void)counter_bump(ctr(a.sync, pub));  // nobody needs the old value: no wait for it
      } else {
        tick = 0;
        if (lane == 0) tick = counter_bump(ctr(a.sync, pub));   // looked at by the next call
        tick_tile = pub - kSyncColDone;
      }
      pub = -1;
    };
    auto consume = [&](int stage) {
      const unsigned st = (unsigned)(stage * kStageBytes);
      bf16x8 f0[kReads], f1[kReads];
      static_assert(kReads == 4, "the fragment reads below are written for four columns per wave and row tile");
      asm volatile(
          "ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:8192\n"
          "ds_read_b128 %2, %9\n ds_read_b128 %3, %9 offset:8192\n"
          "ds_read_b128 %4, %10\n ds_read_b128 %5, %10 offset:8192\n"
          "ds_read_b128 %6, %11\n ds_read_b128 %7, %11 offset:8192\n"
          "s_waitcnt lgkmcnt(0)"
          : "=&v"(f0[0]), "=&v"(f1[0]), "=&v"(f0[1]), "=&v"(f1[1]), "=&v"(f0[2]), "=&v"(f1[2]), "=&v"(f0[3]), "=&v"(f1[3])
          : "v"(rd_off[0] + st), "v"(rd_off[1] + st), "v"(rd_off[2] + st), "v"(rd_off[3] + st)
          : "memory");
#pragma unroll
      for (int t = 0; t < kReads; ++t) {
        if (WB == 2) {
          const bf16x8 bv = __builtin_bit_cast(bf16x8, bbuf[t][0]);
          acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0[t], bv, acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f1[t], bv, acc[1], 0, 0, 0);
        } else {
          const i32x4 w0 = __builtin_bit_cast(i32x4, f0[t]), w1 = __builtin_bit_cast(i32x4, f1[t]);
#pragma unroll
          for (int h = 0; h < kHalves; ++h) {
            const bf16x8 bv = __builtin_bit_cast(bf16x8, bbuf[t][h]);
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(widen_e4m3(w0[2 * h], w0[2 * h + 1]), bv, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(widen_e4m3(w1[2 * h], w1[2 * h + 1]), bv, acc[1], 0, 0, 0);
          }
        }
      }
    };
    // Token rows of chunk (cur, k) into bbuf.  The activations of a down item were written by other
    // workgroups within this kernel: coherent loads.
    auto load_token_rows = [&](bool behind_stores) {
      // Nothing of this wave is in flight any more (the previous token rows were consumed): saying so
      // keeps the compiler from guarding every load below.  Not behind the stores of an epilogue:
      // waiting for their acknowledgement would stall the wave for a memory round trip.
      if (!behind_stores) MM_WAIT_VMCNT(0);
      const __amdgpu_buffer_rsrc_t rb = make_rsrc(cur.b, cur.bbytes);
#pragma unroll
      for (int t = 0; t < kReads; ++t)
#pragma unroll
        for (int h = 0; h < kHalves; ++h) {
          const int kk = k * KC + ((kp + t * kKParts) * 4 + q) * (16 / WB) + h * 8;
          const bool ok = cur.valid && kk < cur.K && cur.boff != kOob;
          const int off = (int)(ok ? cur.boff + (unsigned)kk * 2u : kOob);
          if (cur.down) bbuf[t][h] = __builtin_amdgcn_raw_buffer_load_b128(rb, off, 0, kCoherentLd);
          else bbuf[t][h] = __builtin_amdgcn_raw_buffer_load_b128(rb, off, 0, 0);
        }
    };
    // The item after the current one is decoded as soon as the current one has started, and the
    // loads that look at its dependency are issued then: one item later, when it comes up, the
    // answer has long arrived (the wave's loads return in order) and is almost always "met".
    DItem nx = cur;
    bool nx_known = false;
    int look = 0;                     // this lane's shard of nx's dependency counter
    auto peek = [&]() {
      nx = decode_item<WB>(a, sm, vb + (j + 1) * G, total, n_groups, c, lane);
      nx_known = true;
      look = (nx.valid && nx.dep >= 0) ? shard_load(a.sync, nx.dep, lane) : 0;
    };
    // Blocks until the activations a down item contracts are complete.  One wave per workgroup
    // polls memory, the others watch its word in LDS.
    auto wait_dep = [&]() {
      if (!(cur.valid && cur.dep >= 0)) return;
      const bool ready = shard_sum(shard_load(a.sync, cur.dep, lane)) >= cur.dep_want;
      if (!ready) publish();          // the awaited activations may include the ones this wave has just stored
      if (c == 0) {
        if (!ready) shard_wait(a.sync, cur.dep, cur.dep_want, a.spin_limit, lane);
        if (lane == 0) __hip_atomic_store(&sm.dep_seq, j + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      } else if (!ready && lane == 0) {
        int spins = 0;
        while (__hip_atomic_load(&sm.dep_seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < j + 1) {
          __builtin_amdgcn_s_sleep(4);
          if (++spins > 64 * a.spin_limit) { atomicAdd(ctr(a.sync, kSyncErr), 1); break; }
        }
      }
      compiler_fence();
    };

    for (int s = 0;; ++s) {
      if (!block_done && s == s_star) { dispatch_block(); block_done = true; }
      if (!nx_known && cur.valid && (block_done || vb + (j + 1) * G < total_A)) peek();
      lds_barrier();                                          // "landed"
      MM_TRACE_IT(4, s);
      publish();
      bool stale = false, late = false;
      if (s >= 3 && cur.valid) {
        if (tw < cur.ntn) consume((s + 1) & (kStages - 1));
        if (++k == cur.nch) {                                 // item done: hand the partial sums over
#pragma unroll
          for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int v = 0; v < 4; ++v) s_red[c][rt][v][lane] = acc[rt][v];
          acc[0] = f32x4{0, 0, 0, 0}; acc[1] = f32x4{0, 0, 0, 0};
          f_r0 = cur.r0; f_n0 = cur.n0; f_m = cur.m; f_N = cur.N; f_ntn = cur.ntn; f_out = cur.out;
          f_down = cur.down; f_sig = cur.sig;
          f_sc[0] = sc[0]; f_sc[1] = sc[1];
          pending = 1;
          MM_TRACE(min(5 + 2 * j, 13));                       // item j consumed
          ++j; k = 0;
          stale = true;
          // The next item.  If nothing stands in its way (no dependency, or the early look found it
          // met), its first token rows go out here, in front of the barrier, as within an item.
          const bool had_look = nx_known;
          cur = nx_known ? nx : decode_item<WB>(a, sm, vb + j * G, total, n_groups, c, lane);
          nx_known = false;
          bool ready = cur.valid && cur.dep < 0;
          if (cur.valid && cur.dep >= 0 && had_look) ready = shard_sum(look) >= cur.dep_want;
          if (ready) {
            load_scales(cur);
            if (cur.dep >= 0 && c == 0 && lane == 0)
              __hip_atomic_store(&sm.dep_seq, j + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (tw < cur.ntn) load_token_rows(false);
          } else {
            late = cur.valid;
          }
        }
      }
      // token rows of the chunk consumed in the next iteration (same item)
      if (!stale && s >= 2 && cur.valid) {
        if (!started) { started = 1; load_scales(cur); wait_dep(); }
        if (tw < cur.ntn) load_token_rows(false);
      }
      lds_barrier();                                          // "free"; partial sums of an item that ended are complete
      if (pending) { pending = 0; epilogue(); }
      if (late) {
        // behind the epilogue above: the item may wait for activations this very workgroup has just stored
        load_scales(cur);
        wait_dep();
        if (tw < cur.ntn) load_token_rows(true);
      }
      if (stale) { started = 1; MM_TRACE(min(4 + 2 * j, 12)); }
      if (!cur.valid && block_done && s >= 2) break;
    }
    publish();
    publish();                        // ... and the old value of a bump the call above may have issued
  }

  // ---- the columns whose last y tile this workgroup stored: the final weighted sum ----
  __syncthreads();
  MM_TRACE(14);
  for (int wd = 0; wd < (a.H + 1023) / 1024; ++wd) {
    unsigned bits = sm.tile_bits[wd];
    while (bits) {
      const int tile = wd * 32 + __ffs((int)bits) - 1;
      bits &= bits - 1;
      sum_columns(a, sm, tile, wave, lane);
    }
  }

  // ---- the last workgroup to leave puts the counters back to zero ----
  __syncthreads();
  MM_TRACE(15);
  __shared__ int s_last;
  if (tid == 0) {
    compiler_fence();
    __builtin_amdgcn_s_waitcnt(0);
    // two levels, so that the G tickets do not all queue on one address
    const int sub = blockIdx.x & (kShards - 1);
    const int in_sub = (G - sub + kShards - 1) / kShards;    // workgroups b with b % kShards == sub
    s_last = 0;
    if (counter_bump(ctr(a.sync, kSyncExitSub + sub)) == in_sub - 1)
      s_last = counter_bump(ctr(a.sync, kSyncExit)) == min(G, kShards) - 1;
  }
  __syncthreads();
  if (s_last) {
    const int n_h = (a.n_slabs + a.E) * kShards, n_c = (a.H + 31) / 32;
    if (tid < kShards) coherent_store_i32(a.sync, (unsigned)(kSyncExitSub + tid) * 4u * kCtrStride, 0);
    for (int i = tid; i < n_h; i += kThreadsD) coherent_store_i32(a.sync, (unsigned)(kSyncHDone + i) * 4u * kCtrStride, 0);
    for (int i = tid; i < n_c; i += kThreadsD) coherent_store_i32(a.sync, (unsigned)(kSyncColDone + i) * 4u * kCtrStride, 0);
    if (tid < kDecodeMaxTokens) coherent_store_i32(a.sync, (unsigned)(kSyncToken + tid) * 4u * kCtrStride, 0);
    if (tid == 0) {
      coherent_store_i32(a.sync, kSyncRouteDone * 4u * kCtrStride, 0);
      coherent_store_i32(a.sync, kSyncExit * 4u * kCtrStride, 0);
    }
  }
}

__global__ void decode_sync_clear_kernel(int* sync) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < kSyncInts * kCtrStride; i += gridDim.x * blockDim.x) sync[i] = 0;
}

}  // namespace

#ifdef MOE_DECODE_TRACE
size_t decode_sync_bytes() { return align256(sizeof(int) * kSyncInts * kCtrStride + 8 * kTraceSlots * 4096); }
#else
size_t decode_sync_bytes() { return align256(sizeof(int) * kSyncInts * kCtrStride); }
#endif

template <int WB>
static int launch_decode_typed(DecodeArgs& a, hipStream_t s) {
  static std::atomic<int> per_cu_cached{0};
  int per_cu = per_cu_cached.load(std::memory_order_relaxed);
  if (per_cu == 0) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, decode_step_kernel<WB>, kThreadsD, 0) != hipSuccess || n < 1) n = 1;
    per_cu = n;
    per_cu_cached.store(n, std::memory_order_relaxed);
  }
  // persistent workgroups, all resident at once: the hand-overs inside the kernel rely on it
  const long grid = (long)device_cu_count() * per_cu;
  while (a.route_split > 1 && (long)a.T * a.route_split > grid) --a.route_split;
  if (grid < (long)a.T * a.route_split)
    return fail(MOE_E_UNSUPPORTED, "moe_layer_decode: %ld resident workgroups for %d tokens x %d router parts", grid, a.T, a.route_split);
  hipLaunchKernelGGL((decode_step_kernel<WB>), dim3((unsigned)grid), dim3(kThreadsD), 0, s, a);
  return hip_fail(hipGetLastError(), "decode_step_kernel launch");
}

int launch_decode_step(const moe_config& c, const DecodeLaunch& L, hipStream_t s) {
  DecodeArgs a = {};
  a.T = c.T; a.H = c.H; a.E = c.E; a.I = c.I; a.k_big = c.k_big; a.k_little = c.k_little; a.renorm = c.renorm;
  a.gamma = c.gamma;
  a.n_shared = c.n_shared;
  const SlabPlan plan = slab_plan(c);
  for (int i = 0; i < c.n_shared; ++i) {
    a.shared_I[i] = c.shared_I[i];
    a.shared_kchunk[i] = plan.kchunk[i];
    a.shared_w[i] = L.shared_w[i];
    a.h_shared[i] = L.h_shared[i];
  }
  a.n_slabs = plan.n_slabs;
  for (int i = 0; i < plan.n_slabs; ++i) { a.slab_shared[i] = plan.slab_shared[i]; a.slab_chunk[i] = plan.slab_chunk[i]; }
  a.expert_w = L.expert_w; a.x = L.x; a.Wg = L.Wg; a.bias = L.gate_bias; a.conf = L.conf;
  a.logits_given = L.logits_given;
  a.route_split = L.logits_given ? 1 : (c.E + 31) / 32;     // one pass of 8 waves x 4 experts per workgroup
  a.logits = L.logits; a.topk_idx = L.topk_idx; a.topk_w = L.topk_w;
  a.important = L.important; a.k_t = L.k_t; a.expert_offsets = L.expert_offsets;
  a.sorted_token = L.sorted_token; a.sorted_rank = L.sorted_rank; a.inv_pos = L.inv_pos;
  a.h_routed = L.h_routed; a.y = L.y; a.shared_out = L.shared_out; a.out = L.out;
  a.sync = static_cast<int*>(L.sync);
  a.spin_limit = L.spin_limit;
  if ((c.H + 31) / 32 > kMaxColTiles) return fail(MOE_E_UNSUPPORTED, "moe_layer_decode: H=%d above %d", c.H, 32 * kMaxColTiles);
  return c.dtype == MOE_BF16_W8 ? launch_decode_typed<1>(a, s) : launch_decode_typed<2>(a, s);
}

int launch_decode_sync_clear(void* sync, hipStream_t s) {
  hipLaunchKernelGGL(decode_sync_clear_kernel, dim3(64), dim3(256), 0, s, static_cast<int*>(sync));
  return hip_fail(hipGetLastError(), "decode_sync_clear_kernel launch");
}

int decode_sync_error_word() { return kSyncErr * kCtrStride; }

}  // namespace mm
