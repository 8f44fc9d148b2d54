// Device-side description of the groups of the grouped expert GEMMs (shared by the streaming
// and the tiled kernels): one group per routed expert, per shared expert (gate/up) or per K
// chunk of a shared expert (down), resolved from the kernel arguments and expert_offsets.
#pragma once

#include "internal.h"

namespace mm {
namespace {

constexpr int kMaxGroups = MOE_MAX_EXPERTS + kMaxSlabs;
constexpr unsigned kOob = 0x80000000u;   // offset no buffer reaches (every buffer is < 2 GiB)


__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  // wave-uniform by construction; readfirstlane tells the compiler so
  const uint64_t a = (uint64_t)p;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
  const unsigned n = __builtin_amdgcn_readfirstlane(bytes);
  return __builtin_amdgcn_make_buffer_rsrc((void*)(((uint64_t)hi << 32) | lo), 0, (int)n, 0x00020000);
}

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// One group of the grouped GEMM, fully resolved on the device (kept in LDS).
struct Group {
  int m;            // token rows
  int N;            // weight rows
  int K;            // contraction length of this group (a K chunk for split groups)
  int ldw;          // elements between weight rows = elements between B rows
  int row0;         // first dispatch position (routed), 0 otherwise
  int gather;       // 1: B row r is x[sorted_token[row0 + r]] (routed gate/up)
  unsigned wbytes;  // bytes readable from w0 (both matrices for gate/up)
  unsigned bbytes;  // bytes readable from b
  const void* w0;   // first weight matrix, already advanced to the K chunk
  const void* b;    // B rows, already advanced to the K chunk (and to row0 for routed kDown)
  void* out;        // h rows / y rows / slab base, already advanced to row0 where it applies
};

// Group order: shared experts (many tokens => heaviest items) first, then the routed experts.
template <typename S, int MODE>
__device__ __forceinline__ Group resolve_group(const StreamArgs& a, int g) {
  constexpr unsigned esz = sizeof(S);
  Group G;
  G.gather = 0; G.row0 = 0;
  if (MODE == kRouter) {
    G.m = a.T; G.N = a.E; G.K = a.H; G.ldw = a.H;
    G.w0 = a.Wg; G.b = a.x; G.out = a.logits;
    G.wbytes = (unsigned)a.E * a.H * esz; G.bbytes = (unsigned)a.T * a.H * esz;
    return G;
  }
  const int n_sh_groups = (MODE == kDown) ? a.n_slabs : a.n_shared;
  if (g < n_sh_groups) {
    int s = g, chunk = 0;
    if (MODE == kDown) { s = a.slab_shared[g]; chunk = a.slab_chunk[g]; }
    const int Is = a.shared_I[s];
    const S* blob = static_cast<const S*>(a.shared_w[s]);
    G.m = a.T;
    if (MODE == kGateUp) {
      G.N = Is; G.K = a.H; G.ldw = a.H;
      G.w0 = blob; G.b = a.x; G.out = a.h_shared[s];
      G.wbytes = 2u * Is * a.H * esz; G.bbytes = (unsigned)a.T * a.H * esz;
    } else {
      const int kb = chunk * a.shared_kchunk[s];
      G.N = a.H; G.K = min(a.shared_kchunk[s], Is - kb); G.ldw = Is;
      G.w0 = blob + 2 * (size_t)Is * a.H + kb;
      G.b = static_cast<const S*>(a.h_shared[s]) + kb;
      G.out = a.shared_out + (size_t)g * a.T * a.H;
      G.wbytes = ((unsigned)a.H * Is - kb) * esz; G.bbytes = ((unsigned)a.T * Is - kb) * esz;
    }
    return G;
  }
  const int e = g - n_sh_groups;
  const int b0 = clampi(a.offsets[e], 0, a.max_pairs);
  const int b1 = clampi(a.offsets[e + 1], b0, a.max_pairs);
  const S* blob = static_cast<const S*>(a.expert_w[e]);
  G.m = blob ? min(b1 - b0, a.T) : 0;
  G.row0 = b0;
  if (MODE == kGateUp) {
    G.N = a.I; G.K = a.H; G.ldw = a.H; G.gather = 1;
    G.w0 = blob; G.b = a.x;
    G.out = static_cast<S*>(a.h_routed) + (size_t)b0 * a.I;
    G.wbytes = 2u * a.I * a.H * esz; G.bbytes = (unsigned)a.T * a.H * esz;
  } else {
    G.N = a.H; G.K = a.I; G.ldw = a.I;
    G.w0 = blob + 2 * (size_t)a.I * a.H;
    G.b = static_cast<const S*>(a.h_routed) + (size_t)b0 * a.I;
    G.out = a.y + (size_t)b0 * a.H;
    G.wbytes = (unsigned)a.H * a.I * esz; G.bbytes = (unsigned)G.m * a.I * esz;
  }
  return G;
}


}  // namespace
}  // namespace mm
