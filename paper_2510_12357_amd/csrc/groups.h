// Device-side description of the groups of the grouped expert GEMMs (shared by the streaming
// and the tiled kernels): one group per routed expert, per shared expert (gate/up) or per K
// chunk of a shared expert (down), resolved from the kernel arguments and expert_offsets.
#pragma once

#include "internal.h"

namespace mm {
namespace {

constexpr int kMaxGroups = MOE_MAX_EXPERTS + kMaxSlabs;
constexpr unsigned kOob = 0x80000000u;   // offset no buffer reaches (every buffer is < 2 GiB)
// cache policy of the decode kernels' weight loads ("nt"): a weight is read once per step, so its
// lines are the first to leave the caches again and the activations stay
constexpr int kStreamOnce = 2;


__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  // wave-uniform by construction; readfirstlane tells the compiler so
  const uint64_t a = (uint64_t)p;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
  const unsigned n = __builtin_amdgcn_readfirstlane(bytes);
  return __builtin_amdgcn_make_buffer_rsrc((void*)(((uint64_t)hi << 32) | lo), 0, (int)n, 0x00020000);
}

// Values that are the same in all lanes of a wave but come out of LDS or vector arithmetic:
// moving them to scalar registers frees vector registers.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ unsigned uniform(unsigned v) { return (unsigned)__builtin_amdgcn_readfirstlane((int)v); }
template <typename P>
__device__ __forceinline__ P* uniform(P* p) {
  const uint64_t v = (uint64_t)p;
  const uint64_t lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)v);
  const uint64_t hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(v >> 32));
  return (P*)((hi << 32) | lo);
}

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
// 8 E4M3 codes (two dwords, k ascending with the byte address) -> 8 bf16, exactly.
__device__ __forceinline__ bf16x8 widen_e4m3(int lo, int hi) {
  const auto a = __builtin_amdgcn_cvt_pk_f32_fp8(lo, false), b = __builtin_amdgcn_cvt_pk_f32_fp8(lo, true);
  const auto c = __builtin_amdgcn_cvt_pk_f32_fp8(hi, false), d = __builtin_amdgcn_cvt_pk_f32_fp8(hi, true);
  return bf16x8{(__bf16)a[0], (__bf16)a[1], (__bf16)b[0], (__bf16)b[1], (__bf16)c[0], (__bf16)c[1], (__bf16)d[0], (__bf16)d[1]};
}

// 8 E2M1 codes (one dword, k ascending with the nibble address) times the block scale (a power of
// two as fp32) -> 8 bf16, exactly while the products stay in bf16's range.
__device__ __forceinline__ bf16x8 widen_mx4(int codes, float scale) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4((unsigned)codes, scale, 0);
  const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4((unsigned)codes, scale, 1);
  const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4((unsigned)codes, scale, 2);
  const bf16x2 d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4((unsigned)codes, scale, 3);
  return bf16x8{a[0], a[1], b[0], b[1], c[0], c[1], d[0], d[1]};
}
// An E8M0 byte as fp32: 2^(b - 127); 0 is the subnormal 2^-127, 255 is NaN.
__device__ __forceinline__ float e8m0_to_f32(unsigned b) {
  return __uint_as_float(b == 0 ? 0x00400000u : (b == 255 ? 0x7fc00000u : b << 23));
}

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
  const void* scale;   // 8-bit weights: fp32 scale of weight row n at ((const float*)scale)[n] (gate/up:
                       // the up rows' scales follow at [N + n]).  MXFP4: E8M0 byte of weight row n and
                       // block j of this group's K at ((const uint8_t*)scale)[n * (ldw / 32) + j]
                       // (gate/up: the up rows follow as rows N + n).  Unused otherwise.
};

// What resolving a group has to read from memory; the rest of a Group follows from the kernel
// arguments alone.  A kernel that must not touch global memory while it walks its items (its
// loads are counted) keeps these three words per group and expands them on demand.
struct GroupSrc {
  int m;            // token rows (0 for a routed expert without weights)
  int row0;         // first dispatch position (routed), 0 otherwise
  const void* blob; // expert weights [W_gate | W_up | W_down]
};

// Group order: shared experts (many tokens => heaviest items) first, then the routed experts.
template <int MODE>
__device__ __forceinline__ GroupSrc load_group_src(const StreamArgs& a, int g) {
  GroupSrc s;
  s.row0 = 0;
  if (MODE == kRouter) { s.m = a.T; s.blob = a.Wg; return s; }
  const int n_sh_groups = (MODE == kDown) ? a.n_slabs : a.n_shared;
  if (g < n_sh_groups) {
    s.m = a.T;
    s.blob = a.shared_w[MODE == kDown ? a.slab_shared[g] : g];
    return s;
  }
  const int e = g - n_sh_groups;
  const int b0 = clampi(a.offsets[e], 0, a.max_pairs);
  const int b1 = clampi(a.offsets[e + 1], b0, a.max_pairs);
  s.blob = a.expert_w[e];
  s.m = s.blob ? min(b1 - b0, a.T) : 0;
  s.row0 = b0;
  return s;
}

// Bytes of n expert weights in format WB: WB bytes each, or half a byte for WB == 0 (MXFP4).
template <int WB>
__device__ __forceinline__ constexpr size_t w_bytes(size_t n) { return WB ? n * (size_t)WB : n / 2; }

// S: storage type of the activations (and of the router matrix); WB: format of the expert weights:
// bytes per weight (sizeof(S), or 1 for 8-bit codes with the fp32 row scales [gate | up | down]
// behind the three matrices of a blob), or 0 for MXFP4 (two codes per byte, the block scales
// [gate | up | down] behind the three matrices).  ldw counts elements for both the weight rows and
// the B rows.
template <typename S, int MODE, int WB = (int)sizeof(S)>
__device__ __forceinline__ Group make_group(const StreamArgs& a, int g, const GroupSrc& src) {
  constexpr unsigned esz = sizeof(S);
  Group G;
  G.gather = 0; G.row0 = src.row0; G.m = src.m; G.scale = nullptr;
  const char* blob = static_cast<const char*>(src.blob);
  if (MODE == kRouter) {
    G.N = a.E; G.K = a.H; G.ldw = a.H;
    G.w0 = a.Wg; G.b = a.x; G.out = a.logits;
    G.wbytes = (unsigned)a.E * a.H * esz; G.bbytes = (unsigned)a.T * a.H * esz;
    return G;
  }
  const int n_sh_groups = (MODE == kDown) ? a.n_slabs : a.n_shared;
  if (g < n_sh_groups) {
    int s = g, chunk = 0;
    if (MODE == kDown) { s = a.slab_shared[g]; chunk = a.slab_chunk[g]; }
    const int Is = a.shared_I[s];
    const char* scales = blob + w_bytes<WB>(3 * (size_t)Is * a.H);
    if (MODE == kGateUp) {
      G.N = Is; G.K = a.H; G.ldw = a.H;
      G.w0 = blob; G.b = a.x; G.out = a.h_shared[s];
      G.wbytes = (unsigned)w_bytes<WB>(2 * (size_t)Is * a.H); G.bbytes = (unsigned)a.T * a.H * esz;
      G.scale = scales;
    } else {
      const int kb = chunk * a.shared_kchunk[s];
      G.N = a.H; G.K = min(a.shared_kchunk[s], Is - kb); G.ldw = Is;
      G.w0 = blob + w_bytes<WB>(2 * (size_t)Is * a.H + kb);
      G.b = static_cast<const S*>(a.h_shared[s]) + kb;
      G.out = a.shared_out + (size_t)g * a.T * a.H;
      G.wbytes = (unsigned)w_bytes<WB>((size_t)a.H * Is - kb); G.bbytes = ((unsigned)a.T * Is - kb) * esz;
      // the down scales follow the 2 Is gate and up rows: Is floats each (8-bit), H / 32 bytes each (MXFP4)
      G.scale = WB ? scales + 4 * 2 * (size_t)Is : scales + 2 * (size_t)Is * (a.H / 32) + kb / 32;
    }
    return G;
  }
  const int b0 = src.row0;
  const char* scales = blob + w_bytes<WB>(3 * (size_t)a.I * a.H);
  if (MODE == kGateUp) {
    G.N = a.I; G.K = a.H; G.ldw = a.H; G.gather = 1;
    G.w0 = blob; G.b = a.x;
    G.out = static_cast<S*>(a.h_routed) + (size_t)b0 * a.I;
    G.wbytes = (unsigned)w_bytes<WB>(2 * (size_t)a.I * a.H); G.bbytes = (unsigned)a.T * a.H * esz;
    G.scale = scales;
  } else {
    G.N = a.H; G.K = a.I; G.ldw = a.I;
    G.w0 = blob + w_bytes<WB>(2 * (size_t)a.I * a.H);
    G.b = static_cast<const S*>(a.h_routed) + (size_t)b0 * a.I;
    G.out = a.y + (size_t)b0 * a.H;
    G.wbytes = (unsigned)w_bytes<WB>((size_t)a.H * a.I); G.bbytes = (unsigned)G.m * a.I * esz;
    G.scale = WB ? scales + 4 * 2 * (size_t)a.I : scales + 2 * (size_t)a.I * (a.H / 32);
  }
  return G;
}

template <typename S, int MODE>
__device__ __forceinline__ Group resolve_group(const StreamArgs& a, int g) {
  return make_group<S, MODE>(a, g, load_group_src<MODE>(a, g));
}

// Host side: upper bound of the number of work items of one grouped GEMM (the device computes
// the exact list); row_items rows per item, tok tokens per item.
inline long item_upper_bound(StreamMode mode, const StreamArgs& a, int tok) {
  auto row_items = [](int n, int per) { return (long)((n + per - 1) / per); };
  const long tg_all = (a.T + tok - 1) / tok;
  if (mode == kRouter) return row_items(a.E, 32) * ((a.T + 15) / 16);
  const int per = (mode == kGateUp) ? 16 : 32;
  long items = 0;
  // a routed expert holds at most T pairs, and all experts together at most T*k_big
  const long routed_rows = row_items(mode == kGateUp ? a.I : a.H, per);
  const long pairs_blocks = (a.max_pairs + tok - 1) / tok + a.n_routed;
  items += a.n_routed ? routed_rows * (pairs_blocks < a.n_routed * tg_all ? pairs_blocks : a.n_routed * tg_all) : 0;
  if (mode == kGateUp)
    for (int sidx = 0; sidx < a.n_shared; ++sidx) items += row_items(a.shared_I[sidx], per) * tg_all;
  else
    items += (long)a.n_slabs * row_items(a.H, per) * tg_all;
  return items;
}

}  // namespace
}  // namespace mm
