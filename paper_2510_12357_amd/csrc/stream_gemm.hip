// Skinny grouped GEMM for the decode regime: D[r][n] = sum_k W[n][k] * B[r][k] with few rows r
// (tokens) per group and weights W that are read exactly once from HBM.
//
// Used three times per step (execution stage of Sec. II-A, router of the selection stage):
//   kRouter  logits = x Wg^T + bias
//   kGateUp  h = silu(W_gate x) * (W_up x)     (SwiGLU activation, stored in the storage dtype)
//   kDown    y = W_down h                       (fp32)
//
// Design for gfx950:
//   * The weight matrix is the MFMA "A" operand and goes from global memory straight into
//     registers: each lane fetches 16 contiguous bytes of one weight row, a wavefront covers
//     16 rows x 64 bytes per load instruction, and the waves of a workgroup interleave over
//     the K dimension so that a workgroup touches 16 rows x (NW*64) contiguous bytes at a time.
//     No weight element is needed by more than one wave, so LDS staging would only add traffic.
//   * Tokens are the "B" operand (up to 4 tiles of 16 tokens per work item); rows beyond the
//     group's token count are predicated off, so activation traffic follows the real m.
//   * The K split across waves is reduced through LDS, then the epilogue (SwiGLU / bias) runs
//     on the reduced tile.  Summation order is fixed => results are deterministic.
//   * Work items (group, row tile, token block) are enumerated on the device from
//     expert_offsets, so the host never learns the per-expert token counts; workgroups are
//     persistent and stride over the item list, which terminates after a bounded count.
#include "internal.h"

namespace mm {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kNW = 4;             // waves per workgroup (K interleave factor)
constexpr int kThreads = kNW * 64;
constexpr int kRT = 2;             // row tiles (16 rows each) per work item
constexpr int kNT = 4;             // token tiles (16 tokens each) per work item
constexpr int kMaxGroups = MOE_MAX_EXPERTS + MOE_MAX_SHARED;

// ---- element-type specifics -----------------------------------------------------------------
struct BF16 {
  typedef uint16_t storage;
  typedef bf16x8 frag;                       // 8 consecutive k
  static constexpr int kUnroll = 4;
  static __device__ __forceinline__ frag zero() { return frag{0, 0, 0, 0, 0, 0, 0, 0}; }
  static __device__ __forceinline__ frag load(const storage* p) {
    return *reinterpret_cast<const frag*>(p);
  }
  static __device__ __forceinline__ f32x4 mma(const frag& a, const frag& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ void store4(storage* p, float v0, float v1, float v2, float v3) {
    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
    bf16x4 o = {(__bf16)v0, (__bf16)v1, (__bf16)v2, (__bf16)v3};
    *reinterpret_cast<bf16x4*>(p) = o;
  }
};

struct FP32 {
  typedef float storage;
  struct frag { f32x4 lo, hi; };             // 8 consecutive k
  static constexpr int kUnroll = 2;
  static __device__ __forceinline__ frag zero() { return frag{{0, 0, 0, 0}, {0, 0, 0, 0}}; }
  static __device__ __forceinline__ frag load(const storage* p) {
    frag f;
    f.lo = *reinterpret_cast<const f32x4*>(p);
    f.hi = *reinterpret_cast<const f32x4*>(p + 4);
    return f;
  }
  // eight 16x16x4 fp32 MFMAs: instruction i contracts the i-th element of every lane's chunk,
  // which together cover the same 32 k values as one 16x16x32 bf16 instruction.
  static __device__ __forceinline__ f32x4 mma(const frag& a, const frag& b, f32x4 c) {
#pragma unroll
    for (int i = 0; i < 4; ++i) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.lo[i], b.lo[i], c, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.hi[i], b.hi[i], c, 0, 0, 0);
    return c;
  }
  static __device__ __forceinline__ void store4(storage* p, float v0, float v1, float v2, float v3) {
    *reinterpret_cast<f32x4*>(p) = f32x4{v0, v1, v2, v3};
  }
};

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// Description of one group of the grouped GEMM, resolved on the device.
template <typename ET>
struct Group {
  int m;                                 // token rows
  int N;                                 // weight rows
  int K;                                 // contraction length
  int row0;                              // first dispatch position (routed) or 0 (shared/router)
  const typename ET::storage* w0;        // first weight matrix  (gate / down / Wg)
  const typename ET::storage* w1;        // second weight matrix (up) for kGateUp
  int shared_idx;                        // -1 routed/router
};

template <typename ET, int MODE>
__device__ __forceinline__ Group<ET> resolve_group(const StreamArgs& a, int g) {
  typedef typename ET::storage S;
  Group<ET> G;
  G.shared_idx = -1;
  if (MODE == kRouter) {
    G.m = a.T; G.N = a.E; G.K = a.H; G.row0 = 0;
    G.w0 = static_cast<const S*>(a.Wg); G.w1 = nullptr;
    return G;
  }
  int Ig;
  const S* blob;
  if (g < a.n_routed) {
    const int b = clampi(a.offsets[g], 0, a.max_pairs);
    const int e = clampi(a.offsets[g + 1], b, a.max_pairs);
    blob = static_cast<const S*>(a.expert_w[g]);
    G.m = blob ? min(e - b, a.T) : 0;
    G.row0 = b;
    Ig = a.I;
  } else {
    const int s = g - a.n_routed;
    G.shared_idx = s;
    blob = static_cast<const S*>(a.shared_w[s]);
    G.m = a.T; G.row0 = 0;
    Ig = a.shared_I[s];
  }
  if (MODE == kGateUp) {
    G.N = Ig; G.K = a.H;
    G.w0 = blob; G.w1 = blob + (size_t)Ig * a.H;
  } else {
    G.N = a.H; G.K = Ig;
    G.w0 = blob + 2 * (size_t)Ig * a.H; G.w1 = nullptr;
  }
  return G;
}

template <int MODE>
__device__ __forceinline__ int rows_per_item() { return MODE == kGateUp ? 16 : 16 * kRT; }

template <typename ET, int MODE>
__global__ __launch_bounds__(kThreads) void stream_kernel(const StreamArgs a) {
  typedef typename ET::storage S;
  typedef typename ET::frag Frag;
  constexpr int U = ET::kUnroll;

  __shared__ int s_cnt[kMaxGroups];
  __shared__ int s_prefix[kMaxGroups + 1];
  __shared__ float s_red[kNW][kRT * kNT][4][64];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int q = lane >> 4, c16 = lane & 15;
  const int n_groups = (MODE == kRouter) ? 1 : a.n_routed + a.n_shared;

  // ---- item list: tiles per group, exclusive prefix (wave 0) ----
  for (int g = tid; g < n_groups; g += kThreads) {
    const Group<ET> G = resolve_group<ET, MODE>(a, g);
    const int rows = (G.N + rows_per_item<MODE>() - 1) / rows_per_item<MODE>();
    const int tgs = (G.m + 16 * kNT - 1) / (16 * kNT);
    s_cnt[g] = rows * tgs;
  }
  __syncthreads();
  if (wave == 0) {
    const int C = (n_groups + 63) / 64;
    const int base = lane * C;
    int sum = 0;
    for (int c = 0; c < C; ++c) if (base + c < n_groups) sum += s_cnt[base + c];
    int incl = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int v = __shfl_up(incl, d);
      if (lane >= d) incl += v;
    }
    int run = incl - sum;
    for (int c = 0; c < C; ++c) if (base + c < n_groups) { s_prefix[base + c] = run; run += s_cnt[base + c]; }
    if (lane == 63) s_prefix[n_groups] = incl;
  }
  __syncthreads();
  const int total = s_prefix[n_groups];

  for (int item = blockIdx.x; item < total; item += gridDim.x) {
    // group of this item: largest g with prefix[g] <= item < prefix[g+1]
    int lo = 0, hi = n_groups;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_prefix[mid] <= item) lo = mid; else hi = mid;
    }
    const int g = lo;
    const Group<ET> G = resolve_group<ET, MODE>(a, g);
    const int local = item - s_prefix[g];
    const int tgs = (G.m + 16 * kNT - 1) / (16 * kNT);
    const int row_item = local / tgs;
    const int r0 = (local - row_item * tgs) * (16 * kNT);
    const int n0 = row_item * rows_per_item<MODE>();
    const int ntn = min(kNT, (G.m - r0 + 15) >> 4);       // token tiles in use (wave-uniform)
    const int K = G.K;

    // ---- operand row pointers ----
    const S* Arow[kRT];
    bool Aval[kRT];
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt) {
      const int n = (MODE == kGateUp) ? n0 + c16 : n0 + rt * 16 + c16;
      const S* base = (MODE == kGateUp && rt == 1) ? G.w1 : G.w0;
      Aval[rt] = n < G.N;
      Arow[rt] = base + (size_t)n * K;
    }
    const S* Brow[kNT];
    bool Bval[kNT];
#pragma unroll
    for (int nt = 0; nt < kNT; ++nt) {
      const int r = r0 + nt * 16 + c16;
      Bval[nt] = r < G.m;
      size_t row = 0;
      if (Bval[nt]) {
        if (MODE == kGateUp && G.shared_idx < 0) row = (size_t)clampi(a.sorted_token[G.row0 + r], 0, a.T - 1);
        else row = (size_t)r;
      }
      const S* bbase;
      if (MODE == kDown)
        bbase = (G.shared_idx >= 0) ? static_cast<const S*>(a.h_shared[G.shared_idx])
                                    : static_cast<const S*>(a.h_routed) + (size_t)G.row0 * K;
      else
        bbase = static_cast<const S*>(a.x);
      Brow[nt] = bbase + row * K;
    }

    f32x4 acc[kRT][kNT];
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
      for (int nt = 0; nt < kNT; ++nt) acc[rt][nt] = f32x4{0, 0, 0, 0};

    // ---- K loop: the waves of the workgroup interleave over 32-wide k steps ----
    const int nks = (K + 31) >> 5;
    for (int ks = wave; ks < nks; ks += kNW * U) {
      Frag fa[U][kRT], fb[U][kNT];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int k0 = (ks + u * kNW) * 32 + q * 8;
        const bool kval = k0 < K;
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt) fa[u][rt] = (kval && Aval[rt]) ? ET::load(Arow[rt] + k0) : ET::zero();
#pragma unroll
        for (int nt = 0; nt < kNT; ++nt)
          if (nt < ntn) fb[u][nt] = (kval && Bval[nt]) ? ET::load(Brow[nt] + k0) : ET::zero();
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int nt = 0; nt < kNT; ++nt)
          if (nt < ntn) {
#pragma unroll
            for (int rt = 0; rt < kRT; ++rt) acc[rt][nt] = ET::mma(fa[u][rt], fb[u][nt], acc[rt][nt]);
          }
    }

    // ---- reduce the K split through LDS ----
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
      for (int nt = 0; nt < kNT; ++nt)
        if (nt < ntn) {
#pragma unroll
          for (int v = 0; v < 4; ++v) s_red[wave][rt * kNT + nt][v][lane] = acc[rt][nt][v];
        }
    __syncthreads();

    // ---- epilogue: wave w owns token tiles w, w+NW, ... ----
    for (int nt = wave; nt < ntn; nt += kNW) {
      float val[kRT][4];
#pragma unroll
      for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          float sum = 0.f;
#pragma unroll
          for (int w = 0; w < kNW; ++w) sum += s_red[w][rt * kNT + nt][v][lane];
          val[rt][v] = sum;
        }
      const int r = r0 + nt * 16 + c16;
      if (r < G.m) {
        if (MODE == kGateUp) {
          const int i = n0 + 4 * q;
          if (i < G.N) {
            float hv[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const float gte = val[0][v];
              hv[v] = gte / (1.f + __expf(-gte)) * val[1][v];
            }
            S* hbase = (G.shared_idx >= 0) ? static_cast<S*>(a.h_shared[G.shared_idx])
                                           : static_cast<S*>(a.h_routed) + (size_t)G.row0 * G.N;
            ET::store4(hbase + (size_t)r * G.N + i, hv[0], hv[1], hv[2], hv[3]);
          }
        } else if (MODE == kDown) {
          float* obase = (G.shared_idx >= 0) ? a.shared_out + (size_t)G.shared_idx * a.T * a.H
                                             : a.y + (size_t)G.row0 * a.H;
#pragma unroll
          for (int rt = 0; rt < kRT; ++rt) {
            const int c = n0 + rt * 16 + 4 * q;
            if (c < G.N)
              *reinterpret_cast<f32x4*>(obase + (size_t)r * a.H + c) =
                  f32x4{val[rt][0], val[rt][1], val[rt][2], val[rt][3]};
          }
        } else {  // kRouter
#pragma unroll
          for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const int n = n0 + rt * 16 + 4 * q + v;
              if (n < G.N) a.logits[(size_t)r * a.E + n] = val[rt][v] + (a.bias ? a.bias[n] : 0.f);
            }
        }
      }
    }
    __syncthreads();
  }
}

template <typename ET, int MODE>
int launch_typed(const StreamArgs& a, hipStream_t s) {
  // upper bound of the item count (the device computes the exact list)
  const long tg_all = (a.T + 16 * kNT - 1) / (16 * kNT);
  long items = 0;
  auto row_items = [](int n, int per) { return (long)((n + per - 1) / per); };
  if (MODE == kRouter) {
    items = row_items(a.E, 32) * tg_all;
  } else {
    const int per = (MODE == kGateUp) ? 16 : 32;
    // a routed expert holds at most T pairs, and all experts together at most T*k_big
    const long routed_rows = row_items(MODE == kGateUp ? a.I : a.H, per);
    const long pairs_blocks = (a.max_pairs + 16 * kNT - 1) / (16 * kNT) + a.n_routed;
    items += a.n_routed ? routed_rows * (pairs_blocks < a.n_routed * tg_all ? pairs_blocks : a.n_routed * tg_all) : 0;
    for (int sidx = 0; sidx < a.n_shared; ++sidx)
      items += row_items(MODE == kGateUp ? a.shared_I[sidx] : a.H, per) * tg_all;
  }
  if (items <= 0) return MOE_OK;
  long grid = (long)device_cu_count() * 4;
  if (grid > items) grid = items;
  hipLaunchKernelGGL((stream_kernel<ET, MODE>), dim3((unsigned)grid), dim3(kThreads), 0, s, a);
  return hip_fail(hipGetLastError(), "stream_kernel launch");
}

}  // namespace

int launch_stream(StreamMode mode, int dtype, const StreamArgs& a, hipStream_t s) {
  if (dtype == MOE_BF16) {
    switch (mode) {
      case kRouter: return launch_typed<BF16, kRouter>(a, s);
      case kGateUp: return launch_typed<BF16, kGateUp>(a, s);
      case kDown: return launch_typed<BF16, kDown>(a, s);
    }
  } else {
    switch (mode) {
      case kRouter: return launch_typed<FP32, kRouter>(a, s);
      case kGateUp: return launch_typed<FP32, kGateUp>(a, s);
      case kDown: return launch_typed<FP32, kDown>(a, s);
    }
  }
  return fail(MOE_E_BADARG, "bad stream mode/dtype");
}

}  // namespace mm
