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
//   * All operand loads are raw buffer loads: a lane whose row, token or k chunk does not exist
//     gets an offset beyond the buffer's size, for which the hardware returns zeros without a
//     memory access.  The K loop is therefore straight-line code (no branches, no selects), and
//     activation traffic follows the real number of tokens.
//   * Loads run ahead of the MFMAs in a ring of registers (kDepth k-steps deep): every k-step
//     consumes the oldest ring entry and refills it with the load of the k-step kDepth ahead, so
//     a wave keeps a fixed number of bytes in flight.
//   * The K split across waves is reduced through LDS, then the epilogue (SwiGLU / bias) runs
//     on the reduced tile.  Summation order is fixed => results are deterministic.
//   * Work items (group, row tile, token block) are enumerated on the device from
//     expert_offsets, so the host never learns the per-expert token counts; workgroups are
//     persistent and stride over the item list, which terminates after a bounded count.  The
//     groups with many tokens (shared experts) come first in the list.
//   * A long contraction (down projection of a wide shared expert) is cut into K chunks that
//     become separate groups writing separate output slabs; the combine kernel adds the slabs
//     in a fixed order.
#include <atomic>

#include "internal.h"
#include "groups.h"

namespace mm {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int kRT = 2;             // row tiles (16 rows each) per work item
#ifndef MOE_STREAM_NT
#define MOE_STREAM_NT 4
#endif
constexpr int kNT = MOE_STREAM_NT; // token tiles (16 tokens each) per work item, at most
#ifndef MOE_STREAM_D1
#define MOE_STREAM_D1 4
#endif
#ifndef MOE_STREAM_D4
#define MOE_STREAM_D4 2
#endif

// ---- element-type specifics -----------------------------------------------------------------
struct BF16 {
  typedef uint16_t storage;
  typedef bf16x8 frag;                       // 8 consecutive k
  static constexpr int kWavesPerSimd = 3;        // register budget: three workgroups per CU
  static constexpr int kDepth1 = MOE_STREAM_D1;  // k-steps in flight with 1 token tile
  static constexpr int kDepth4 = MOE_STREAM_D4;  // ... with up to 4 token tiles
  static __device__ __forceinline__ frag load(__amdgpu_buffer_rsrc_t r, unsigned off) {
    const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
    return __builtin_bit_cast(frag, v);
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
  static constexpr int kWavesPerSimd = 2;
  static constexpr int kDepth1 = 4;
  static constexpr int kDepth4 = 2;
  static __device__ __forceinline__ frag load(__amdgpu_buffer_rsrc_t r, unsigned off) {
    frag f;
    f.lo = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0));
    f.hi = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)(off + 16u), 0, 0));
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

template <int MODE>
__device__ __forceinline__ int rows_per_item() { return MODE == kGateUp ? 16 : 16 * kRT; }
// tokens per work item: the router uses single token tiles (its weight matrix is tiny and stays
// in L2, so more and smaller items only add parallelism); the expert GEMMs reuse the streamed
// weights for up to kNT tiles
template <int MODE>
__device__ __forceinline__ int tokens_per_item() { return MODE == kRouter ? 16 : 16 * kNT; }

// What a wave needs of a work item to run its K loop.
struct Operands {
  const void* w; const void* b;       // buffers of the weight rows / token rows
  unsigned wbytes, bbytes;
  unsigned aoff[kRT], boff[kNT];      // byte offsets of this lane's rows at k = 0 (kOob: no such row);
                                      // boff[1..] only for the k loop with several token tiles
  int K;
};

// The ring of k-steps in flight is one pool of fragments, laid out per k-loop shape: entry d
// holds kRT weight fragments and NTI token fragments.  One pool serves both shapes, so that the
// ring that persists across items and the ring of the many-token items share registers.
template <int NTI, int DEPTH>
struct RingLayout {
  static constexpr int kSize = DEPTH * (kRT + NTI);
  static __device__ __forceinline__ constexpr int a(int d, int rt) { return d * kRT + rt; }
  static __device__ __forceinline__ constexpr int b(int d, int nt) { return DEPTH * kRT + d * NTI + nt; }
};

// Loads of k-step (wave + step * NW) of an item into ring entry d.
template <typename ET, int NTI, int DEPTH, int NW, typename POOL>
__device__ __forceinline__ void fill_step(POOL& pool, int d, const Operands& o, __amdgpu_buffer_rsrc_t ra_rsrc,
                                          __amdgpu_buffer_rsrc_t rb_rsrc, int step, int wave, int q) {
  typedef RingLayout<NTI, DEPTH> L;
  constexpr unsigned esz = sizeof(typename ET::storage);
  const int k0 = (wave + step * NW) * 32 + q * 8;
  const bool kval = k0 < o.K;
  const unsigned koff = (unsigned)k0 * esz;                 // kOob + koff stays out of range
#pragma unroll
  for (int rt = 0; rt < kRT; ++rt) pool[L::a(d, rt)] = ET::load(ra_rsrc, kval ? o.aoff[rt] + koff : kOob);
#pragma unroll
  for (int nt = 0; nt < NTI; ++nt) pool[L::b(d, nt)] = ET::load(rb_rsrc, kval ? o.boff[nt] + koff : kOob);
}

// K loop of one work item for one wave: k-steps ks = wave, wave + NW, ...  (32 k each).
// The ring (ra, rb) lives outside: when `primed`, it already holds the first DEPTH k-steps of this
// item, loaded while the previous item was finishing; when `chain`, the last DEPTH refills fetch
// the first k-steps of the next item instead of nothing, so that the loads never pause at an
// item boundary (epilogue, reduction and item set-up run under them).
template <typename ET, int NTI, int DEPTH, int NW, typename POOL>
__device__ __forceinline__ void k_loop(f32x4 (&acc)[kRT][kNT], POOL& pool, const Operands& cur,
                                       const Operands& nxt, bool primed, bool chain, int wave, int q) {
  typedef RingLayout<NTI, DEPTH> L;
  const __amdgpu_buffer_rsrc_t ca = make_rsrc(cur.w, cur.wbytes), cb = make_rsrc(cur.b, cur.bbytes);
  const int nks = (cur.K + 31) >> 5;
  const int nsteps = (nks + NW - 1) / NW;                   // same for every wave of the workgroup
  if (!primed) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) fill_step<ET, NTI, DEPTH, NW>(pool, d, cur, ca, cb, d, wave, q);
  }
  auto consume = [&](int d) {
#pragma unroll
    for (int nt = 0; nt < NTI; ++nt)
#pragma unroll
      for (int rt = 0; rt < kRT; ++rt) acc[rt][nt] = ET::mma(pool[L::a(d, rt)], pool[L::b(d, nt)], acc[rt][nt]);
  };
  int i = 0;
  for (; i + DEPTH < nsteps; i += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      consume(d);
      fill_step<ET, NTI, DEPTH, NW>(pool, d, cur, ca, cb, i + d + DEPTH, wave, q);   // k-steps past the end fetch nothing
      // keep the per-step order (consume oldest, refill it): without this the scheduler hoists
      // all MFMAs above all loads and the ring degenerates into load-all / wait-all / compute-all
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // last DEPTH k-steps of this item
  if (chain) {
    const __amdgpu_buffer_rsrc_t na = make_rsrc(nxt.w, nxt.wbytes), nb = make_rsrc(nxt.b, nxt.bbytes);
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      consume(d);
      fill_step<ET, NTI, DEPTH, NW>(pool, d, nxt, na, nb, d, wave, q);
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) consume(d);
  }
}

// NW = waves of a workgroup that split the K dimension of one work item.
template <typename ET, int MODE, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(ET::kWavesPerSimd, ET::kWavesPerSimd))) void stream_kernel(const StreamArgs a) {
  typedef typename ET::storage S;
  typedef typename ET::frag Frag;
  constexpr int kThreads = NW * 64;
  constexpr unsigned esz = sizeof(S);

  __shared__ int s_cnt[kMaxGroups];
  __shared__ int s_prefix[kMaxGroups + 1];
  __shared__ Group s_group[kMaxGroups];
  __shared__ float s_red[NW][kRT * kNT][4][64];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int q = lane >> 4, c16 = lane & 15;
  const int n_groups = (MODE == kRouter) ? 1 : a.n_routed + (MODE == kDown ? a.n_slabs : a.n_shared);

  // ---- group table and item list: tiles per group, exclusive prefix (wave 0) ----
  for (int g = tid; g < n_groups; g += kThreads) {
    const Group G = resolve_group<typename ET::storage, MODE>(a, g);
    const int rows = (G.N + rows_per_item<MODE>() - 1) / rows_per_item<MODE>();
    const int tgs = (G.m + tokens_per_item<MODE>() - 1) / tokens_per_item<MODE>();
    s_group[g] = G;
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

  // One work item, resolved for this lane.
  struct Item {
    int valid, g, r0, n0, ntn, K;
    const void* w; const void* b;
    unsigned wbytes, bbytes, aoff[kRT], boff0;
  };
  // byte offset of token row (r0 + nt * 16 + c16) of group G, kOob if this lane has no such row
  auto token_offset = [&](const Group& G, int valid, int r0, int ntn, int nt) -> unsigned {
    const int r = r0 + nt * 16 + c16;
    const bool val = valid && nt < ntn && r < G.m;
    int row = r;
    if (G.gather) row = val ? clampi(a.sorted_token[G.row0 + r], 0, a.T - 1) : 0;
    return val ? (unsigned)row * (unsigned)G.ldw * esz : kOob;
  };
  auto operands = [&](const Item& it) -> Operands {
    Operands o;
    o.w = it.w; o.b = it.b; o.wbytes = it.wbytes; o.bbytes = it.bbytes; o.K = it.K;
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt) o.aoff[rt] = it.aoff[rt];
    o.boff[0] = it.boff0;
#pragma unroll
    for (int nt = 1; nt < kNT; ++nt) o.boff[nt] = kOob;
    return o;
  };
  auto decode = [&](int item) -> Item {
    Item it;
    it.valid = item < total;
    // group of this item: largest g with prefix[g] <= item < prefix[g+1]
    int lo = 0, hi = n_groups;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_prefix[mid] <= item) lo = mid; else hi = mid;
    }
    it.g = uniform(it.valid ? lo : 0);
    Group G = s_group[it.g];
    G.m = uniform(G.m); G.N = uniform(G.N); G.K = uniform(G.K); G.ldw = uniform(G.ldw); G.row0 = uniform(G.row0);
    G.gather = uniform(G.gather); G.wbytes = uniform(G.wbytes); G.bbytes = uniform(G.bbytes);
    G.w0 = uniform(G.w0); G.b = uniform(G.b);
    const int local = item - uniform(s_prefix[it.g]);
    const int tgs = max(1, (G.m + tokens_per_item<MODE>() - 1) / tokens_per_item<MODE>());
    const int row_item = local / tgs;
    it.r0 = (local - row_item * tgs) * tokens_per_item<MODE>();
    it.n0 = row_item * rows_per_item<MODE>();
    it.ntn = (MODE == kRouter) ? 1 : clampi((G.m - it.r0 + 15) >> 4, 1, kNT);   // token tiles in use (wave-uniform)
    // an item past the end of the list keeps valid pointers and empty buffers
    it.w = it.valid ? G.w0 : a.x; it.b = it.valid ? G.b : a.x;
    it.wbytes = it.valid ? G.wbytes : 0u; it.bbytes = it.valid ? G.bbytes : 0u;
    it.K = it.valid ? G.K : 0;
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt) {
      const int n = (MODE == kGateUp) ? it.n0 + c16 : it.n0 + rt * 16 + c16;
      unsigned off = (unsigned)n * (unsigned)G.ldw * esz;
      if (MODE == kGateUp && rt == 1) off += (unsigned)G.N * (unsigned)G.ldw * esz;   // W_up follows W_gate
      it.aoff[rt] = (it.valid && n < G.N) ? off : kOob;
    }
    it.boff0 = token_offset(G, it.valid, it.r0, it.ntn, 0);
    return it;
  };

  // the ring; for items with one token tile it persists across items (see k_loop)
  constexpr int kPool1 = RingLayout<1, ET::kDepth1>::kSize, kPool4 = RingLayout<kNT, ET::kDepth4>::kSize;
  Frag pool[kPool1 > kPool4 ? kPool1 : kPool4];
  bool primed = false;

  // Workgroups stride over the list: at any time the resident workgroups read neighbouring
  // row tiles, i.e. one window of a few dozen MB that sweeps through the weights (measured
  // faster than giving each workgroup its own contiguous range).
  Item cur = decode(blockIdx.x);
  for (int item = blockIdx.x; item < total; item += gridDim.x) {
    const Item nxt = decode(item + gridDim.x);
    Group G = s_group[cur.g];
    G.m = uniform(G.m); G.N = uniform(G.N); G.ldw = uniform(G.ldw); G.row0 = uniform(G.row0);
    G.gather = uniform(G.gather); G.out = uniform(G.out);
    const int r0 = cur.r0, n0 = cur.n0, ntn = cur.ntn;

    f32x4 acc[kRT][kNT];
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
      for (int nt = 0; nt < kNT; ++nt) acc[rt][nt] = f32x4{0, 0, 0, 0};

    if (ntn == 1 || kNT == 1) {
      const bool chain = nxt.valid && (nxt.ntn == 1 || kNT == 1);
      k_loop<ET, 1, ET::kDepth1, NW>(acc, pool, operands(cur), operands(nxt), primed, chain, wave, q);
      primed = chain;
    } else {
      Operands o = operands(cur);
#pragma unroll
      for (int nt = 1; nt < kNT; ++nt) o.boff[nt] = token_offset(G, 1, r0, ntn, nt);
      k_loop<ET, kNT, ET::kDepth4, NW>(acc, pool, o, o, false, false, wave, q);
      primed = false;
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
    for (int nt = wave; nt < ntn; nt += NW) {
      float val[kRT][4];
#pragma unroll
      for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          float sum = 0.f;
#pragma unroll
          for (int w = 0; w < NW; ++w) sum += s_red[w][rt * kNT + nt][v][lane];
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
            ET::store4(static_cast<S*>(G.out) + (size_t)r * G.N + i, hv[0], hv[1], hv[2], hv[3]);
          }
        } else if (MODE == kDown) {
#pragma unroll
          for (int rt = 0; rt < kRT; ++rt) {
            const int c = n0 + rt * 16 + 4 * q;
            if (c < G.N)
              *reinterpret_cast<f32x4*>(static_cast<float*>(G.out) + (size_t)r * a.H + c) =
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
    cur = nxt;
  }
}

template <typename ET, int MODE, int NW>
int launch_typed(const StreamArgs& a, hipStream_t s) {
  constexpr int kThreads = NW * 64;
  const long items = item_upper_bound((StreamMode)MODE, a, MODE == kRouter ? 16 : 16 * kNT);
  if (items <= 0) return MOE_OK;
  // persistent workgroups: exactly as many as are resident at once, so that the static striding
  // over the item list never leaves a second, partially filled round of workgroups
  static std::atomic<int> cached{0};
  int per_cu = cached.load(std::memory_order_relaxed);
  if (per_cu == 0) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, stream_kernel<ET, MODE, NW>, kThreads, 0) != hipSuccess || n < 1) n = 2;
    per_cu = n;
    cached.store(n, std::memory_order_relaxed);
  }
  long grid = (long)device_cu_count() * per_cu;
  if (grid > items) grid = items;
  hipLaunchKernelGGL((stream_kernel<ET, MODE, NW>), dim3((unsigned)grid), dim3(kThreads), 0, s, a);
  return hip_fail(hipGetLastError(), "stream_kernel launch");
}

}  // namespace

int launch_stream(StreamMode mode, int dtype, const StreamArgs& a, hipStream_t s) {
  if (dtype == MOE_BF16_W8 || dtype == MOE_BF16_MXFP4) {
    // the router matrix of such a layer is bf16; its expert weights exist for the LDS kernel only
    if (mode == kRouter) return launch_typed<BF16, kRouter, 4>(a, s);
    return launch_stream_lds(mode, dtype == MOE_BF16_W8 ? 1 : 0, a, s);
  }
  if (dtype == MOE_BF16) {
    // the bf16 expert GEMMs stream through LDS (stream_lds.hip); this file's kernel serves the
    // router GEMM and the fp32 layers
    if (mode != kRouter) return launch_stream_lds(mode, 2, a, s);
    return launch_typed<BF16, kRouter, 4>(a, s);
  } else {
    switch (mode) {
      case kRouter: return launch_typed<FP32, kRouter, 4>(a, s);
      case kGateUp: return launch_typed<FP32, kGateUp, 4>(a, s);
      case kDown: return launch_typed<FP32, kDown, 4>(a, s);
    }
  }
  return fail(MOE_E_BADARG, "bad stream mode/dtype");
}

}  // namespace mm
