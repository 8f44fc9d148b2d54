// Grouped expert GEMM for the prefill regime (many tokens per expert): LDS-tiled bf16 MFMA.
//
//   kGateUp  h[r][i] = silu(sum_k x[tok(r)][k] Wgate[i][k]) * (sum_k x[tok(r)][k] Wup[i][k])
//   kDown    y[r][c] = sum_i h[r][i] Wdown[c][i]
//
// Both are "NT" products (tokens and weight rows are both K-contiguous), so tokens are the MFMA
// A operand and weight rows the B operand, each read from LDS as 16-byte K chunks.
//
// Tiling for gfx950 (64-wide waves, v_mfma_f32_32x32x16_bf16):
//   * workgroup tile (Shape<WM,WN,TM,TN>): default 128 tokens x 128 weight rows, K chunk 64,
//     4 waves in a 2x2 grid, each wave 64 x 64 outputs = 2x2 MFMA tiles (64 accumulator
//     registers), two workgroups per CU.  (256 x 256 with 8 waves measured the same on a
//     compute-bound layer and worse on layers with ~150 tokens per expert.)  For gate/up the
//     weight rows of a tile are half rows of W_gate plus the same rows of W_up, arranged so
//     that a wave holds gate and up of the same outputs and applies SwiGLU in registers.
//   * global -> LDS goes through registers with raw buffer loads (token gather and all ragged
//     edges are offsets beyond the buffer: zeros, no branches); two register sets and two LDS
//     stages form a software pipeline in which requests, LDS writes and fragment reads are
//     spread between the MFMAs of a chunk (one barrier per chunk).
//   * LDS rows are padded by 16 bytes so that the rows a b128 fragment read touches fall
//     into different banks.
//   * tiles are enumerated on the device from expert_offsets (the host never sees the counts);
//     persistent workgroups; the tile list is cut into 8 contiguous ranges, one per XCD, and
//     the token tiles that share a weight panel are adjacent in the list, so a panel is fetched
//     from HBM once and re-read from that XCD's L2.
#include <stdlib.h>

#include "internal.h"
#include "groups.h"

namespace mm {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef uint16_t S;

#ifndef MOE_TILED_BK
#define MOE_TILED_BK 64
#endif
constexpr int BK = MOE_TILED_BK;   // K chunk
constexpr int LDK = BK + 8;        // padded LDS row, elements
constexpr int kCPR = BK / 8;       // 16-byte chunks per tile row

// WM x WN waves; each wave TM x TN MFMA tiles of 32 x 32.
template <int WM_, int WN_, int TM_, int TN_>
struct Shape {
  static constexpr int WM = WM_, WN = WN_, TM = TM_, TN = TN_;
  static constexpr int kThreads = WM * WN * 64;
  static constexpr int BM = WM * TM * 32;            // tokens per tile
  static constexpr int BNR = WN * TN * 32;           // weight rows per tile (gate/up: half + half)
  static constexpr int kRowsPerPass = kThreads / kCPR;
  static constexpr int kLoadsA = BM / kRowsPerPass;
  static constexpr int kLoadsB = BNR / kRowsPerPass;
  static_assert(BM % kRowsPerPass == 0 && BNR % kRowsPerPass == 0, "tile rows must divide evenly");
  static_assert(TN % 2 == 0, "gate/up needs an even number of column tiles per wave");
};

template <int MODE, typename SH>
__global__ __launch_bounds__(SH::kThreads) void tiled_kernel(const StreamArgs a) {
  constexpr int BM = SH::BM, BNR = SH::BNR, TM = SH::TM, TN = SH::TN;
  constexpr int kThreads = SH::kThreads, kRowsPerPass = SH::kRowsPerPass;
  constexpr int kLoadsA = SH::kLoadsA, kLoadsB = SH::kLoadsB;
  constexpr int kOutCols = (MODE == kGateUp) ? BNR / 2 : BNR;     // output columns per tile

  __shared__ int s_cnt[kMaxGroups];
  __shared__ int s_prefix[kMaxGroups + 1];
  extern __shared__ __attribute__((aligned(16))) S s_tiles[];      // As[2][BM*LDK] | Bs[2][BNR*LDK]
  S* const As = s_tiles;
  S* const Bs = s_tiles + 2 * BM * LDK;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / SH::WN, wn = wave % SH::WN;
  const int n_groups = a.n_routed + (MODE == kDown ? a.n_slabs : a.n_shared);

  // ---- tile list: tiles per group, exclusive prefix ----
  for (int g = tid; g < n_groups; g += kThreads) {
    const Group G = resolve_group<S, MODE>(a, g);
    s_cnt[g] = ((G.N + kOutCols - 1) / kOutCols) * ((G.m + BM - 1) / BM);
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

  // ---- XCD-aware walk: workgroup b runs on XCD b % 8; each XCD owns a contiguous range ----
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, nslots = gridDim.x >> 3;
  const int lo_t = (int)((long)total * xcd / 8), hi_t = (int)((long)total * (xcd + 1) / 8);

  // per-thread chunk of the global -> LDS copy: rows tid/kCPR + kRowsPerPass*p, column tid%kCPR
  const int ld_row = tid / kCPR, ld_kc = tid % kCPR;

  for (int tile = lo_t + slot; tile < hi_t; tile += nslots) {
    int lo = 0, hi = n_groups;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_prefix[mid] <= tile) lo = mid; else hi = mid;
    }
    const Group G = resolve_group<S, MODE>(a, lo);
    const int local = tile - s_prefix[lo];
    const int mt = (G.m + BM - 1) / BM;
    const int n_tile = local / mt;                         // token tiles of one weight panel adjacent
    const int m0 = (local - n_tile * mt) * BM;
    const int n0 = n_tile * kOutCols;
    const int K = G.K;

    const __amdgpu_buffer_rsrc_t ra = make_rsrc(G.b, G.bbytes);      // tokens
    const __amdgpu_buffer_rsrc_t rb = make_rsrc(G.w0, G.wbytes);     // weights
    unsigned aoff[kLoadsA], boff[kLoadsB];
#pragma unroll
    for (int p = 0; p < kLoadsA; ++p) {
      const int r = m0 + ld_row + kRowsPerPass * p;        // token row of the tile
      const bool val = r < G.m;
      int row = r;
      if (G.gather) row = val ? clampi(a.sorted_token[G.row0 + r], 0, a.T - 1) : 0;
      aoff[p] = val ? (unsigned)row * (unsigned)G.ldw * 2u : kOob;
    }
#pragma unroll
    for (int p = 0; p < kLoadsB; ++p) {
      // weight row of the tile: gate/up tiles hold BNR/2 rows of W_gate, then the same rows of W_up
      const int br = ld_row + kRowsPerPass * p;
      int n;
      unsigned extra = 0;
      if (MODE == kGateUp) {
        n = n0 + (br % (BNR / 2));
        if (br >= BNR / 2) extra = (unsigned)G.N * (unsigned)G.ldw * 2u;
      } else {
        n = n0 + br;
      }
      boff[p] = n < G.N ? (unsigned)n * (unsigned)G.ldw * 2u + extra : kOob;
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // Software pipeline of one wave.  Two register sets hold chunks on their way from global
    // memory: while chunk k is multiplied out of LDS stage k%2, chunk k+1 (requested one chunk
    // earlier) is written to the other stage and chunk k+2 is requested.  The requests are issued
    // during the first two of the four 16-wide k steps of a chunk, the LDS writes during the last
    // two, and the fragments of k step j+1 are read while step j is multiplied, so memory
    // instructions sit between the MFMAs instead of in phases of their own.  Chunks past the end
    // have offsets beyond the buffers and fetch nothing.
    i32x4 ga[2][kLoadsA], gb[2][kLoadsB];
    auto gload_a = [&](int set, int kt) {
      const int k0 = kt * BK + ld_kc * 8;
      const bool kval = k0 < K;
#pragma unroll
      for (int p = 0; p < kLoadsA; ++p)
        ga[set][p] = __builtin_amdgcn_raw_buffer_load_b128(ra, (int)(kval ? aoff[p] + (unsigned)k0 * 2u : kOob), 0, 0);
    };
    auto gload_b = [&](int set, int kt) {
      const int k0 = kt * BK + ld_kc * 8;
      const bool kval = k0 < K;
#pragma unroll
      for (int p = 0; p < kLoadsB; ++p)
        gb[set][p] = __builtin_amdgcn_raw_buffer_load_b128(rb, (int)(kval ? boff[p] + (unsigned)k0 * 2u : kOob), 0, 0);
    };
    auto lstore_a = [&](int set, int st) {
#pragma unroll
      for (int p = 0; p < kLoadsA; ++p)
        *reinterpret_cast<i32x4*>(&As[st * BM * LDK + (ld_row + kRowsPerPass * p) * LDK + ld_kc * 8]) = ga[set][p];
    };
    auto lstore_b = [&](int set, int st) {
#pragma unroll
      for (int p = 0; p < kLoadsB; ++p)
        *reinterpret_cast<i32x4*>(&Bs[st * BNR * LDK + (ld_row + kRowsPerPass * p) * LDK + ld_kc * 8]) = gb[set][p];
    };
    auto read_frags = [&](int st, int kk, bf16x8 (&fa)[TM], bf16x8 (&fb)[TN]) {
      const S* Ast = As + st * BM * LDK;
      const S* Bst = Bs + st * BNR * LDK;
      const int kcol = kk * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(&Ast[(wm * TM * 32 + i * 32 + (lane & 31)) * LDK + kcol]);
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        // gate/up: j < TN/2 gate rows, j >= TN/2 the matching up rows; down: TN column blocks
        const int brow = (MODE == kGateUp)
                             ? (j / (TN / 2)) * (BNR / 2) + wn * (TN / 2) * 32 + (j % (TN / 2)) * 32 + (lane & 31)
                             : wn * TN * 32 + j * 32 + (lane & 31);
        fb[j] = *reinterpret_cast<const bf16x8*>(&Bst[brow * LDK + kcol]);
      }
    };
    // one chunk: multiply LDS stage st, write register set set_st to the other stage, request
    // chunk kt_ld into register set set_ld
    auto half = [&](int st, int set_st, int set_ld, int kt_ld) {
      constexpr int KK = BK / 16;
      bf16x8 fa[2][TM], fb[2][TN];
      read_frags(st, 0, fa[0], fb[0]);
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        if (kk + 1 < KK) read_frags(st, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
        if (kk == 0) gload_a(set_ld, kt_ld);
        if (kk == 1 || KK == 1) gload_b(set_ld, kt_ld);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][i], fb[kk & 1][j], acc[i][j], 0, 0, 0);
        if (kk == KK - 2 || KK == 1) lstore_a(set_st, st ^ 1);
        if (kk == KK - 1) lstore_b(set_st, st ^ 1);
        __builtin_amdgcn_sched_barrier(0);                 // keep the steps apart; free order inside a step
      }
    };

    const int nk = (K + BK - 1) / BK;
    gload_a(0, 0); gload_b(0, 0);
    gload_a(1, 1); gload_b(1, 1);
    lstore_a(0, 0); lstore_b(0, 0);                        // waits for chunk 0 only
    __syncthreads();
    for (int kt = 0; kt < nk; kt += 2) {
      half(0, 1, 0, kt + 2);
      __syncthreads();
      half(1, 0, 1, kt + 3);                               // multiplies zeros when nk is odd
      __syncthreads();
    }

    // ---- epilogue: accumulator v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32 ----
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = m0 + wm * TM * 32 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (r >= G.m) continue;
        if (MODE == kGateUp) {
#pragma unroll
          for (int j = 0; j < TN / 2; ++j) {
            const int col = n0 + wn * (TN / 2) * 32 + j * 32 + (lane & 31);
            if (col < G.N) {
              const float gte = acc[i][j][v];
              const float hv = gte / (1.f + __expf(-gte)) * acc[i][j + TN / 2][v];
              const __bf16 o = (__bf16)hv;
              static_cast<S*>(G.out)[(size_t)r * G.N + col] = __builtin_bit_cast(uint16_t, o);
            }
          }
        } else {
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * TN * 32 + j * 32 + (lane & 31);
            if (col < G.N) static_cast<float*>(G.out)[(size_t)r * a.H + col] = acc[i][j][v];
          }
        }
      }
  }
}

template <int MODE, typename SH>
int launch_tiled_shape(const StreamArgs& a, hipStream_t s) {
  constexpr size_t kLds = 2 * (size_t)(SH::BM + SH::BNR) * LDK * sizeof(S);
  static int per_cu = 0;
  if (per_cu == 0) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&tiled_kernel<MODE, SH>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds) != hipSuccess)
      return hip_fail(hipGetLastError(), "tiled_kernel: LDS size attribute");
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, tiled_kernel<MODE, SH>, SH::kThreads, kLds) != hipSuccess || n < 1) n = 1;
    if (const char* env = getenv("MOE_TILED_WG_PER_CU")) { const int v = atoi(env); if (v > 0) n = v; }
    per_cu = n;
  }
  int grid = device_cu_count() * per_cu;
  grid = grid / 8 * 8;                                      // the XCD walk wants a multiple of 8
  if (grid < 8) grid = 8;
  hipLaunchKernelGGL((tiled_kernel<MODE, SH>), dim3((unsigned)grid), dim3(SH::kThreads), kLds, s, a);
  return hip_fail(hipGetLastError(), "tiled_kernel launch");
}

#ifndef MOE_TILED_SHAPE
#define MOE_TILED_SHAPE 2, 2, 2, 2
#endif
typedef Shape<MOE_TILED_SHAPE> DefaultShape;

}  // namespace

int launch_tiled(StreamMode mode, const StreamArgs& a, hipStream_t s) {
  if (mode == kGateUp) return launch_tiled_shape<kGateUp, DefaultShape>(a, s);
  if (mode == kDown) return launch_tiled_shape<kDown, DefaultShape>(a, s);
  return fail(MOE_E_BADARG, "tiled kernel: bad mode");
}

}  // namespace mm
