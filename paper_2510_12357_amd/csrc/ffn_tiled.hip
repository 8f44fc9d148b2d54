// Grouped expert GEMM for the prefill regime (many tokens per expert): LDS-tiled bf16 MFMA.
//
//   kGateUp  h[r][i] = silu(sum_k x[tok(r)][k] Wgate[i][k]) * (sum_k x[tok(r)][k] Wup[i][k])
//   kDown    y[r][c] = sum_i h[r][i] Wdown[c][i]
//
// Both are "NT" products (tokens and weight rows are both K-contiguous), so tokens are the MFMA
// A operand and weight rows the B operand, each read from LDS as 16-byte K chunks.
//
// Tiling for gfx950 (64-wide waves, v_mfma_f32_32x32x16_bf16):
//   * workgroup tile (Shape<WM,WN,TM,TN>): default 128 tokens x 256 weight rows, K chunk 64,
//     one workgroup per CU.  Waves 0..3 compute, in a 2x2 grid, each 64 x 128 outputs = 2x4 MFMA
//     tiles (128 accumulator registers, 6 fragment reads per 8 MFMAs); waves 4..7 only load, so a
//     full vector-memory queue never stops the MFMA issue.  For gate/up the weight rows of a
//     tile are half rows of W_gate plus the same rows of W_up, arranged so that a wave holds
//     gate and up of the same outputs and applies SwiGLU in registers.
//   * global -> LDS without registers: buffer loads with the LDS destination move 8 tile rows x
//     128 bytes per instruction (token gather and all ragged edges are offsets beyond the
//     buffer: zero fill, no branches).  A ring of stages; a loader issues the chunk that is
//     (stages - 1) ahead, waits with a counted s_waitcnt vmcnt until its share of the next chunk
//     has landed, and joins the one barrier per chunk.  The loaders start the next tile while
//     the computing waves store the epilogue.
//   * a tile row is 128 bytes in LDS; the 16-byte column c of row r sits at column
//     c ^ ((r >> 1) & 7), which spreads the 16 rows that a b128 fragment read touches in one
//     pass over all banks.
//   * tiles are enumerated on the device from expert_offsets (the host never sees the counts);
//     persistent workgroups; the tile list is cut into 8 contiguous ranges, one per XCD, and
//     the token tiles that share a weight panel are adjacent in the list, so a panel is fetched
//     from HBM once and re-read from that XCD's L2.
//   * 8-bit weights (WB = 1: E4M3 codes with one fp32 scale per weight row): the weight rows of a
//     tile are 64 bytes in LDS (half the loads and half the LDS of a bf16 panel), 16 rows per load
//     instruction, swizzled with the key (row >> 2) & 3 so that a 16-byte fragment read of 16 rows
//     hits every bank once.  One such read holds a lane's codes of two k-steps, so the k order
//     inside a chunk is permuted: k-step 2p + e takes, for the lanes of half h, the 8 k behind
//     32 p + 16 h + 8 e, and the token fragments are read with the same permutation.  A computing
//     wave widens the codes of the next k-step to bf16 (exact) between the MFMAs of the current one,
//     and the row scale multiplies the fp32 sum in the epilogue.  Tokens, tile shape, pipeline and
//     tile order are those of the bf16 kernel.
//   * MXFP4 weights (WB = 0: 4-bit E2M1 codes, one E8M0 scale per 32 k): a weight tile row is 32
//     bytes (32 rows per load instruction, key (row >> 3) & 1).  The 16 bytes a lane reads per
//     column tile and chunk are the 32 codes of ONE scale block, i.e. of all four k-steps of the
//     chunk: k-step e takes, in the lanes of half h, the 8 k behind 32 h + 8 e.  The lane fetches
//     that block's scale byte itself, one chunk ahead, with a byte load (4 per lane and chunk),
//     and code x scale is widened to bf16 in one instruction per two codes (exact).
#include <atomic>
#include <type_traits>

#include "internal.h"
#include "groups.h"

namespace mm {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) void lds_void;
typedef uint16_t S;

#ifndef MOE_TILED_BK
#define MOE_TILED_BK 64
#endif
#ifndef MOE_TILED_STAGES
#define MOE_TILED_STAGES 3
#endif
constexpr int BK = MOE_TILED_BK;   // K chunk, elements (32 or 64)
constexpr int kRowB = BK * 2;      // bytes of a tile row in LDS
constexpr int kStages = MOE_TILED_STAGES;
constexpr int kCols = BK / 8;                  // 16-byte columns of a tile row
constexpr int kRowsPerIns = 1024 / kRowB;      // tile rows that one load instruction fills
constexpr int kKeyShift = BK == 64 ? 1 : 2;    // rows per 256 bytes of LDS = 1 << kKeyShift
static_assert(BK == 32 || BK == 64, "K chunk of 32 or 64");
static_assert(MOE_TILED_STAGES >= 3, "the pipeline needs at least three stages");
// swizzle key of a tile row: rows that share 256 bytes of LDS get the same key, the next ones the next
__device__ __forceinline__ constexpr int row_key(int row) { return (row >> kKeyShift) & (kCols - 1); }

// Weight rows of a tile in LDS, by weight format (WB bytes per weight).
template <int WB>
struct WFmt {
  static_assert(WB == 0 || WB == 1 || WB == 2, "bf16, 8-bit or MXFP4 weights");
  static constexpr int kRowB = WB ? BK * WB : BK / 2;   // bytes of a weight tile row
  static constexpr int kCols = kRowB / 16;           // its 16-byte columns
  static constexpr int kRowsPerIns = 1024 / kRowB;   // tile rows that one load instruction fills
  static constexpr int kPerCol = WB ? 16 / WB : 32;  // weights per 16-byte column
  static constexpr int kStepsPerRead = WB == 2 ? 1 : (WB == 1 ? 2 : 4);   // MFMA k-steps fed by one 16-byte fragment read
  static_assert(WB != 0 || BK == 64, "MXFP4: a chunk is two scale blocks");
  // 64-byte rows: four rows share 256 bytes of LDS, and 16 consecutive rows get every key once per
  // residue of the row number mod 4; 32-byte rows: eight rows share 256 bytes
  static __device__ __forceinline__ constexpr int key(int row) {
    return WB == 2 ? row_key(row) : (WB == 1 ? (row >> 2) & 3 : (row >> 3) & 1);
  }
  static __device__ __forceinline__ constexpr unsigned bytes(unsigned n) { return WB ? n * (unsigned)WB : n / 2u; }
};

// vmcnt(n): bits [3:0] and [15:14]; expcnt and lgkmcnt left at their maxima (no wait)
#define MM_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0f70 | ((n) & 15) | (((n) >> 4) << 14))

// Workgroup barrier that orders LDS accesses only (no global-memory fence: that would make the
// compiler wait for every outstanding load).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Two fragment reads off one address register.  The compiler does not see them as LDS accesses,
// so it neither waits for the loads-to-LDS in flight nor for these; frag_wait() does the latter.
template <int OFF0, int OFF1>
__device__ __forceinline__ void frag_read2(bf16x8& f0, bf16x8& f1, unsigned addr) {
  asm volatile("ds_read_b128 %0, %2 offset:%3\n\tds_read_b128 %1, %2 offset:%4"
               : "=&v"(f0), "=&v"(f1) : "v"(addr), "n"(OFF0), "n"(OFF1) : "memory");
}
template <int OFF0>
__device__ __forceinline__ void frag_read1(bf16x8& f0, unsigned addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(f0) : "v"(addr), "n"(OFF0) : "memory");
}
template <int N>
__device__ __forceinline__ void frag_wait(bf16x8 (&f)[N]) {
  static_assert(N == 2 || N == 4, "fragment sets of 2 or 4");
  if constexpr (N == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]) :: "memory");
  else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) :: "memory");
}

#ifndef MOE_TILED_ATTR
#define MOE_TILED_ATTR
#endif

// WM x WN waves; each wave TM x TN MFMA tiles of 32 x 32.
template <int WM_, int WN_, int TM_, int TN_>
struct Shape {
  static constexpr int WM = WM_, WN = WN_, TM = TM_, TN = TN_;
  static constexpr int kWaves = WM * WN;              // computing waves, and as many loader waves
  static constexpr int kThreads = 2 * kWaves * 64;
  static constexpr int BM = WM * TM * 32;            // tokens per tile
  static constexpr int BNR = WN * TN * 32;           // weight rows per tile (gate/up: half + half)
  static constexpr int kInsA = BM / kRowsPerIns / kWaves;      // token-row load instructions per wave and chunk
  template <int WB> static constexpr int ins_b() { return BNR / WFmt<WB>::kRowsPerIns / kWaves; }   // weight-row ones
  template <int WB> static constexpr int stage_bytes() { return BM * kRowB + BNR * WFmt<WB>::kRowB; }
  static_assert(BM % (kRowsPerIns * kWaves) == 0 && BNR % (32 * kWaves) == 0, "tile rows must divide evenly");
  static_assert((TM == 2 || TM == 4) && (TN == 2 || TN == 4), "the fragment reads are written for 2 or 4 MFMA tiles per wave and side");
};

template <int MODE, typename SH, int WB>
__global__ __launch_bounds__(SH::kThreads) MOE_TILED_ATTR void tiled_kernel(const StreamArgs a) {
  typedef WFmt<WB> WF;
  constexpr int BM = SH::BM, BNR = SH::BNR, TM = SH::TM, TN = SH::TN;
  constexpr int kThreads = SH::kThreads, kInsA = SH::kInsA, kInsB = SH::template ins_b<WB>();
  constexpr int kStageBytes = SH::template stage_bytes<WB>();
  constexpr int kRowBW = WF::kRowB;                                // bytes of a weight tile row
  constexpr int kPerChunk = kInsA + kInsB;                         // loads of one wave per chunk
  constexpr int kOutCols = (MODE == kGateUp) ? BNR / 2 : BNR;     // output columns per tile

  __shared__ int s_cnt[kMaxGroups];
  __shared__ int s_prefix[kMaxGroups + 1];
  extern __shared__ __attribute__((aligned(1024))) char s_tiles[];   // kStages x (A rows | B rows)

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool loader = wave >= SH::kWaves;                          // waves kWaves.. only move data
  const int lw = wave - SH::kWaves;                                // index among the loaders
  const int wm = (wave % SH::kWaves) / SH::WN, wn = wave % SH::WN;
  constexpr int kAhead = kStages - 1;                              // chunks in flight ahead of the one consumed
  const int n_groups = a.n_routed + (MODE == kDown ? a.n_slabs : a.n_shared);

  // ---- tile list: tiles per group, exclusive prefix ----
  for (int g = tid; g < n_groups; g += kThreads) {
    const Group G = make_group<S, MODE, WB>(a, g, load_group_src<MODE>(a, g));
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

  // ---- per-lane constants of the loads: instruction p of this wave fills tile rows
  // kRowsPerIns * (lw * kIns + p) + lane / kCols at physical column lane % kCols ----
  const int ld_sub = lane / kCols, ld_pc = lane % kCols;
  const int ld_subw = lane / WF::kCols, ld_pcw = lane % WF::kCols;   // the same for weight rows
  // ---- per-lane constants of the fragment reads: row (lane & 31) of a 32-row block, logical
  // column 2 * kk + lane / 32; every block starts at a multiple of 32 rows, so the swizzle key
  // of the row depends on the lane only ----
  const unsigned lds0 = (unsigned)(size_t)s_tiles;
  const unsigned fkey = (unsigned)row_key(lane & 31);
  const unsigned fkeyw = (unsigned)WF::key(lane & 31);
  const unsigned a_rd = lds0 + (unsigned)((wm * TM * 32 + (lane & 31)) * kRowB);
  const unsigned b_rd = lds0 + (unsigned)(BM * kRowB) +
                        (unsigned)(((MODE == kGateUp ? wn * (TN / 2) * 32 : wn * TN * 32) + (lane & 31)) * kRowBW);
  // byte distance between the fragment rows of consecutive token blocks i / column tiles j
  constexpr int kJ = 32 * kRowB;                                   // next 32 token rows
  constexpr int kJw = 32 * kRowBW;                                 // next 32 weight rows
  constexpr int kUp = (MODE == kGateUp) ? (BNR / 2) * kRowBW : (TN / 2) * kJw;   // j >= TN/2: the up rows / the next blocks

  for (int tile = lo_t + slot; tile < hi_t; tile += nslots) {
    int lo = 0, hi = n_groups;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_prefix[mid] <= tile) lo = mid; else hi = mid;
    }
    const Group G = make_group<S, MODE, WB>(a, lo, load_group_src<MODE>(a, lo));
    const int local = tile - s_prefix[lo];
    const int mt = (G.m + BM - 1) / BM;
    const int n_tile = local / mt;                         // token tiles of one weight panel adjacent
    const int m0 = (local - n_tile * mt) * BM;
    const int n0 = n_tile * kOutCols;
    const int K = G.K;

    const int nk = (K + BK - 1) / BK;

    if (loader) {
      // ================= loader waves: nothing but loads into LDS, waits and barriers =================
      const __amdgpu_buffer_rsrc_t ra = make_rsrc(G.b, G.bbytes);      // tokens
      const __amdgpu_buffer_rsrc_t rb = make_rsrc(G.w0, G.wbytes);     // weights
      // running byte offsets of this lane's 16 bytes per load instruction (kOob + small stays out
      // of range), and the logical column (in elements) behind them for the K tail
      unsigned aoff[kInsA], boff[kInsB];
      int acol[kInsA], bcol[kInsB];
#pragma unroll
      for (int p = 0; p < kInsA; ++p) {
        const int tr = kRowsPerIns * (lw * kInsA + p) + ld_sub;        // row of the tile
        const int r = m0 + tr;
        const bool val = r < G.m;
        int row = r;
        if (G.gather) row = val ? clampi(a.sorted_token[G.row0 + r], 0, a.T - 1) : 0;
        acol[p] = (ld_pc ^ row_key(tr)) * 8;
        aoff[p] = (val ? (unsigned)row * (unsigned)G.ldw * 2u : kOob) + (unsigned)acol[p] * 2u;
      }
#pragma unroll
      for (int p = 0; p < kInsB; ++p) {
        // weight row of the tile: gate/up tiles hold BNR/2 rows of W_gate, then the same rows of W_up
        const int br = WF::kRowsPerIns * (lw * kInsB + p) + ld_subw;
        int n;
        unsigned extra = 0;
        if (MODE == kGateUp) {
          n = n0 + (br % (BNR / 2));
          if (br >= BNR / 2) extra = (unsigned)G.N * WF::bytes((unsigned)G.ldw);
        } else {
          n = n0 + br;
        }
        bcol[p] = (ld_pcw ^ WF::key(br)) * WF::kPerCol;
        boff[p] = (n < G.N ? (unsigned)n * WF::bytes((unsigned)G.ldw) + extra : kOob) + WF::bytes((unsigned)bcol[p]);
      }
      // chunk `kt` into stage `st`, then step the offsets to the next chunk
      auto issue = [&](int st, int kt) {
        char* const sa = s_tiles + st * kStageBytes + (lw * kInsA) * 1024;
        char* const sb = s_tiles + st * kStageBytes + BM * kRowB + (lw * kInsB) * 1024;
        const bool full = (kt + 1) * BK <= K;
#pragma unroll
        for (int p = 0; p < kInsA; ++p) {
          const unsigned off = full ? aoff[p] : ((kt * BK + acol[p] < K) ? aoff[p] : kOob);
          __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void*)(sa + p * 1024), 16, (int)off, 0, 0, 0);
          aoff[p] += kRowB;
        }
#pragma unroll
        for (int p = 0; p < kInsB; ++p) {
          const unsigned off = full ? boff[p] : ((kt * BK + bcol[p] < K) ? boff[p] : kOob);
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void*)(sb + p * 1024), 16, (int)off, 0, 0, 0);
          boff[p] += kRowBW;
        }
      };
      // wait until at most `pending` whole chunks of this wave's loads are still in flight
      auto wait_chunks = [&](int pending) {
        static_assert(kStages <= 4, "wait_chunks covers up to two chunks in flight behind the awaited one");
        if (pending <= 0) MM_WAIT_VMCNT(0);
        else if (pending == 1) MM_WAIT_VMCNT(kPerChunk);
        else MM_WAIT_VMCNT(2 * kPerChunk);
      };
      int issued = 0, st_is = 0;                             // chunks issued; stage of the next one
      for (; issued < kAhead && issued < nk; ++issued) { issue(st_is, issued); st_is = st_is + 1 == kStages ? 0 : st_is + 1; }
      wait_chunks(issued - 1);                               // chunk 0 has landed
      lds_barrier();                                         // barrier 0
      for (int kt = 0; kt < nk; ++kt) {
        // barrier kt was passed: every computing wave is done reading chunk kt-1, whose stage
        // is the one that chunk kt+kAhead goes to
        if (issued < nk) { issue(st_is, issued); st_is = st_is + 1 == kStages ? 0 : st_is + 1; ++issued; }
        wait_chunks(issued - (kt + 2));                      // chunk kt+1 has landed (or nothing is left)
        lds_barrier();                                       // barrier kt+1
      }
      continue;
    }

    // ================= computing waves: fragment reads, MFMAs, barriers, epilogue =================
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // 32-token blocks of this wave that hold rows of the group: a group's last token tile is
    // mostly empty when the group is small against BM, and a block without rows is neither read
    // from LDS nor multiplied (its accumulators stay zero and are not stored).  A wave without any
    // rows only keeps the barriers.
    const int rows_w = G.m - m0 - wm * TM * 32;
    const int n_blk = rows_w <= 0 ? 0 : (rows_w >= TM * 32 ? TM : (rows_w + 31) >> 5);

    // Barrier kt says "chunk kt has landed" (the loaders waited for it) and "chunk kt-1 has been
    // read" (it sits in front of the last k-step's MFMAs of chunk kt-1, whose fragments were read
    // one k-step earlier).  The fragments of the first k-step of chunk kt are read right behind
    // it, under those MFMAs.
    constexpr int kParts = BK / 16;
    // MXFP4: the scale bytes of this lane's weight rows, one row of ldw / 32 bytes per weight row
    // (gate/up: the up rows follow the N gate rows); a lane of half h needs block 2 kt + h of chunk kt
    unsigned sc_row[TN];
    __amdgpu_buffer_rsrc_t rsc = make_rsrc(a.x, 0);
    if constexpr (WB == 0) {
      const unsigned blocks = (unsigned)G.ldw >> 5;
      rsc = make_rsrc(G.scale, (unsigned)((MODE == kGateUp ? 2 : 1) * G.N - 1) * blocks + ((unsigned)K >> 5));
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        int n;
        if (MODE == kGateUp) n = n0 + wn * (TN / 2) * 32 + (j % (TN / 2)) * 32 + (lane & 31);
        else n = n0 + wn * TN * 32 + j * 32 + (lane & 31);
        sc_row[j] = n < G.N ? (unsigned)((MODE == kGateUp && j >= TN / 2 ? G.N : 0) + n) * blocks : kOob;
      }
    }
    auto main_loop = [&](auto nb_tag) {
      constexpr int NB = decltype(nb_tag)::value;          // token blocks in use: 1 .. TM
      // token fragments of k-step kk of the chunk in stage st (8-bit weights: k-step 2p + e reads
      // the 16-byte column 4p + 2h + e, see the head of the file)
      auto read_a = [&](int st, int kk, bf16x8 (&fa)[TM]) {
        const unsigned lc = WB == 2 ? (unsigned)(kk * 2 + (lane >> 5))
                          : (WB == 1 ? (unsigned)((kk >> 1) * 4 + (lane >> 5) * 2 + (kk & 1)) : (unsigned)((lane >> 5) * 4 + kk));
        const unsigned col = (lc ^ fkey) * 16u + (unsigned)(st * kStageBytes);
        if constexpr (NB == 1) frag_read1<0>(fa[0], a_rd + col);
        else frag_read2<0, kJ>(fa[0], fa[1], a_rd + col);
        if constexpr (NB == 3) frag_read1<2 * kJ>(fa[2], a_rd + col);
        if constexpr (NB == 4) frag_read2<2 * kJ, 3 * kJ>(fa[2], fa[3], a_rd + col);
      };
      // weight fragments, 16 bytes per lane and column tile: bf16, the 8 k of k-step c; 8-bit, the
      // 2 x 8 codes of the k-steps 2c and 2c + 1; MXFP4 (c = 0), the 4 x 8 codes of the chunk
      auto read_b = [&](int st, int c, bf16x8 (&fb)[TN]) {
        const unsigned lc = (unsigned)(c * 2 + (lane >> 5));
        const unsigned col = (lc ^ (WB == 2 ? fkey : fkeyw)) * 16u + (unsigned)(st * kStageBytes);
        if constexpr (TN == 2) {
          frag_read2<0, kUp>(fb[0], fb[1], b_rd + col);
        } else {
          frag_read2<0, kJw>(fb[0], fb[1], b_rd + col);
          frag_read2<kUp, kUp + kJw>(fb[2], fb[3], b_rd + col);
        }
      };
      bf16x8 fa[2][TM] = {}, fb[2][TN];
      bf16x8 fr[TN];                                       // narrow formats: the codes of kPer k-steps
      constexpr int kPer = WF::kStepsPerRead;
      // MXFP4: the scale of this lane's block of the chunk, per column tile: in use (as fp32) and
      // being loaded for the next chunk (as a byte)
      float scf[TN];
      unsigned scn[TN];
      auto load_mx_scales = [&](int kt) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
          scn[j] = __builtin_amdgcn_raw_buffer_load_b8(rsc, (int)(sc_row[j] == kOob ? kOob : sc_row[j] + (unsigned)(kt * 2 + (lane >> 5))), 0, 0);
      };
      auto take_mx_scales = [&]() {
#pragma unroll
        for (int j = 0; j < TN; ++j) scf[j] = e8m0_to_f32(scn[j] & 0xffu);
      };
      auto widen = [&](bf16x8 (&dst)[TN], int e) {         // k-step e of the kPer in fr
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const i32x4 w = __builtin_bit_cast(i32x4, fr[j]);
          if constexpr (WB == 1) dst[j] = e ? widen_e4m3(w[2], w[3]) : widen_e4m3(w[0], w[1]);
          else dst[j] = widen_mx4(w[e & 3], scf[j]);
        }
      };
      if constexpr (WB == 0) { load_mx_scales(0); }
      lds_barrier();                                       // barrier 0
      read_a(0, 0, fa[0]);
      if constexpr (WB == 2) { read_b(0, 0, fb[0]); frag_wait(fa[0]); frag_wait(fb[0]); }
      else {
        read_b(0, 0, fr); frag_wait(fa[0]); frag_wait(fr);
        if constexpr (WB == 0) { take_mx_scales(); load_mx_scales(1); }
        widen(fb[0], 0);
      }
      int st = 0;                                          // stage of chunk kt
      for (int kt = 0; kt < nk; ++kt) {
        const int st_nx = st + 1 == kStages ? 0 : st + 1;  // stage of chunk kt+1
#pragma unroll
        for (int kk = 0; kk < kParts; ++kk) {
          const int cur = kk & 1, nxt = (kk + 1) & 1;      // kParts is even: set 0 again holds k-step 0 of the next chunk
          int st_rd = st, kk_rd = kk + 1;
          if (kk + 1 == kParts) {
            lds_barrier();                                 // barrier kt+1
            st_rd = st_nx; kk_rd = 0;                      // stale data behind the last chunk; never used
          }
          read_a(st_rd, kk_rd, fa[nxt]);
          if constexpr (WB == 2) {
            read_b(st_rd, kk_rd, fb[nxt]);
#pragma unroll
            for (int i = 0; i < NB; ++i)
#pragma unroll
              for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
            frag_wait(fa[nxt]); frag_wait(fb[nxt]);
          } else {
            // fr holds the codes of kPer k-steps.  In the last of them fr is free (everything widened)
            // and takes the next kPer; in the others the codes of the next k-step are in fr already.
            // They are widened behind the first token block's MFMAs, so that the conversions run while
            // the matrix unit works.
            const bool kRead = (kk % kPer) == kPer - 1;     // known after unrolling
            if (kRead) read_b(st_rd, kk_rd / kPer, fr);
#pragma unroll
            for (int j = 0; j < TN; ++j)
              acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][0], fb[cur][j], acc[0][j], 0, 0, 0);
            frag_wait(fa[nxt]);
            if (kRead) frag_wait(fr);
            if constexpr (WB == 0) {
              if (kRead) { take_mx_scales(); load_mx_scales(kt + 2); }   // the next chunk's scales in use, the one after on its way
            }
            widen(fb[nxt], (kk + 1) % kPer);
#pragma unroll
            for (int i = 1; i < NB; ++i)
#pragma unroll
              for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
          }
          __builtin_amdgcn_sched_barrier(0);               // keep the steps apart; free order inside a step
        }
        st = st_nx;
      }
    };
    if (n_blk == TM) {
      main_loop(std::integral_constant<int, TM>{});
    } else if (n_blk == 0) {
      for (int kt = 0; kt <= nk; ++kt) lds_barrier();      // barriers 0 .. nk, as the other waves pass them
    } else {
      if constexpr (TM == 2) {
        main_loop(std::integral_constant<int, 1>{});
      } else {
        if (n_blk == 1) main_loop(std::integral_constant<int, 1>{});
        else if (n_blk == 2) main_loop(std::integral_constant<int, 2>{});
        else main_loop(std::integral_constant<int, 3>{});
      }
    }

    // ---- epilogue: accumulator v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32 ----
    // 8-bit weights: the scale of the weight row behind column tile j (gate/up: of the gate row and
    // of the up row behind output column j)
    float wsc[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      wsc[j] = 1.f;
      if (WB == 1) {
        const float* sc = static_cast<const float*>(G.scale);
        if (MODE == kGateUp) {
          const int col = n0 + wn * (TN / 2) * 32 + (j % (TN / 2)) * 32 + (lane & 31);
          if (col < G.N) wsc[j] = sc[(j >= TN / 2 ? G.N : 0) + col];
        } else {
          const int col = n0 + wn * TN * 32 + j * 32 + (lane & 31);
          if (col < G.N) wsc[j] = sc[col];
        }
      }
    }
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
              const float gte = WB == 1 ? acc[i][j][v] * wsc[j] : acc[i][j][v];
              const float upv = WB == 1 ? acc[i][j + TN / 2][v] * wsc[j + TN / 2] : acc[i][j + TN / 2][v];
              const float hv = gte / (1.f + __expf(-gte)) * upv;
              const __bf16 o = (__bf16)hv;
              static_cast<S*>(G.out)[(size_t)r * G.N + col] = __builtin_bit_cast(uint16_t, o);
            }
          }
        } else {
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * TN * 32 + j * 32 + (lane & 31);
            if (col < G.N) static_cast<float*>(G.out)[(size_t)r * a.H + col] = WB == 1 ? acc[i][j][v] * wsc[j] : acc[i][j][v];
          }
        }
      }
  }
}

template <int MODE, typename SH, int WB>
int launch_tiled_shape(const StreamArgs& a, hipStream_t s) {
  constexpr size_t kLds = (size_t)kStages * SH::template stage_bytes<WB>();
  static std::atomic<int> cached{0};
  int per_cu = cached.load(std::memory_order_relaxed);
  if (per_cu == 0) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&tiled_kernel<MODE, SH, WB>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds) != hipSuccess)
      return hip_fail(hipGetLastError(), "tiled_kernel: LDS size attribute");
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, tiled_kernel<MODE, SH, WB>, SH::kThreads, kLds) != hipSuccess || n < 1) n = 1;
    per_cu = n;
    cached.store(n, std::memory_order_relaxed);
  }
  int grid = device_cu_count() * per_cu;
  grid = grid / 8 * 8;                                      // the XCD walk wants a multiple of 8
  if (grid < 8) grid = 8;
  hipLaunchKernelGGL((tiled_kernel<MODE, SH, WB>), dim3((unsigned)grid), dim3(SH::kThreads), kLds, s, a);
  return hip_fail(hipGetLastError(), "tiled_kernel launch");
}

#ifndef MOE_TILED_SHAPE
#define MOE_TILED_SHAPE 2, 2, 2, 4
#endif
typedef Shape<MOE_TILED_SHAPE> DefaultShape;

}  // namespace

int launch_tiled(StreamMode mode, int weight_format, const StreamArgs& a, hipStream_t s) {
  if (weight_format == 2) {
    if (mode == kGateUp) return launch_tiled_shape<kGateUp, DefaultShape, 2>(a, s);
    if (mode == kDown) return launch_tiled_shape<kDown, DefaultShape, 2>(a, s);
  }
#if MOE_TILED_BK == 64   // the narrow formats are written for 64-k chunks
  else if (weight_format == 1) {
    if (mode == kGateUp) return launch_tiled_shape<kGateUp, DefaultShape, 1>(a, s);
    if (mode == kDown) return launch_tiled_shape<kDown, DefaultShape, 1>(a, s);
  } else if (weight_format == 0) {
    if (mode == kGateUp) return launch_tiled_shape<kGateUp, DefaultShape, 0>(a, s);
    if (mode == kDown) return launch_tiled_shape<kDown, DefaultShape, 0>(a, s);
  }
#endif
  return fail(MOE_E_BADARG, "tiled kernel: bad mode or weight format");
}

}  // namespace mm
