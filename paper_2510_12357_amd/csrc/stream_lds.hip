// Skinny grouped GEMM for the decode regime with the weights streamed from HBM directly into
// LDS (bf16 activations; bf16 weights, or 8-bit E4M3 weights with fp32 row scales; same
// operation, groups and work items as stream_gemm.hip).
//
//   kGateUp  h = silu(W_gate x) * (W_up x)     (execution stage of Sec. II-A, SwiGLU)
//   kDown    y = W_down h
//
// Why: a kernel that loads the weights straight into registers (MFMA "A" operand layout) touches
// 16 rows x 64 bytes per load instruction and is limited, by its registers, in the bytes it
// keeps in flight.  Here a load instruction moves two rows x 512 contiguous bytes into LDS
// without passing through registers, and a workgroup keeps a 64 KB ring (4 stages) in flight.
//
// A workgroup has two kinds of waves:
//   * waves 0..3, loaders: issue the global->LDS loads of the weight chunks and nothing else.  A
//     work item is 32 weight rows (16 gate + 16 up rows, or 32 down rows) x all of K for up to 32
//     token rows, cut into chunks of 256 k (bf16; the narrower formats take 64 rows, see below);
//     one chunk = 32 rows x 512 B = one 16 KB stage = 4 load instructions per loader.  The chunks of all items of the workgroup form one stream, so the
//     ring never drains at an item boundary.  A loader issues exactly 4 loads per iteration (a
//     slot without a chunk issues 4 loads with out-of-range offsets, which the hardware turns
//     into zero fills without memory traffic), so its hand-counted s_waitcnt vmcnt(12) means:
//     the chunk issued three iterations ago has landed.  It decodes its next item while its
//     loads fly.
//   * waves 4..7, computers: read MFMA fragments from the stage that landed, load the token rows
//     (MFMA "B" operand, from L2) one chunk ahead into registers with ordinary loads (issued
//     right behind the MFMAs, so that they arrive during the barrier waits), run the
//     MFMAs, reduce the K split through LDS, apply the epilogue (SwiGLU) and store.  Computer c
//     owns token tile c & 1 (16 token rows) and the k-steps of parity c >> 1.
//   * Two workgroup barriers per iteration: "landed" (the chunk issued three iterations ago is in
//     LDS for every wave) and "free" (the stage just consumed may be refilled; partial sums of an
//     item that ended are complete).  Loaders and computers execute the same number of iterations: the number of
//     chunks of the workgroup's items, which both derive from blockIdx and the item table, plus
//     the three iterations that the computers lag behind.
//   * Inside a stage, the 16-byte column c of row r sits at column c ^ (r & 15): the
//     ds_read_b128 of a fragment (16 rows x the same logical column) is bank-conflict free.
//   * Groups with more than 32 token rows become several items that read the same weights; the
//     item order places them 8 items apart, i.e. on workgroups of the same XCD at the same time,
//     so that the repeats hit in that XCD's L2.
//   * 8-bit weights (WB = 1): a stage is 64 rows x 256 bytes (256 k per chunk; see Fmt).  A 16-byte column
//     then holds 16 consecutive k of a row, i.e. the weights of two MFMA k-steps; the k order
//     inside a chunk is permuted accordingly, and the token rows are loaded with the same
//     permutation.  The computers widen the codes to bf16 (exact: 3 mantissa bits) in front of
//     the MFMAs, and the row scale multiplies the fp32 sum in the epilogue.
//   * MXFP4 weights (WB = 0: OCP microscaling, 4-bit E2M1 codes with one E8M0 scale per 32 k):
//     64 rows x 256 bytes per stage, 512 k per chunk; a 16-byte column holds the 32 codes of one scale block, i.e. the weights
//     of four MFMA k-steps, with the k order inside a chunk permuted accordingly.  The scale
//     bytes of a chunk (64 rows x 16 blocks = 1 KB) are fetched by one computer wave with one
//     load instruction, one chunk ahead, and handed to the others through a double-buffered KB
//     of LDS (byte loads from global memory by every lane cost more than the weight stream);
//     code x scale is widened to bf16 in one instruction (exact) in front of the MFMAs.
#include <atomic>
#include <type_traits>

#include "internal.h"
#include "groups.h"

namespace mm {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int kStageBytes = 16384;           // one stage of the ring = one chunk of an item: rows x bytes per row
constexpr int kStages = 4;
constexpr int kWorkers = 4;                  // loader waves = computer waves
constexpr int kThreadsL = 2 * kWorkers * 64;
constexpr int kTok = 32;                     // token rows per item, at most (two tiles of 16)
constexpr int kKParts = 2;                   // worker waves that split the k-steps of one token tile

// Weight formats (template parameter WB): 2 = bf16, 1 = 8-bit codes, 0 = MXFP4 (half a byte), and
// the shape of a stage that goes with them.  The fewer bytes a weight has, the more k a row of
// given bytes covers, and every 8 k of a token tile cost the computers one load of token rows
// whatever the weights weigh; the 8-bit and 4-bit formats therefore take items of 64 rows x 256
// bytes (256 / 512 k) instead of 32 rows x 512 bytes, which halves the token-row loads per weight
// byte.
template <int WB> struct Fmt {
  static constexpr int kRows = WB == 2 ? 32 : 64;                 // weight rows per item
  static constexpr int kRowBytes = kStageBytes / kRows;           // bytes of one weight row per chunk
  static constexpr int kTiles = kRows / 16;                       // MFMA row tiles per item
  static constexpr int kCols = kRowBytes / 16;                    // 16-byte columns of a row in a stage
  static constexpr int kRowsPerIns = 1024 / kRowBytes;            // rows one load instruction fills
  static constexpr int kReads = kCols / 4 / kKParts;              // fragment reads per worker, row tile and chunk
  static constexpr int kPerColumn = WB ? 16 / WB : 32;            // k per 16-byte column
  static constexpr int kPerChunk = kCols * kPerColumn;            // k per chunk
  static constexpr int kSteps = kPerColumn / 8;                   // MFMA k-steps fed by one column
  static constexpr int kOutRows = kRows;                          // output rows per down item; gate/up: half
  static __device__ __forceinline__ unsigned row_bytes(int k) { return WB ? (unsigned)k * WB : (unsigned)k / 2u; }
};

// vmcnt(n): bits [3:0] and [15:14]; expcnt and lgkmcnt left at their maxima (no wait)
#define MM_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0f70 | ((n) & 15) | (((n) >> 4) << 14))

// Workgroup barrier that orders LDS accesses only.  __syncthreads() also fences global memory,
// which makes the compiler wait for every outstanding load, i.e. it would drain the ring.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ unsigned uni(unsigned v) { return (unsigned)__builtin_amdgcn_readfirstlane((int)v); }
template <typename P>
__device__ __forceinline__ P* uni(P* p) {
  const uint64_t v = (uint64_t)p;
  const uint64_t lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)v);
  const uint64_t hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(v >> 32));
  return (P*)((hi << 32) | lo);
}

struct Item {
  // ---- same value in all lanes of the workgroup ----
  int valid;
  int nch;          // chunks
  int K, N, m;
  int r0, n0;       // first token row / first weight row of the item
  int ntn;          // token tiles in use (1..2)
  int gather, row0;
  unsigned ldwb;    // bytes between rows of W
  unsigned ldbb;    // bytes between rows of B
  const void* scale;    // 8-bit weights: row scales of the group; MXFP4: its block scales (see Group::scale)
  unsigned sbytes;      // MXFP4: bytes readable from scale
  unsigned wbytes, bbytes;
  const void* w0;
  const void* b;
  void* out;
  // ---- per lane ----
  unsigned a_row[4];    // loaders: byte offset of the weight row behind each of the wave's 4 load instructions
  // computers: this lane's token row.  decode_item leaves the row number here (for a routed
  // gate/up item it comes from sorted_token, i.e. from memory) and resolve_row turns it into a byte
  // offset when the item becomes the current one, chunks later: no wave waits for that load.
  unsigned boff;        // byte offset of the row (kOob: none)
};

__device__ __forceinline__ void resolve_row(Item& it, int T) {
  it.boff = it.boff == kOob ? kOob : (unsigned)clampi((int)it.boff, 0, T - 1) * it.ldbb;
}

template <int MODE, int WB>
__device__ __forceinline__ Item decode_item(const StreamArgs& a, int j, int total, int n_groups,
                                            const int* s_prefix, const GroupSrc* s_src, int wave, int lane) {
  Item it;
  const int item = blockIdx.x + j * gridDim.x;
  it.valid = item < total;
  // group of the item = number of prefix entries 1..n_groups that are <= item (the prefix is
  // nondecreasing): 64 entries per ballot
  int cnt = 0;
  for (int g0 = 1; g0 <= n_groups; g0 += 64) {
    const int gg = g0 + lane;
    cnt += __popcll(__ballot(gg <= n_groups && s_prefix[gg] <= item));
  }
  const int g = it.valid ? __builtin_amdgcn_readfirstlane(cnt) : 0;
  GroupSrc src = s_src[g];
  src.m = uni(src.m); src.row0 = uni(src.row0); src.blob = uni(src.blob);
  const Group G = make_group<uint16_t, MODE, WB>(a, g, src);
  constexpr int KC = Fmt<WB>::kPerChunk;
  // Items of a group, in blocks of 8 row tiles: all token blocks of row tile (8 b + i) are
  // 8 items apart, i.e. they run at the same time on workgroups of the same XCD.
  const int local = item - uni(s_prefix[g]);
  constexpr int per = MODE == kGateUp ? Fmt<WB>::kRows / 2 : Fmt<WB>::kRows;
  const int rows = (G.N + per - 1) / per;
  const int tgs = max(1, (G.m + kTok - 1) / kTok);
  int tg = 0, row_item = local;     // one token block (the usual case at decode): nothing to divide
  if (tgs > 1) {
    const int block = local / (8 * tgs);
    const int rem = local - block * 8 * tgs;
    const int nb = max(1, min(8, rows - 8 * block));
    tg = rem / nb;
    row_item = block * 8 + (rem - tg * nb);
  }
  it.r0 = tg * kTok;
  it.n0 = row_item * per;
  it.K = it.valid ? G.K : 0;
  it.N = G.N; it.m = it.valid ? G.m : 0;
  it.nch = (it.K + KC - 1) / KC;
  it.ntn = clampi((it.m - it.r0 + 15) >> 4, 1, kTok / 16);
  it.gather = G.gather; it.row0 = G.row0;
  it.ldwb = Fmt<WB>::row_bytes(G.ldw);
  it.ldbb = (unsigned)G.ldw * 2u;
  it.scale = G.scale;
  // MXFP4: the scale rows of the group (gate and up for gate/up) end with the last row's last block
  it.sbytes = (WB == 0 && it.valid) ? (unsigned)((MODE == kGateUp ? 2 : 1) * G.N - 1) * ((unsigned)G.ldw >> 5) + ((unsigned)G.K >> 5) : 0u;
  // an item that does not exist keeps valid pointers and empty buffers: every load is out of range
  it.wbytes = it.valid ? G.wbytes : 0u; it.bbytes = it.valid ? G.bbytes : 0u;
  it.w0 = it.valid ? G.w0 : a.x; it.b = it.valid ? G.b : a.x; it.out = G.out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row_local = Fmt<WB>::kRowsPerIns * ((wave % kWorkers) * 4 + i) + lane / Fmt<WB>::kCols;
    unsigned off;
    int n;
    if (MODE == kGateUp) {       // the first half of an item's rows are gate rows, the second half the same up rows
      n = it.n0 + (row_local % per);
      off = (unsigned)n * it.ldwb + ((row_local >= per) ? (unsigned)G.N * it.ldwb : 0u);   // W_up follows W_gate
    } else {
      n = it.n0 + row_local;
      off = (unsigned)n * it.ldwb;
    }
    it.a_row[i] = (it.valid && n < G.N) ? off : kOob;
  }
  {
    const int r = it.r0 + (wave & 1) * 16 + (lane & 15);
    const bool val = it.valid && r < it.m;
    it.boff = val ? (it.gather ? (unsigned)a.sorted_token[it.row0 + r] : (unsigned)r) : kOob;
  }
  return it;
}


template <int WB>
struct Smem {
  char ring[kStages * kStageBytes];
  // K-split partial sums (the item counts during set-up).  Two row tiles: every computer writes its
  // sums; four row tiles: only the computers of the second k part do, the others add their own
  float red[Fmt<WB>::kTiles > 2 ? 2 : kWorkers][Fmt<WB>::kTiles][4][64];
  GroupSrc src[kMaxGroups];
  int prefix[kMaxGroups + 1];
  // MXFP4: the scale bytes of the chunk being consumed, double-buffered by iteration parity:
  // [row of the item][kp][q][t] for block (kp + 2 t) * 4 + q of the chunk, so that the bytes a
  // computing lane needs for one row sit side by side
  unsigned char mx_scale[WB == 0 ? 2 : 1][WB == 0 ? Fmt<WB>::kRows * Fmt<WB>::kCols : 16];
};


template <int MODE, int WB>
__global__ __launch_bounds__(kThreadsL) __attribute__((amdgpu_waves_per_eu(4, 4))) void stream_lds_kernel(const StreamArgs a) {
  typedef Fmt<WB> F;
  constexpr int KC = F::kPerChunk;           // k per chunk
  constexpr int kHalves = F::kSteps;         // MFMA k-steps fed by one 16-byte column: 1 (bf16), 2 (8-bit), 4 (MXFP4)
  constexpr int kTiles = F::kTiles, kReads = F::kReads, kRowBytes = F::kRowBytes;
  constexpr bool kOwnSums = kTiles > 2;      // the computers of k part 0 add their own sums to those of part 1
  // One LDS object, ring first (1 KB aligned: every load instruction fills one aligned KB).
  __shared__ __attribute__((aligned(1024))) Smem<WB> sm;
  char* const s_ring = sm.ring;
  auto& s_red = sm.red;
  GroupSrc* const s_src = sm.src;
  int* const s_prefix = sm.prefix;

  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  const int q = lane >> 4, c16 = lane & 15;
  const int n_groups = a.n_routed + (MODE == kDown ? a.n_slabs : a.n_shared);
  int* s_cnt = reinterpret_cast<int*>(&s_red[0][0][0][0]);           // kMaxGroups ints fit easily

  // ---- group table and item list ----
  for (int g = tid; g < n_groups; g += kThreadsL) {
    const GroupSrc src = load_group_src<MODE>(a, g);
    const Group G = make_group<uint16_t, MODE, WB>(a, g, src);
    constexpr int per = MODE == kGateUp ? F::kRows / 2 : F::kRows;
    const int rows = (G.N + per - 1) / per;
    const int tgs = (G.m + kTok - 1) / kTok;
    s_src[g] = src;
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
    if (lane == 0) s_prefix[0] = 0;
    for (int c = 0; c < C; ++c) if (base + c < n_groups) { run += s_cnt[base + c]; s_prefix[base + c + 1] = run; }
  }
  __syncthreads();
  const int total = s_prefix[n_groups];
  __syncthreads();                  // s_cnt (aliases the partial sums) is dead from here on

  if (wave < kWorkers) {
    // =================================== loader ===================================
    Item it = decode_item<MODE, WB>(a, 0, total, n_groups, s_prefix, s_src, wave, lane);
    Item nx = it;
    int j = 0, k = 0, drain = 0, s = 0;
    unsigned a_col[4], addr[4];     // logical 16-byte column per load instruction; running offsets
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row_local = F::kRowsPerIns * (wave * 4 + i) + lane / F::kCols;
      a_col[i] = (unsigned)((lane % F::kCols) ^ (row_local & 15));
      addr[i] = it.a_row[i] + a_col[i] * 16u;               // kOob + small stays out of range
    }
    __amdgpu_buffer_rsrc_t rs = make_rsrc(it.w0, it.wbytes);
    MM_WAIT_VMCNT(0);
    // Issues the next chunk of the stream (4 loads of this wave) into stage s & 3 and advances;
    // false for a slot behind the last chunk (4 loads that only zero-fill).
    auto issue_next = [&]() -> bool {
      const bool real = k < it.nch;                         // an item that does not exist has no chunks
      char* stage = s_ring + (s & (kStages - 1)) * kStageBytes + wave * 4096;
      if (real && (k + 1) * KC <= it.K) {                   // whole chunk inside K
#pragma unroll
        for (int i = 0; i < 4; ++i)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)(stage + i * 1024), 16, (int)addr[i], 0, 0, kStreamOnce);
      } else {
        // last, partial chunk, or no chunk: lanes out of range fill their part of the stage with zeros
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int kk = k * KC + (int)a_col[i] * F::kPerColumn;
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)(stage + i * 1024), 16,
                                                   (int)((real && kk < it.K) ? addr[i] : kOob), 0, 0, kStreamOnce);
        }
      }
      if (real) {
        ++k;
#pragma unroll
        for (int i = 0; i < 4; ++i) addr[i] += kRowBytes;
        if (k == 1) nx = decode_item<MODE, WB>(a, j + 1, total, n_groups, s_prefix, s_src, wave, lane);   // under the loads
        if (k == it.nch) {
          it = nx; ++j; k = 0;
          rs = make_rsrc(it.w0, it.wbytes);
#pragma unroll
          for (int i = 0; i < 4; ++i) addr[i] = it.a_row[i] + a_col[i] * 16u;
        }
      }
      ++s;
      return real;
    };
    for (;;) {
      const bool real = issue_next();
      MM_WAIT_VMCNT(12);                                    // the chunk issued three iterations ago has landed
      lds_barrier();                                        // "landed"
      lds_barrier();                                        // "free": stage (s + 1) & 3 was consumed
      if (!real && ++drain == 3) break;                     // the computers lag three iterations
    }
    MM_WAIT_VMCNT(0);
    return;
  }

  // =================================== computer ===================================
  const int c = wave - kWorkers, tw = c & 1, kp = c >> 1;
  Item cur = decode_item<MODE, WB>(a, 0, total, n_groups, s_prefix, s_src, c, lane);
  resolve_row(cur, a.T);
  Item nx = decode_item<MODE, WB>(a, 1, total, n_groups, s_prefix, s_src, c, lane);
  int j = 0, k = 0;                 // item ordinal and chunk being consumed
  int pending = 0;                  // the previous item's partial sums wait for their epilogue
  int need_nx = 0;                  // nx is stale (cur just moved on)
  int f_r0 = 0, f_n0 = 0, f_m = 0, f_N = 0, f_ntn = 0;
  void* f_out = nullptr;
  // Row tiles of an item: gate/up items hold kTiles / 2 tiles of gate rows and then the same tiles
  // of up rows; down items kTiles tiles of consecutive rows.
  constexpr int kHalfTiles = kTiles / 2;
  // 8-bit weights: the row scales this lane's outputs need, loaded when an item starts, so that no
  // epilogue waits for memory (the next item's are loaded behind the epilogue of this one)
  f32x4 sc[kTiles];
#pragma unroll
  for (int rt = 0; rt < kTiles; ++rt) sc[rt] = f32x4{0, 0, 0, 0};
  auto load_scales = [&](const Item& it) {
    if (WB != 1) return;
    // gate rows n0 + 16 rt + 4q + v and the same up rows (N further on); down rows n0 + 16 rt + 4q + v.
    // Buffer loads: rows that do not exist read zeros without a select that would wait for the load.
    const __amdgpu_buffer_rsrc_t rsc = make_rsrc(it.scale, it.valid ? (unsigned)((MODE == kGateUp ? 2 : 1) * it.N) * 4u : 0u);
#pragma unroll
    for (int rt = 0; rt < kTiles; ++rt) {
      const bool up = MODE == kGateUp && rt >= kHalfTiles;
      const int n = it.n0 + (up ? rt - kHalfTiles : rt) * 16 + 4 * q;
      const bool ok = it.valid && n < it.N;                 // N is a multiple of 16: all four or none
      sc[rt] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rsc, (int)(ok ? (unsigned)(up ? it.N + n : n) * 4u : kOob), 0, 0));
    }
  };
  load_scales(cur);
  const unsigned ring_base = (unsigned)(size_t)s_ring;
  unsigned rd_off[kReads];          // LDS offsets of this lane's fragments inside a stage (row tile 0)
#pragma unroll
  for (int t = 0; t < kReads; ++t)
    rd_off[t] = ring_base + (unsigned)c16 * kRowBytes + (unsigned)((((kp + t * kKParts) * 4 + q) ^ c16) * 16);
  // token rows of one chunk: for read t, the kHalves x 8 k behind column (kp + 2t) * 4 + q
  i32x4 bbuf[kReads][kHalves];
#pragma unroll
  for (int t = 0; t < kReads; ++t)
#pragma unroll
    for (int h = 0; h < kHalves; ++h) bbuf[t][h] = i32x4{0, 0, 0, 0};
  // MXFP4: computer 3 moves the scale bytes.  Lane l fetches the 16 blocks of item row l of the
  // chunk with one 16-byte load, one chunk ahead, and writes them to LDS in front of the "landed"
  // barrier of the iteration that consumes the chunk.
  static_assert(WB != 0 || (F::kRows == 64 && F::kCols == 16), "the scale mover is written for 64 rows of 16 blocks");
  i32x4 mx_regs = i32x4{0, 0, 0, 0};
  int mx_loaded = 0;
  auto load_mx_scales = [&]() {
    const __amdgpu_buffer_rsrc_t rsc = make_rsrc(cur.scale, cur.sbytes);
    int n;
    unsigned row;
    if (MODE == kGateUp) { n = cur.n0 + (lane & 31); row = (unsigned)n + ((lane >> 5) ? (unsigned)cur.N : 0u); }
    else { n = cur.n0 + lane; row = (unsigned)n; }
    const int blk0 = k * F::kCols;                                 // first block of the chunk, in the group's K
    const int nvalid = clampi((cur.K >> 5) - blk0, 0, 16);         // blocks of the row that exist from there on
    const bool ok = cur.valid && n < cur.N && nvalid > 0;
    i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsc, (int)(ok ? row * ((unsigned)cur.ldwb >> 4) + (unsigned)blk0 : kOob), 0, 0);
    // bytes behind the row's last block belong to the next row: cleared (their codes are zeros,
    // and zero times a NaN scale would not be)
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const int vb = clampi(nvalid - 4 * d, 0, 4);
      v[d] &= vb == 4 ? -1 : (int)((1u << (8 * vb)) - 1u);
    }
    mx_regs = v;
    mx_loaded = 1;
  };
  // byte j of a row's 16 is block j = (kp + 2t) * 4 + q; the computing lanes read [kp][q][t]
  auto store_mx_scales = [&](unsigned char* buf) {
    unsigned out[4] = {0, 0, 0, 0};
#pragma unroll
    for (int jb = 0; jb < 16; ++jb) {
      const int pos = ((jb >> 2) & 1) * 8 + (jb & 3) * 2 + (jb >> 3);
      const unsigned byte = ((unsigned)mx_regs[jb >> 2] >> (8 * (jb & 3))) & 0xffu;
      out[pos >> 2] |= byte << (8 * (pos & 3));
    }
    *reinterpret_cast<i32x4*>(buf + lane * 16) = i32x4{(int)out[0], (int)out[1], (int)out[2], (int)out[3]};
  };

  f32x4 acc[kTiles];                // the sums of an item stay here until its epilogue, one barrier after its last chunk
#pragma unroll
  for (int rt = 0; rt < kTiles; ++rt) acc[rt] = f32x4{0, 0, 0, 0};

  // Scale (8-bit weights), activate and store this lane's kTiles x 4 sums of the item that ended.
  auto store_outputs = [&](float (&val)[kTiles][4]) {
    if (WB == 1) {
#pragma unroll
      for (int rt = 0; rt < kTiles; ++rt)
#pragma unroll
        for (int v = 0; v < 4; ++v) val[rt][v] *= sc[rt][v];
    }
    const int r = f_r0 + tw * 16 + c16;
    if (r < f_m) {
      if (MODE == kGateUp) {
#pragma unroll
        for (int rt = 0; rt < kHalfTiles; ++rt) {
          const int i = f_n0 + rt * 16 + 4 * q;
          if (i < f_N) {
            float hv[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const float gte = val[rt][v];
              hv[v] = gte / (1.f + __expf(-gte)) * val[rt + kHalfTiles][v];
            }
            bf16x4 o = {(__bf16)hv[0], (__bf16)hv[1], (__bf16)hv[2], (__bf16)hv[3]};
            *reinterpret_cast<bf16x4*>(static_cast<uint16_t*>(f_out) + (size_t)r * f_N + i) = o;
          }
        }
      } else {
#pragma unroll
        for (int rt = 0; rt < kTiles; ++rt) {
          const int col = f_n0 + rt * 16 + 4 * q;
          if (col < f_N)
            *reinterpret_cast<f32x4*>(static_cast<float*>(f_out) + (size_t)r * a.H + col) =
                f32x4{val[rt][0], val[rt][1], val[rt][2], val[rt][3]};
        }
      }
    }
  };
  auto epilogue = [&]() {
    // computers 0 and 1 finish token tiles 0 and 1: add the two k parts (part 0 first), activate, store
    if (kp == 0 && tw < f_ntn) {
      float val[kTiles][4];
#pragma unroll
      for (int rt = 0; rt < kTiles; ++rt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          if constexpr (kOwnSums) val[rt][v] = acc[rt][v] + s_red[tw][rt][v][lane];
          else val[rt][v] = s_red[tw][rt][v][lane] + s_red[tw + 2][rt][v][lane];
        }
      store_outputs(val);
    }
  };

  // Fragments of the chunk in stage `stage`, MFMAs against the token rows in bbuf.
  auto consume = [&](int stage, const unsigned char* mx_sc) {
    const unsigned st = (unsigned)(stage * kStageBytes);
    bf16x8 f[kTiles][kReads];                               // row tile, 16-byte column
    constexpr int kT = 16 * kRowBytes;                      // bytes between row tiles
    if constexpr (kTiles == 2) {
      static_assert(kTiles != 2 || kReads == 4, "two row tiles: four columns per wave and tile");
      asm volatile(
          "ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:%12\n"
          "ds_read_b128 %2, %9\n ds_read_b128 %3, %9 offset:%12\n"
          "ds_read_b128 %4, %10\n ds_read_b128 %5, %10 offset:%12\n"
          "ds_read_b128 %6, %11\n ds_read_b128 %7, %11 offset:%12\n"
          "s_waitcnt lgkmcnt(0)"
          : "=&v"(f[0][0]), "=&v"(f[1][0]), "=&v"(f[0][1]), "=&v"(f[1][1]), "=&v"(f[0][2]), "=&v"(f[1][2]),
            "=&v"(f[0][3]), "=&v"(f[1][3])
          : "v"(rd_off[0] + st), "v"(rd_off[1] + st), "v"(rd_off[2] + st), "v"(rd_off[3] + st), "n"(kT)
          : "memory");
    } else {
      static_assert(kTiles == 2 || (kTiles == 4 && kReads == 2), "four row tiles: two columns per wave and tile");
      asm volatile(
          "ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:%10\n"
          "ds_read_b128 %2, %8 offset:%11\n ds_read_b128 %3, %8 offset:%12\n"
          "ds_read_b128 %4, %9\n ds_read_b128 %5, %9 offset:%10\n"
          "ds_read_b128 %6, %9 offset:%11\n ds_read_b128 %7, %9 offset:%12\n"
          "s_waitcnt lgkmcnt(0)"
          : "=&v"(f[0][0]), "=&v"(f[1][0]), "=&v"(f[2][0]), "=&v"(f[3][0]), "=&v"(f[0][1]), "=&v"(f[1][1]),
            "=&v"(f[2][1]), "=&v"(f[3][1])
          : "v"(rd_off[0] + st), "v"(rd_off[1 % kReads] + st), "n"(kT), "n"(2 * kT), "n"(3 * kT)
          : "memory");
    }
    unsigned mx_s[kTiles];                                  // MXFP4: this lane's scale bytes (t = 0, 1) per row tile
    if constexpr (WB == 0) {
#pragma unroll
      for (int rt = 0; rt < kTiles; ++rt)
        mx_s[rt] = *reinterpret_cast<const unsigned short*>(mx_sc + (rt * 16 + c16) * 16 + kp * 8 + q * 2);
    }
#pragma unroll
    for (int t = 0; t < kReads; ++t) {
      if constexpr (WB == 2) {
        const bf16x8 bv = __builtin_bit_cast(bf16x8, bbuf[t][0]);
#pragma unroll
        for (int rt = 0; rt < kTiles; ++rt)
          acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[rt][t], bv, acc[rt], 0, 0, 0);
      } else if constexpr (WB == 1) {
#pragma unroll
        for (int h = 0; h < kHalves; ++h) {
          const bf16x8 bv = __builtin_bit_cast(bf16x8, bbuf[t][h]);
#pragma unroll
          for (int rt = 0; rt < kTiles; ++rt) {
            const i32x4 w = __builtin_bit_cast(i32x4, f[rt][t]);
            acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(widen_e4m3(w[2 * h], w[2 * h + 1]), bv, acc[rt], 0, 0, 0);
          }
        }
      } else {
        float sv[kTiles];
#pragma unroll
        for (int rt = 0; rt < kTiles; ++rt) sv[rt] = e8m0_to_f32((mx_s[rt] >> (8 * t)) & 0xffu);
#pragma unroll
        for (int h = 0; h < kHalves; ++h) {
          const bf16x8 bv = __builtin_bit_cast(bf16x8, bbuf[t][h]);
#pragma unroll
          for (int rt = 0; rt < kTiles; ++rt) {
            const i32x4 w = __builtin_bit_cast(i32x4, f[rt][t]);
            acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(widen_mx4(w[h], sv[rt]), bv, acc[rt], 0, 0, 0);
          }
        }
      }
    }
  };
  // Token rows of chunk (cur, k) into bbuf.  Nothing of this wave is in flight any more (the
  // previous token rows were consumed or belong to a tile this wave skips); saying so keeps the
  // compiler from guarding every one of the loads against a load of the previous iteration into
  // the same registers.
  auto load_token_rows = [&]() {
    MM_WAIT_VMCNT(0);
    const __amdgpu_buffer_rsrc_t rb = make_rsrc(cur.b, cur.bbytes);
#pragma unroll
    for (int t = 0; t < kReads; ++t)
#pragma unroll
      for (int h = 0; h < kHalves; ++h) {
        // the k behind 16-byte column (kp + 2t) * 4 + q of the weight rows (k-step h of that column)
        const int kk = k * KC + ((kp + t * kKParts) * 4 + q) * F::kPerColumn + h * 8;
        const bool ok = cur.valid && kk < cur.K && cur.boff != kOob;
        bbuf[t][h] = __builtin_amdgcn_raw_buffer_load_b128(rb, (int)(ok ? cur.boff + (unsigned)kk * 2u : kOob), 0, 0);
      }
  };

  // One iteration.
  auto step = [&](int s) -> bool {
    if (WB == 0 && c == 3 && mx_loaded) {                   // the scales of the chunk consumed below
      store_mx_scales(sm.mx_scale[s & 1]);
      mx_loaded = 0;
    }
    lds_barrier();                                          // "landed": the chunk issued three iterations ago
    if (s >= 3 && cur.valid) {
      if (tw < cur.ntn) consume((s + 1) & (kStages - 1), sm.mx_scale[s & 1]);
      if (++k == cur.nch) {         // item done: hand the partial sums over, move on
        if (!kOwnSums || kp == 1) {
#pragma unroll
          for (int rt = 0; rt < kTiles; ++rt)
#pragma unroll
            for (int v = 0; v < 4; ++v) s_red[kOwnSums ? tw : c][rt][v][lane] = acc[rt][v];
        }
        f_r0 = cur.r0; f_n0 = cur.n0; f_m = cur.m; f_N = cur.N; f_ntn = cur.ntn; f_out = cur.out;
        pending = 1;
        cur = nx; ++j; k = 0;
        resolve_row(cur, a.T);
        need_nx = 1;
      }
    }
    // Token rows of the chunk consumed in the next iteration: issued here, behind the MFMAs that
    // read the previous ones, they arrive while this wave waits at the two barriers.  That chunk
    // is (cur, k): the one after the chunk just consumed; a wave whose token tile is empty loads
    // nothing (its MFMAs are skipped as well).
    if (s >= 2 && tw < cur.ntn) load_token_rows();
    if (WB == 0 && c == 3 && s >= 2) load_mx_scales();      // after the token rows: they start with a wait for everything in flight
    lds_barrier();                                          // "free"; partial sums of an item that ended are complete
    // what follows runs while the loaders wait for their next chunk
    if (pending) {
      pending = 0;
      epilogue();
#pragma unroll
      for (int rt = 0; rt < kTiles; ++rt) acc[rt] = f32x4{0, 0, 0, 0};    // the next chunk is consumed in the next iteration
    }
    if (need_nx) {
      need_nx = 0;
      load_scales(cur);
      nx = decode_item<MODE, WB>(a, j + 1, total, n_groups, s_prefix, s_src, c, lane);
    }
    return cur.valid || s < 2;
  };

  for (int s = 0; step(s); ++s) {}
}

template <int MODE, int WB>
int launch_lds_typed(const StreamArgs& a, hipStream_t s) {
  const long items = item_upper_bound((StreamMode)MODE, a, kTok);
  if (items <= 0) return MOE_OK;
  // persistent workgroups: exactly as many as are resident at once
  static std::atomic<int> cached{0};                      // the same on every device this library runs on (gfx950)
  int per_cu = cached.load(std::memory_order_relaxed);
  if (per_cu == 0) {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, stream_lds_kernel<MODE, WB>, kThreadsL, 0) != hipSuccess || n < 1) n = 1;
    per_cu = n;
    cached.store(n, std::memory_order_relaxed);
  }
  long grid = (long)device_cu_count() * per_cu;
  if (grid > items) grid = items;
  hipLaunchKernelGGL((stream_lds_kernel<MODE, WB>), dim3((unsigned)grid), dim3(kThreadsL), 0, s, a);
  return hip_fail(hipGetLastError(), "stream_lds_kernel launch");
}

}  // namespace

int launch_stream_lds(StreamMode mode, int weight_format, const StreamArgs& a, hipStream_t s) {
  if (weight_format == 2) {
    if (mode == kGateUp) return launch_lds_typed<kGateUp, 2>(a, s);
    if (mode == kDown) return launch_lds_typed<kDown, 2>(a, s);
  } else if (weight_format == 1) {
    if (mode == kGateUp) return launch_lds_typed<kGateUp, 1>(a, s);
    if (mode == kDown) return launch_lds_typed<kDown, 1>(a, s);
  } else if (weight_format == 0) {
    if (mode == kGateUp) return launch_lds_typed<kGateUp, 0>(a, s);
    if (mode == kDown) return launch_lds_typed<kDown, 0>(a, s);
  }
  return fail(MOE_E_BADARG, "bad stream mode / weight format");
}

}  // namespace mm
