// Token-to-expert dispatch with a variable expert count per token (k_t = k_big for important
// tokens, k_little otherwise; Sec. III-A).  The execution stage (Sec. II-A) wants the
// (token, rank) pairs grouped per expert; the order is fixed to (expert asc, token asc), i.e. a
// stable counting sort of the pair list by expert id.
//
// The order is produced without order-dependent operations: expert e's segment comes from scanning
// the tokens in ascending order and compacting the matches with ballot/popcount prefix sums, so the
// result is unique and reproducible (the large-T count pass adds up per-chunk histograms with LDS
// integer atomics: a sum, which does not depend on their order).  The experts of one token must be
// distinct, as the selection stage produces them.  Two shapes:
//   * T <= kSmallT: one workgroup, one wave per expert (round-robin), one launch.
//   * larger T: one workgroup per chunk of 128 tokens; a count kernel, then a scatter kernel
//     that rebuilds the prefixes of the counts itself.
#include "internal.h"

namespace mm {
namespace {

constexpr int kSmallT = 256;
constexpr int kSmallThreads = 1024;
constexpr int kBigThreads = 256;

__device__ __forceinline__ unsigned long long lanemask_lt(int lane) {
  return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

// rank at which token t names expert e in the LDS copy of the selection (-1 = not named);
// entries beyond k_t were stored as -1, so no k_t lookup is needed here
__device__ __forceinline__ int match_rank_lds(const int* s_idx, int t, int T, int K, int e) {
  if (t >= T) return -1;
  int found = -1;
  for (int j = K - 1; j >= 0; --j)
    if (s_idx[t * K + j] == e) found = j;
  return found;
}

__global__ __launch_bounds__(kSmallThreads) void dispatch_small_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ k_t, int j_lo, int T, int E, int K,
    int32_t* __restrict__ offsets, int32_t* __restrict__ sorted_token,
    int32_t* __restrict__ sorted_rank, int32_t* __restrict__ inv_pos) {
  __shared__ int s_idx[kSmallT * MOE_MAX_TOPK];
  __shared__ int s_count[MOE_MAX_EXPERTS];
  __shared__ int s_off[MOE_MAX_EXPERTS + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int kWaves = kSmallThreads / 64;

  // stage the selection once: every later pass reads LDS only
  for (int i = tid; i < T * K; i += kSmallThreads) {
    const int t = i / K, j = i - t * K;
    int kt = k_t[t];
    kt = kt < 0 ? 0 : (kt > K ? K : kt);
    const int e = idx[i];
    const bool pair = j >= j_lo && j < kt && (unsigned)e < (unsigned)E;
    s_idx[i] = pair ? e : -1;
    if (!pair) inv_pos[i] = -1;
  }
  __syncthreads();
  for (int e = wave; e < E; e += kWaves) {
    int cnt = 0;
    for (int t0 = 0; t0 < T; t0 += 64)
      cnt += __popcll(__ballot(match_rank_lds(s_idx, t0 + lane, T, K, e) >= 0));
    if (lane == 0) s_count[e] = cnt;
  }
  __syncthreads();
  if (wave == 0) {                                     // exclusive prefix over <= 256 experts
    constexpr int C = MOE_MAX_EXPERTS / 64;
    int loc[C], sum = 0;
#pragma unroll
    for (int c = 0; c < C; ++c) { const int e = lane * C + c; loc[c] = e < E ? s_count[e] : 0; sum += loc[c]; }
    int incl = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) { const int v = __shfl_up(incl, d); if (lane >= d) incl += v; }
    int run = incl - sum;
#pragma unroll
    for (int c = 0; c < C; ++c) { const int e = lane * C + c; if (e < E) s_off[e] = run; run += loc[c]; }
    if (lane == 63) s_off[E] = incl;
  }
  __syncthreads();
  for (int e = wave; e < E; e += kWaves) {
    int pos = s_off[e];
    for (int t0 = 0; t0 < T; t0 += 64) {
      const int t = t0 + lane;
      const int j = match_rank_lds(s_idx, t, T, K, e);
      const unsigned long long b = __ballot(j >= 0);
      if (j >= 0) {
        const int p = pos + __popcll(b & lanemask_lt(lane));
        sorted_token[p] = t;
        sorted_rank[p] = j;
        inv_pos[(size_t)t * K + j] = p;
      }
      pos += __popcll(b);
    }
  }
  for (int e = tid; e <= E; e += kSmallThreads) offsets[e] = s_off[e];
  const int P = s_off[E];
  for (int i = P + tid; i < T * K; i += kSmallThreads) { sorted_token[i] = -1; sorted_rank[i] = -1; }
}

// ---- large T: one workgroup per chunk of kChunk tokens ------------------------------------------
// Pass 1 counts, per chunk, the pairs of every expert (LDS integer atomics: a sum, so the result
// does not depend on their order).  Pass 2 turns the counts into each chunk's first position
// inside every expert segment, then places the chunk's pairs expert by expert with ballot
// prefixes, which keeps tokens ascending inside a segment.
constexpr int kChunk = 128;
constexpr int kCountSlab = 32 * MOE_MAX_EXPERTS;        // ints of the count table held in LDS at a time

__device__ __forceinline__ void stage_chunk(const int32_t* __restrict__ idx, const int32_t* __restrict__ k_t,
                                            int j_lo, int t0, int T, int E, int K, int* s_idx,
                                            int32_t* __restrict__ inv_pos) {
  const int n = min(kChunk, T - t0) * K;
  for (int i = threadIdx.x; i < n; i += kBigThreads) {
    const int tl = i / K, j = i - tl * K;
    int kt = k_t[t0 + tl];
    kt = kt < 0 ? 0 : (kt > K ? K : kt);
    const int e = idx[(size_t)t0 * K + i];
    const bool pair = j >= j_lo && j < kt && (unsigned)e < (unsigned)E;
    s_idx[i] = pair ? e : -1;
    if (inv_pos && !pair) inv_pos[(size_t)t0 * K + i] = -1;
  }
}

__global__ __launch_bounds__(kBigThreads) void dispatch_count_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ k_t, int j_lo, int T, int E, int K,
    int32_t* __restrict__ counts /* [chunks][E] */) {
  __shared__ int s_idx[kChunk * MOE_MAX_TOPK];
  __shared__ int s_hist[MOE_MAX_EXPERTS];
  const int t0 = blockIdx.x * kChunk;
  for (int e = threadIdx.x; e < E; e += kBigThreads) s_hist[e] = 0;
  stage_chunk(idx, k_t, j_lo, t0, T, E, K, s_idx, nullptr);
  __syncthreads();
  const int n = min(kChunk, T - t0) * K;
  for (int i = threadIdx.x; i < n; i += kBigThreads)
    if (s_idx[i] >= 0) atomicAdd(&s_hist[s_idx[i]], 1);
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += kBigThreads) counts[(size_t)blockIdx.x * E + e] = s_hist[e];
}

__global__ __launch_bounds__(kBigThreads) void dispatch_scatter_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ k_t, int j_lo, int T, int E, int K,
    const int32_t* __restrict__ counts, int n_chunks, int32_t* __restrict__ offsets,
    int32_t* __restrict__ sorted_token, int32_t* __restrict__ sorted_rank,
    int32_t* __restrict__ inv_pos) {
  __shared__ int s_idx[kChunk * MOE_MAX_TOPK];
  __shared__ int s_base[MOE_MAX_EXPERTS];       // first position of this chunk inside expert e's segment
  __shared__ int s_wsum[kBigThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = blockIdx.x, t0 = chunk * kChunk;
  stage_chunk(idx, k_t, j_lo, t0, T, E, K, s_idx, inv_pos);
  // per expert (one thread each, E <= 256 = kBigThreads): pairs in earlier chunks, pairs in all
  // chunks.  The count table goes through LDS in slabs with coalesced, independent loads (a
  // per-thread loop over global memory would pay one memory latency per chunk).
  __shared__ int s_cnt[kCountSlab];
  int before = 0, tot = 0;
  const int slab_chunks = kCountSlab / E;                  // >= 32 chunks per slab
  for (int c0 = 0; c0 < n_chunks; c0 += slab_chunks) {
    const int nc = min(slab_chunks, n_chunks - c0);
    __syncthreads();
    for (int i = tid; i < nc * E; i += kBigThreads) s_cnt[i] = counts[(size_t)c0 * E + i];
    __syncthreads();
    if (tid < E)
      for (int c = 0; c < nc; ++c) {
        const int v = s_cnt[c * E + tid];
        if (c0 + c < chunk) before += v;
        tot += v;
      }
  }
  // exclusive prefix of tot over the experts -> expert_offsets
  int incl = tot;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) { const int v = __shfl_up(incl, d); if (lane >= d) incl += v; }
  if (lane == 63) s_wsum[wave] = incl;
  __syncthreads();
  int wbase = 0, P = 0;
#pragma unroll
  for (int w = 0; w < kBigThreads / 64; ++w) { if (w < wave) wbase += s_wsum[w]; P += s_wsum[w]; }
  const int off_e = wbase + incl - tot;
  if (tid < E) {
    s_base[tid] = off_e + before;
    if (chunk == 0) offsets[tid] = off_e;
  }
  if (chunk == 0 && tid == 0) offsets[E] = P;
  __syncthreads();
  const int nt = min(kChunk, T - t0);
  // each lane keeps the selections of its two tokens (one per 64-token half of the chunk) in
  // registers, so the loop over experts is compares, a ballot and the stores
  static_assert(kChunk == 128, "two 64-token halves per chunk");
  int sel[2][MOE_MAX_TOPK];
#pragma unroll
  for (int hb = 0; hb < 2; ++hb)
#pragma unroll
    for (int j = 0; j < MOE_MAX_TOPK; ++j) {
      const int tl = hb * 64 + lane;
      sel[hb][j] = (tl < nt && j < K) ? s_idx[tl * K + j] : -1;
    }
  for (int e = wave; e < E; e += kBigThreads / 64) {
    int pos = s_base[e];
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
      int j = -1;
#pragma unroll
      for (int jj = MOE_MAX_TOPK - 1; jj >= 0; --jj) if (sel[hb][jj] == e) j = jj;
      const unsigned long long b = __ballot(j >= 0);
      if (j >= 0) {
        const int tl = hb * 64 + lane;
        const int p = pos + __popcll(b & lanemask_lt(lane));
        sorted_token[p] = t0 + tl;
        sorted_rank[p] = j;
        inv_pos[(size_t)(t0 + tl) * K + j] = p;
      }
      pos += __popcll(b);
    }
  }
  // positions beyond P are not pairs
  const int n = T * K;
  for (int i = P + chunk * kBigThreads + tid; i < n; i += n_chunks * kBigThreads) { sorted_token[i] = -1; sorted_rank[i] = -1; }
}

// T == 0: only the offsets exist
__global__ void dispatch_empty_kernel(int E, int32_t* offsets) {
  for (int e = threadIdx.x; e <= E; e += blockDim.x) offsets[e] = 0;
}

}  // namespace

int dispatch_chunks(int T) { return (T + kChunk - 1) / kChunk; }

int launch_dispatch(const moe_config& c, const int32_t* idx, const int32_t* k_t, int j_lo, int32_t* offsets,
                    int32_t* sorted_token, int32_t* sorted_rank, int32_t* inv_pos, int32_t* counts,
                    hipStream_t s) {
  if (c.T == 0) {
    hipLaunchKernelGGL(dispatch_empty_kernel, dim3(1), dim3(256), 0, s, c.E, offsets);
  } else if (c.T <= kSmallT) {
    hipLaunchKernelGGL(dispatch_small_kernel, dim3(1), dim3(kSmallThreads), 0, s, idx, k_t, j_lo, c.T, c.E,
                       c.k_big, offsets, sorted_token, sorted_rank, inv_pos);
  } else {
    const int n_chunks = dispatch_chunks(c.T);
    hipLaunchKernelGGL(dispatch_count_kernel, dim3((unsigned)n_chunks), dim3(kBigThreads), 0, s, idx, k_t,
                       j_lo, c.T, c.E, c.k_big, counts);
    hipLaunchKernelGGL(dispatch_scatter_kernel, dim3((unsigned)n_chunks), dim3(kBigThreads), 0, s, idx, k_t,
                       j_lo, c.T, c.E, c.k_big, counts, n_chunks, offsets, sorted_token, sorted_rank, inv_pos);
  }
  return hip_fail(hipGetLastError(), "dispatch launch");
}

}  // namespace mm
