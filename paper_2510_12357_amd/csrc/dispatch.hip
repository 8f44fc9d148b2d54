// Token-to-expert dispatch with a variable expert count per token (k_t = k_big for important
// tokens, k_little otherwise; Sec. III-A).  The execution stage (Sec. II-A) wants the
// (token, rank) pairs grouped per expert; the order is fixed to (expert asc, token asc), i.e. a
// stable counting sort of the pair list by expert id.
//
// The sort is done without atomics: expert e's segment is produced by scanning the tokens in
// ascending order and compacting the matches with ballot/popcount prefix sums, so the result is
// unique and reproducible.  Two shapes:
//   * T <= kSmallT: one workgroup, one wave per expert (round-robin), one launch.
//   * larger T: one workgroup per expert; a count kernel, then a scatter kernel that rebuilds
//     the exclusive prefix of the counts itself.
#include "internal.h"

namespace mm {
namespace {

constexpr int kSmallT = 256;
constexpr int kSmallThreads = 1024;
constexpr int kBigThreads = 256;

__device__ __forceinline__ unsigned long long lanemask_lt(int lane) {
  return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

// does token t route to expert e?  returns the rank j or -1
__device__ __forceinline__ int match_rank(const int32_t* __restrict__ idx, const int32_t* __restrict__ k_t,
                                          int t, int T, int K, int e) {
  if (t >= T) return -1;
  int kt = k_t[t];
  kt = kt < 0 ? 0 : (kt > K ? K : kt);
  int found = -1;
  for (int j = 0; j < kt; ++j)
    if (found < 0 && idx[(size_t)t * K + j] == e) found = j;
  return found;
}

// -1 fill of everything that is not a pair: positions >= P and ranks >= k_t
__device__ __forceinline__ void fill_pads(int first, int stride, int P, int T, int E, int K,
                                          const int32_t* __restrict__ idx,
                                          const int32_t* __restrict__ k_t, int32_t* sorted_token,
                                          int32_t* sorted_rank, int32_t* inv_pos) {
  const int n = T * K;
  for (int i = first; i < n; i += stride) {
    if (i >= P) { sorted_token[i] = -1; sorted_rank[i] = -1; }
    const int t = i / K, j = i - t * K;
    int kt = k_t[t];
    kt = kt < 0 ? 0 : (kt > K ? K : kt);
    // ranks beyond k_t, and pairs naming an expert id outside [0,E), are not dispatched
    if (j >= kt || (unsigned)idx[i] >= (unsigned)E) inv_pos[i] = -1;
  }
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
    const int32_t* __restrict__ idx, const int32_t* __restrict__ k_t, int T, int E, int K,
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
    const bool pair = j < kt && (unsigned)e < (unsigned)E;
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

// ---- large T: one workgroup per expert -----------------------------------------------------
__device__ __forceinline__ int block_sum(int v, int* s_tmp) {   // kBigThreads threads
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  __syncthreads();
  if (lane == 0) s_tmp[wave] = v;
  __syncthreads();
  int tot = 0;
#pragma unroll
  for (int w = 0; w < kBigThreads / 64; ++w) tot += s_tmp[w];
  return tot;
}

__global__ __launch_bounds__(kBigThreads) void dispatch_count_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ k_t, int T, int K,
    int32_t* __restrict__ counts) {
  __shared__ int s_tmp[kBigThreads / 64];
  const int e = blockIdx.x;
  int cnt = 0;
  for (int t0 = 0; t0 < T; t0 += kBigThreads)
    cnt += match_rank(idx, k_t, t0 + threadIdx.x, T, K, e) >= 0 ? 1 : 0;
  cnt = block_sum(cnt, s_tmp);
  if (threadIdx.x == 0) counts[e] = cnt;
}

__global__ __launch_bounds__(kBigThreads) void dispatch_scatter_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ k_t, int T, int E, int K,
    const int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
    int32_t* __restrict__ sorted_token, int32_t* __restrict__ sorted_rank,
    int32_t* __restrict__ inv_pos) {
  __shared__ int s_tmp[kBigThreads / 64];
  __shared__ int s_wave[kBigThreads / 64];
  const int e = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // exclusive prefix of the counts up to e, and the total P (E <= 256 = one entry per thread)
  const int mine = tid < E ? counts[tid] : 0;
  const int before = block_sum(tid < e ? mine : 0, s_tmp);
  const int P = block_sum(mine, s_tmp);
  if (tid == 0) {
    offsets[e] = before;
    if (e == E - 1) offsets[E] = P;
  }
  int pos = before;
  for (int t0 = 0; t0 < T; t0 += kBigThreads) {
    const int t = t0 + tid;
    const int j = match_rank(idx, k_t, t, T, K, e);
    const unsigned long long b = __ballot(j >= 0);
    if (lane == 0) s_wave[wave] = __popcll(b);
    __syncthreads();
    int wbase = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kBigThreads / 64; ++w) { if (w < wave) wbase += s_wave[w]; tot += s_wave[w]; }
    if (j >= 0) {
      const int p = pos + wbase + __popcll(b & lanemask_lt(lane));
      sorted_token[p] = t;
      sorted_rank[p] = j;
      inv_pos[(size_t)t * K + j] = p;
    }
    pos += tot;
    __syncthreads();
  }
  fill_pads(e * kBigThreads + tid, E * kBigThreads, P, T, E, K, idx, k_t, sorted_token, sorted_rank, inv_pos);
}

// T == 0: only the offsets exist
__global__ void dispatch_empty_kernel(int E, int32_t* offsets) {
  for (int e = threadIdx.x; e <= E; e += blockDim.x) offsets[e] = 0;
}

}  // namespace

int launch_dispatch(const moe_config& c, const int32_t* idx, const int32_t* k_t, int32_t* offsets,
                    int32_t* sorted_token, int32_t* sorted_rank, int32_t* inv_pos, int32_t* counts,
                    hipStream_t s) {
  if (c.T == 0) {
    hipLaunchKernelGGL(dispatch_empty_kernel, dim3(1), dim3(256), 0, s, c.E, offsets);
  } else if (c.T <= kSmallT) {
    hipLaunchKernelGGL(dispatch_small_kernel, dim3(1), dim3(kSmallThreads), 0, s, idx, k_t, c.T, c.E,
                       c.k_big, offsets, sorted_token, sorted_rank, inv_pos);
  } else {
    hipLaunchKernelGGL(dispatch_count_kernel, dim3((unsigned)c.E), dim3(kBigThreads), 0, s, idx, k_t,
                       c.T, c.k_big, counts);
    hipLaunchKernelGGL(dispatch_scatter_kernel, dim3((unsigned)c.E), dim3(kBigThreads), 0, s, idx, k_t,
                       c.T, c.E, c.k_big, counts, offsets, sorted_token, sorted_rank, inv_pos);
  }
  return hip_fail(hipGetLastError(), "dispatch launch");
}

}  // namespace mm
