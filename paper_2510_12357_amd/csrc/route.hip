// Selection stage after the router GEMM (Sec. II-A) with the big-little rule (Sec. III-A,
// Alg. 1): softmax over all experts, importance flag from the token's confidence, and the
// k_t best experts in the order (logit descending, expert id ascending).
//
// One wavefront per token; an expert row of up to 256 logits lives in registers (4 per lane)
// and every reduction is a butterfly of cross-lane shuffles.  All selection decisions are
// comparisons on the fp32 logits, so they are exact and reproducible bit for bit.
#include <math.h>

#include "internal.h"

namespace mm {
namespace {

constexpr int kPerLane = MOE_MAX_EXPERTS / 64;   // 4
constexpr int kWavesPerBlock = 4;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  return v;
}
__device__ __forceinline__ int wave_min_int(int v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v = min(v, __shfl_xor(v, d));
  return v;
}

__global__ __launch_bounds__(kWavesPerBlock * 64) void route_kernel(
    const float* __restrict__ logits, const float* __restrict__ conf, float gamma, int T, int E,
    int k_big, int k_little, int renorm, int32_t* __restrict__ idx, float* __restrict__ w,
    uint8_t* __restrict__ important, int32_t* __restrict__ k_t) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  if (t >= T) return;                                  // whole wave leaves together

  const float NINF = -INFINITY;
  float v[kPerLane];
#pragma unroll
  for (int c = 0; c < kPerLane; ++c) {
    const int e = lane + 64 * c;
    float x = (e < E) ? logits[(size_t)t * E + e] : NINF;
    v[c] = (x != x) ? NINF : x;                        // NaN counts as -inf
  }
  // softmax statistics over all E
  float m = v[0];
#pragma unroll
  for (int c = 1; c < kPerLane; ++c) m = fmaxf(m, v[c]);
  m = wave_max(m);
  float p[kPerLane];
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kPerLane; ++c) {
    const int e = lane + 64 * c;
    p[c] = (e < E && m != NINF) ? expf(v[c] - m) : 0.f;
    s += p[c];
  }
  s = wave_sum(s);
  const float inv_s = s > 0.f ? 1.f / s : 0.f;

  // Alg. 1: the little result is kept only if the confidence is strictly above gamma
  const bool imp = conf ? !(conf[t] > gamma) : true;
  const int k = imp ? k_big : k_little;

  // k rounds of "best expert not taken yet"
  unsigned taken = 0;                                  // bit c: this lane's c-th expert is taken
  float my_w = 0.f;                                    // lane j keeps the j-th weight
  int my_e = -1;
  float wsum = 0.f;
  for (int j = 0; j < k; ++j) {
    float best = NINF;
    bool any = false;
#pragma unroll
    for (int c = 0; c < kPerLane; ++c) {
      const int e = lane + 64 * c;
      if (e < E && !((taken >> c) & 1u)) { best = any ? fmaxf(best, v[c]) : v[c]; any = true; }
    }
    const float gbest = wave_max(any ? best : NINF);
    int cand = 0x7fffffff;                             // lowest expert id holding the best value
#pragma unroll
    for (int c = kPerLane - 1; c >= 0; --c) {
      const int e = lane + 64 * c;
      if (e < E && !((taken >> c) & 1u) && v[c] == gbest) cand = e;
    }
    const int sel = wave_min_int(cand);
    float psel = 0.f;
#pragma unroll
    for (int c = 0; c < kPerLane; ++c)
      if (lane + 64 * c == sel) { taken |= 1u << c; psel = p[c]; }
    psel = wave_sum(psel) * inv_s;                     // exactly one lane contributes
    wsum += psel;
    if (lane == j) { my_w = psel; my_e = sel; }
  }
  if (renorm) my_w = wsum > 0.f ? my_w / wsum : 0.f;
  if (lane < k_big) {
    idx[(size_t)t * k_big + lane] = lane < k ? my_e : -1;
    w[(size_t)t * k_big + lane] = lane < k ? my_w : 0.f;
  }
  if (lane == 0) {
    important[t] = imp ? 1 : 0;
    k_t[t] = k;
  }
}

// conf[t] = 1 / sum_v exp(z_tv - max_v z_tv): one workgroup per token, two sweeps over the row.
constexpr int kConfThreads = 256;
__global__ __launch_bounds__(kConfThreads) void confidence_kernel(const float* __restrict__ z, int V,
                                                                   float* __restrict__ conf) {
  __shared__ float s_part[kConfThreads / 64];
  const float* row = z + (size_t)blockIdx.x * V;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float m = -INFINITY;
  for (int v = tid; v < V; v += kConfThreads) m = fmaxf(m, row[v]);
  m = wave_max(m);
  if (lane == 0) s_part[wave] = m;
  __syncthreads();
  m = s_part[0];
#pragma unroll
  for (int i = 1; i < kConfThreads / 64; ++i) m = fmaxf(m, s_part[i]);
  __syncthreads();
  float s = 0.f;
  for (int v = tid; v < V; v += kConfThreads) s += expf(row[v] - m);
  s = wave_sum(s);
  if (lane == 0) s_part[wave] = s;
  __syncthreads();
  if (tid == 0) {
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < kConfThreads / 64; ++i) tot += s_part[i];
    conf[blockIdx.x] = 1.f / tot;
  }
}

}  // namespace

int launch_route(const moe_config& c, const float* conf, const float* logits, int32_t* idx, float* w,
                 uint8_t* important, int32_t* k_t, hipStream_t s) {
  if (c.T == 0) return MOE_OK;
  const unsigned grid = (unsigned)((c.T + kWavesPerBlock - 1) / kWavesPerBlock);
  hipLaunchKernelGGL(route_kernel, dim3(grid), dim3(kWavesPerBlock * 64), 0, s, logits, conf, c.gamma,
                     c.T, c.E, c.k_big, c.k_little, c.renorm, idx, w, important, k_t);
  return hip_fail(hipGetLastError(), "route_kernel launch");
}

int launch_confidence(const float* z, int T, int V, float* conf, hipStream_t s) {
  if (T == 0) return MOE_OK;
  hipLaunchKernelGGL(confidence_kernel, dim3((unsigned)T), dim3(kConfThreads), 0, s, z, V, conf);
  return hip_fail(hipGetLastError(), "confidence_kernel launch");
}

}  // namespace mm
