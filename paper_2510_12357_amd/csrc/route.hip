// Selection stage (Sec. II-A) with the big-little rule (Sec. III-A, Alg. 1): softmax over all
// experts, importance flag from the token's confidence, and the k_t best experts in the order
// (logit descending, expert id ascending).
//
// Selection runs in one wavefront per token; an expert row of up to 256 logits lives in
// registers (4 per lane) and every reduction is a butterfly of cross-lane shuffles.  All
// selection decisions are comparisons on the fp32 logits, so they are exact and reproducible.
//
// Kernels:
//   gate_route_kernel router logits and selection of one token per workgroup (decode batches)
//   gate_gemv_kernel  router logits alone (up to 256 tokens): plain fp32 FMAs, one wave per
//                     small block of logits, so that even one token spreads over E waves
//   route_kernel      softmax / importance / top-k on given logits
#include "internal.h"
#include "route_device.h"

namespace mm {
namespace {

__global__ __launch_bounds__(kWavesPerBlock * 64) void route_kernel(const float* __restrict__ logits,
                                                                     const RouteParams P) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  if (t >= P.T) return;                                // whole wave leaves together
  float raw[kPerLane];
#pragma unroll
  for (int c = 0; c < kPerLane; ++c) {
    const int e = lane + 64 * c;
    raw[c] = (e < P.E) ? logits[(size_t)t * P.E + e] : 0.f;
  }
  select_token(P, t, lane, raw);
}

// One wave per block of TE experts x TT tokens: the lanes split the hidden dimension, every
// operand chunk is a 16/32-byte load, and the block's sums are reduced with shuffles.  Decode
// batches give E*T/(TE*TT) waves, enough to pull the gate matrix at full speed.
constexpr int kGemvWaves = 4;

template <typename S, int TE, int TT>
__global__ __launch_bounds__(kGemvWaves * 64) void gate_gemv_kernel(const S* __restrict__ x,
                                                                     const S* __restrict__ Wg,
                                                                     const float* __restrict__ bias, int T,
                                                                     int H, int E,
                                                                     float* __restrict__ logits) {
  const int lane = threadIdx.x & 63;
  const int wid = blockIdx.x * kGemvWaves + (threadIdx.x >> 6);
  const int n_eb = (E + TE - 1) / TE, n_tb = (T + TT - 1) / TT;
  if (wid >= n_eb * n_tb) return;                      // whole wave leaves together
  const int e0 = (wid % n_eb) * TE, t0 = (wid / n_eb) * TT;
  float acc[TE][TT];
#pragma unroll
  for (int a = 0; a < TE; ++a)
#pragma unroll
    for (int b = 0; b < TT; ++b) acc[a][b] = 0.f;
  const int nchunk = H >> 3;                           // 8 elements per chunk
  // U chunks per trip with all loads issued before the first FMA: a lane has only H/512 chunks,
  // so with one chunk per trip the kernel would be a chain of exposed load latencies.  The FMA
  // order per accumulator (chunks ascending) is the same for every U.
  constexpr int U = sizeof(S) == 2 ? 4 : 2;
  for (int c0 = lane; c0 < nchunk; c0 += 64 * U) {
    Raw8<S> xr[U][TT], wr[U][TE];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int c = min(c0 + 64 * u, nchunk - 1);      // a chunk past the end is loaded again and skipped
#pragma unroll
      for (int b = 0; b < TT; ++b) xr[u][b].load(x + (size_t)min(t0 + b, T - 1) * H + c * 8);
#pragma unroll
      for (int a = 0; a < TE; ++a) wr[u][a].load(Wg + (size_t)min(e0 + a, E - 1) * H + c * 8);   // clamped rows are discarded below
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (c0 + 64 * u < nchunk) {
        float xv[TT][8];
#pragma unroll
        for (int b = 0; b < TT; ++b) xr[u][b].get(xv[b]);
#pragma unroll
        for (int a = 0; a < TE; ++a) {
          float wv[8];
          wr[u][a].get(wv);
#pragma unroll
          for (int b = 0; b < TT; ++b)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[a][b] = fmaf(xv[b][i], wv[i], acc[a][b]);
        }
      }
    }
  }
#pragma unroll
  for (int a = 0; a < TE; ++a)
#pragma unroll
    for (int b = 0; b < TT; ++b) {
      const float sum = wave_sum(acc[a][b]);
      const int e = e0 + a, t = t0 + b;
      if (lane == 0 && e < E && t < T) logits[(size_t)t * E + e] = sum + (bias ? bias[e] : 0.f);
    }
}

template <typename S, int TE, int TT>
void launch_gemv(const moe_config& c, const void* x, const void* Wg, const float* bias, float* logits,
                 hipStream_t s) {
  const int waves = ((c.E + TE - 1) / TE) * ((c.T + TT - 1) / TT);
  hipLaunchKernelGGL((gate_gemv_kernel<S, TE, TT>), dim3((unsigned)((waves + kGemvWaves - 1) / kGemvWaves)),
                     dim3(kGemvWaves * 64), 0, s, static_cast<const S*>(x), static_cast<const S*>(Wg), bias,
                     c.T, c.H, c.E, logits);
}

// Router logits and selection of one token in one workgroup (decode batches): the waves split the
// experts, every wave sums its experts' dot products exactly as gate_gemv_kernel does (per lane
// the 8-element chunks lane, lane + 64, ... in ascending order, then the same shuffle reduction),
// so the logits are bit-identical to that kernel's; they go to global memory and to LDS, and wave
// 0 selects from LDS.  One launch instead of two dependent ones.
constexpr int kFusedWaves = 16;

template <typename S>
__global__ __launch_bounds__(kFusedWaves * 64) void gate_route_kernel(const S* __restrict__ x,
                                                                       const S* __restrict__ Wg,
                                                                       const float* __restrict__ bias, int H,
                                                                       float* __restrict__ logits,
                                                                       const RouteParams P) {
  __shared__ float s_logit[MOE_MAX_EXPERTS];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x, E = P.E;
  float* const logits_row = logits + (size_t)t * E;
  gate_logits_token<S, kFusedWaves>(x + (size_t)t * H, Wg, bias, H, E, 0, E, wave, lane,
                                    [&](int e, float z) { logits_row[e] = z; s_logit[e] = z; });
  __syncthreads();
  if (wave != 0) return;
  float raw[kPerLane];
#pragma unroll
  for (int c = 0; c < kPerLane; ++c) {
    const int e = lane + 64 * c;
    raw[c] = (e < E) ? s_logit[e] : 0.f;
  }
  select_token(P, t, lane, raw);
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

RouteParams make_params(const moe_config& c, const float* conf, int32_t* idx, float* w, uint8_t* important,
                        int32_t* k_t) {
  RouteParams P;
  P.conf = conf; P.gamma = c.gamma; P.T = c.T; P.E = c.E; P.k_big = c.k_big; P.k_little = c.k_little;
  P.renorm = c.renorm; P.idx = idx; P.w = w; P.important = important; P.k_t = k_t;
  return P;
}

}  // namespace

int launch_route(const moe_config& c, const float* conf, const float* logits, int32_t* idx, float* w,
                 uint8_t* important, int32_t* k_t, hipStream_t s) {
  if (c.T == 0) return MOE_OK;
  const unsigned grid = (unsigned)((c.T + kWavesPerBlock - 1) / kWavesPerBlock);
  hipLaunchKernelGGL(route_kernel, dim3(grid), dim3(kWavesPerBlock * 64), 0, s, logits,
                     make_params(c, conf, idx, w, important, k_t));
  return hip_fail(hipGetLastError(), "route_kernel launch");
}

// Router logits + selection in one launch; for steps of at most kFusedRouteMaxT tokens.
int launch_gate_route(const moe_config& c, const void* x, const void* Wg, const float* bias, const float* conf,
                      float* logits, int32_t* idx, float* w, uint8_t* important, int32_t* k_t, hipStream_t s) {
  if (c.T == 0) return MOE_OK;
  const RouteParams P = make_params(c, conf, idx, w, important, k_t);
  if (c.dtype != MOE_FP32)
    hipLaunchKernelGGL(gate_route_kernel<uint16_t>, dim3((unsigned)c.T), dim3(kFusedWaves * 64), 0, s,
                       static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(Wg), bias, c.H, logits, P);
  else
    hipLaunchKernelGGL(gate_route_kernel<float>, dim3((unsigned)c.T), dim3(kFusedWaves * 64), 0, s,
                       static_cast<const float*>(x), static_cast<const float*>(Wg), bias, c.H, logits, P);
  return hip_fail(hipGetLastError(), "gate_route_kernel launch");
}

int launch_gate_gemv(const moe_config& c, const void* x, const void* Wg, const float* bias, float* logits,
                     hipStream_t s) {
  if (c.T == 0) return MOE_OK;
  const bool bf = c.dtype != MOE_FP32;
  if (c.T <= 4) {
    if (bf) launch_gemv<uint16_t, 1, 1>(c, x, Wg, bias, logits, s); else launch_gemv<float, 1, 1>(c, x, Wg, bias, logits, s);
  } else if (c.T <= 32) {
    if (bf) launch_gemv<uint16_t, 1, 4>(c, x, Wg, bias, logits, s); else launch_gemv<float, 1, 4>(c, x, Wg, bias, logits, s);
  } else {
    if (bf) launch_gemv<uint16_t, 2, 4>(c, x, Wg, bias, logits, s); else launch_gemv<float, 2, 4>(c, x, Wg, bias, logits, s);
  }
  return hip_fail(hipGetLastError(), "gate_gemv_kernel launch");
}

int launch_confidence(const float* z, int T, int V, float* conf, hipStream_t s) {
  if (T == 0) return MOE_OK;
  hipLaunchKernelGGL(confidence_kernel, dim3((unsigned)T), dim3(kConfThreads), 0, s, z, V, conf);
  return hip_fail(hipGetLastError(), "confidence_kernel launch");
}

}  // namespace mm
