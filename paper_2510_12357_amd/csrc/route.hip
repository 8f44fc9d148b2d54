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
#include <math.h>

#include <type_traits>

#include "internal.h"

namespace mm {
namespace {

constexpr int kPerLane = MOE_MAX_EXPERTS / 64;   // 4
constexpr int kWavesPerBlock = 4;

// Wave-wide reductions on the data-parallel-primitive path (no LDS round trips): quads, half
// rows and rows with quad_perm / row_half_mirror / row_mirror, then lane 15 of a row into the
// next row and lane 31 into rows 2 and 3, so that lane 63 holds the result, which is read back
// as a scalar.  `ident` is what a lane outside the row mask contributes.
template <typename T, typename Op>
__device__ __forceinline__ T wave_reduce(T v, T ident, Op op) {
  const auto dpp = [](T old, T x, auto ctrl, auto rows) {
    const int r = __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old), __builtin_bit_cast(int, x),
                                              decltype(ctrl)::value, decltype(rows)::value, 0xf, false);
    return __builtin_bit_cast(T, r);
  };
  using std::integral_constant;
  v = op(v, dpp(v, v, integral_constant<int, 0xB1>{}, integral_constant<int, 0xf>{}));    // quad_perm [1,0,3,2]
  v = op(v, dpp(v, v, integral_constant<int, 0x4E>{}, integral_constant<int, 0xf>{}));    // quad_perm [2,3,0,1]
  v = op(v, dpp(v, v, integral_constant<int, 0x141>{}, integral_constant<int, 0xf>{}));   // row_half_mirror
  v = op(v, dpp(v, v, integral_constant<int, 0x140>{}, integral_constant<int, 0xf>{}));   // row_mirror
  v = op(v, dpp(ident, v, integral_constant<int, 0x142>{}, integral_constant<int, 0xa>{}));   // row_bcast:15 into rows 1, 3
  v = op(v, dpp(ident, v, integral_constant<int, 0x143>{}, integral_constant<int, 0xc>{}));   // row_bcast:31 into rows 2, 3
  return __builtin_bit_cast(T, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
  return wave_reduce(v, -INFINITY, [](float a, float b) { return fmaxf(a, b); });
}
__device__ __forceinline__ float wave_sum(float v) {
  return wave_reduce(v, 0.f, [](float a, float b) { return a + b; });
}
__device__ __forceinline__ int wave_min_int(int v) {
  return wave_reduce(v, 0x7fffffff, [](int a, int b) { return min(a, b); });
}

struct RouteParams {
  const float* conf;
  float gamma;
  int T, E, k_big, k_little, renorm;
  int32_t* idx;
  float* w;
  uint8_t* important;
  int32_t* k_t;
};

// One wave selects for token t.  raw[c] = logit of expert lane + 64*c (anything for e >= E).
__device__ __forceinline__ void select_token(const RouteParams& P, int t, int lane, const float (&raw)[kPerLane]) {
  const float NINF = -INFINITY;
  const int E = P.E;
  float v[kPerLane];
#pragma unroll
  for (int c = 0; c < kPerLane; ++c) {
    const float x = (lane + 64 * c < E) ? raw[c] : NINF;
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
    p[c] = (lane + 64 * c < E && m != NINF) ? expf(v[c] - m) : 0.f;
    s += p[c];
  }
  s = wave_sum(s);
  const float inv_s = s > 0.f ? 1.f / s : 0.f;

  // Alg. 1: the little result is kept only if the confidence is strictly above gamma
  const bool imp = P.conf ? !(P.conf[t] > P.gamma) : true;
  const int k = imp ? P.k_big : P.k_little;

  // k rounds of "best expert not taken yet"
  unsigned taken = 0;                                  // bit c: this lane's c-th expert is taken
  float my_w = 0.f;                                    // lane j keeps the j-th weight
  int my_e = -1;
  float wsum = 0.f;
  for (int j = 0; j < k; ++j) {
    float best = NINF;
    bool any = false;
#pragma unroll
    for (int c = 0; c < kPerLane; ++c)
      if (lane + 64 * c < E && !((taken >> c) & 1u)) { best = any ? fmaxf(best, v[c]) : v[c]; any = true; }
    const float gbest = wave_max(any ? best : NINF);
    int cand = 0x7fffffff;                             // lowest expert id holding the best value
#pragma unroll
    for (int c = kPerLane - 1; c >= 0; --c)
      if (lane + 64 * c < E && !((taken >> c) & 1u) && v[c] == gbest) cand = lane + 64 * c;
    const int sel = wave_min_int(cand);
    float psel = 0.f;
#pragma unroll
    for (int c = 0; c < kPerLane; ++c)
      if (lane + 64 * c == sel) { taken |= 1u << c; psel = p[c]; }
    psel = wave_sum(psel) * inv_s;                     // exactly one lane contributes
    wsum += psel;
    if (lane == j) { my_w = psel; my_e = sel; }
  }
  if (P.renorm) my_w = wsum > 0.f ? my_w / wsum : 0.f;
  if (lane < P.k_big) {
    P.idx[(size_t)t * P.k_big + lane] = lane < k ? my_e : -1;
    P.w[(size_t)t * P.k_big + lane] = lane < k ? my_w : 0.f;
  }
  if (lane == 0) {
    P.important[t] = imp ? 1 : 0;
    P.k_t[t] = k;
  }
}

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

// ---- fused router for decode sizes ----------------------------------------------------------
// Eight consecutive elements as loaded (16 or 32 bytes), converted to fp32 on demand.
template <typename S> struct Raw8;
template <> struct Raw8<uint16_t> {
  uint4 u;
  __device__ __forceinline__ void load(const uint16_t* p) { u = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void get(float (&f)[8]) const {
    const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);            // bf16 -> fp32 is a 16-bit shift
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};
template <> struct Raw8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = *reinterpret_cast<const float4*>(p); b = *reinterpret_cast<const float4*>(p + 4);
  }
  __device__ __forceinline__ void get(float (&f)[8]) const {
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
  }
};

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
  const S* xr = x + (size_t)t * H;
  const int nchunk = H >> 3;
  constexpr int U = sizeof(S) == 2 ? 4 : 2;
  constexpr int TE = 4;                                // experts per pass of a wave
  for (int e0 = wave * TE; e0 < E; e0 += kFusedWaves * TE) {
    float acc[TE];
#pragma unroll
    for (int a = 0; a < TE; ++a) acc[a] = 0.f;
    for (int c0 = lane; c0 < nchunk; c0 += 64 * U) {
      Raw8<S> xv[U], wv[U][TE];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int c = min(c0 + 64 * u, nchunk - 1);    // a chunk past the end is loaded again and skipped
        xv[u].load(xr + c * 8);
#pragma unroll
        for (int a = 0; a < TE; ++a) wv[u][a].load(Wg + (size_t)min(e0 + a, E - 1) * H + c * 8);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (c0 + 64 * u < nchunk) {
          float xf[8];
          xv[u].get(xf);
#pragma unroll
          for (int a = 0; a < TE; ++a) {
            float wf[8];
            wv[u][a].get(wf);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[a] = fmaf(xf[i], wf[i], acc[a]);
          }
        }
      }
    }
#pragma unroll
    for (int a = 0; a < TE; ++a) {
      const float sum = wave_sum(acc[a]);
      const int e = e0 + a;
      if (lane == 0 && e < E) {
        const float z = sum + (bias ? bias[e] : 0.f);
        logits[(size_t)t * E + e] = z;
        s_logit[e] = z;
      }
    }
  }
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
