// Device-side pieces of the selection stage (Sec. II-A with the big-little rule of Sec. III-A,
// Alg. 1) shared by the kernels that route tokens: wave-wide reductions, the selection of one token
// by one wavefront, and the router dot products of one token.
#pragma once

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

// What one wave decides for a token: lane j < k_big holds the j-th selected expert and its routing
// weight (-1 / 0 from rank k on); k and imp are the same in all lanes.
struct Selection {
  int expert;
  float weight;
  int k;
  bool imp;
};

// One wave selects for token t.  raw[c] = logit of expert lane + 64*c (anything for e >= E).
__device__ __forceinline__ Selection select_token_values(const RouteParams& P, int t, int lane,
                                                         const float (&raw)[kPerLane]) {
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
  Selection sel;
  sel.expert = lane < k ? my_e : -1;
  sel.weight = lane < k ? my_w : 0.f;
  sel.k = k;
  sel.imp = imp;
  return sel;
}

// ... and writes the token's rows of the four output arrays.
__device__ __forceinline__ void select_token(const RouteParams& P, int t, int lane, const float (&raw)[kPerLane]) {
  const Selection sel = select_token_values(P, t, lane, raw);
  if (lane < P.k_big) {
    P.idx[(size_t)t * P.k_big + lane] = sel.expert;
    P.w[(size_t)t * P.k_big + lane] = sel.weight;
  }
  if (lane == 0) {
    P.important[t] = sel.imp ? 1 : 0;
    P.k_t[t] = sel.k;
  }
}

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

// Router logits of one token for the experts [e_begin, e_end), computed by the NWAVES waves of a
// workgroup: the waves split the experts, every wave sums its experts' dot products with the lanes
// striding the 8-element chunks of the hidden dimension (chunks lane, lane + 64, ... in ascending
// order, U chunks per trip with all loads issued before the first FMA) and reduces with the same
// shuffles everywhere, so a logit has the same bits whichever kernel calls this and however the
// experts are split.  Lane 0 of the wave that owns expert e calls store(e, logit).
template <typename S, int NWAVES, typename Store>
__device__ __forceinline__ void gate_logits_token(const S* __restrict__ xr, const S* __restrict__ Wg,
                                                  const float* __restrict__ bias, int H, int E, int e_begin,
                                                  int e_end, int wave, int lane, Store store) {
  const int nchunk = H >> 3;
  constexpr int U = sizeof(S) == 2 ? 4 : 2;
  constexpr int TE = 4;                                // experts per pass of a wave
  for (int e0 = e_begin + wave * TE; e0 < e_end; e0 += NWAVES * TE) {
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
      if (lane == 0 && e < e_end) store(e, sum + (bias ? bias[e] : 0.f));
    }
  }
}

}  // namespace
}  // namespace mm
