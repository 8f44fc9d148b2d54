// CPU oracle for the big-little MoE layer (MoBiLE, arXiv 2510.12357).
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the layer
// computes.  It shares no code with the HIP library and must never be called from the
// product path; only tests, the smoke check and the benchmark's CPU-baseline leg use it.
//
// Everything floating point is evaluated in double.  Router logits are the one exception:
// they are stored as fp32 because the expert selection is defined on the fp32 logits
// (both the oracle and the GPU path take that integer decision on the same fp32 values).
//
// No blocking, fusion or reordering: every function is the loop nest of its definition.
// Rows of independent work are spread over host threads with OpenMP; the arithmetic of a
// single output element is never split.
//
// Passages followed (paper sections):
//   Sec. II-A   selection stage (router picks experts, yields routing weights) and
//               execution stage (hidden states through the selected experts, summed)
//   Sec. III-A  big model = K experts, little model = K/2 experts of the same layer
//   Alg. 1      keep the little result iff max(p) > gamma, otherwise fall back to big
//   Sec. III-B  the confidence is the highest probability of the output distribution
//
// Parity pins: see tests/test_oracle_*.py (brute-force dense evaluation, textbook top-K,
// closed forms, structural invariants).  No function here is unpinned.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// dtype codes of the storage formats the oracle can read
constexpr int kBF16 = 0;   // uint16 holding the upper half of an IEEE fp32
constexpr int kFP32 = 1;

inline double load_elem(const void* base, size_t i, int dtype) {
  if (dtype == kFP32) return (double)static_cast<const float*>(base)[i];
  uint32_t bits = (uint32_t)static_cast<const uint16_t*>(base)[i] << 16;
  float f;
  std::memcpy(&f, &bits, sizeof f);
  return (double)f;
}

inline size_t elem_size(int dtype) { return dtype == kFP32 ? 4 : 2; }

// 8-bit float E4M3 of the OCP 8-bit floating point specification ("e4m3fn"): 1 sign, 4 exponent
// (bias 7), 3 mantissa bits; no infinities; S.1111.111 is NaN; exponent field 0 is subnormal.
inline double e4m3_value(uint8_t b) {
  const int sign = b >> 7, e = (b >> 3) & 15, m = b & 7;
  double v;
  if (e == 15 && m == 7) v = std::numeric_limits<double>::quiet_NaN();
  else if (e == 0) v = std::ldexp((double)m, -9);            // (m / 8) * 2^-6
  else v = std::ldexp(1.0 + m / 8.0, e - 7);
  return sign ? -v : v;
}

// 4-bit float E2M1 of the OCP microscaling formats (the element type of MXFP4): 1 sign, 2 exponent
// (bias 1), 1 mantissa bit; no infinities, no NaN; exponent field 0 is subnormal (0 or 0.5).
inline double e2m1_value(unsigned code) {
  const int sign = (code >> 3) & 1, e = (code >> 1) & 3, m = code & 1;
  const double v = e == 0 ? 0.5 * m : std::ldexp(1.0 + 0.5 * m, e - 1);
  return sign ? -v : v;
}

// E8M0, the scale type of the microscaling formats: an unsigned exponent with bias 127; 255 is NaN.
inline double e8m0_value(uint8_t b) {
  return b == 255 ? std::numeric_limits<double>::quiet_NaN() : std::ldexp(1.0, (int)b - 127);
}

// Element k of a row of MXFP4 data: codes two per byte (even k in the low four bits), one scale
// per block of 32 consecutive k.
inline double mx4_elem(const uint8_t* codes, const uint8_t* scales, size_t row, size_t k, size_t K) {
  const uint8_t byte = codes[(row * K + k) >> 1];
  const unsigned code = (k & 1) ? (byte >> 4) : (byte & 15);
  return e8m0_value(scales[(row * K + k) >> 5]) * e2m1_value(code);
}

// NaN router scores take part in selection and softmax as minus infinity.
inline double clean_logit(float v) {
  return std::isnan(v) ? -std::numeric_limits<double>::infinity() : (double)v;
}

}  // namespace

extern "C" {

// Sec. II-A, selection stage: logits[t][e] = sum_h x[t][h] * Wg[e][h] (+ bias[e]).
// x [T,H], Wg [E,H] row-major in `dtype`; bias fp32 or NULL; logits fp32 [T,E].
int oracle_gate_logits(const void* x, const void* Wg, const float* bias, int T, int H, int E,
                       int dtype, float* logits) {
  if (!x || !Wg || !logits || T < 0 || H <= 0 || E <= 0) return -1;
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    for (int e = 0; e < E; ++e) {
      double acc = 0.0;
      for (int h = 0; h < H; ++h)
        acc += load_elem(x, (size_t)t * H + h, dtype) * load_elem(Wg, (size_t)e * H + h, dtype);
      if (bias) acc += (double)bias[e];
      logits[(size_t)t * E + e] = (float)acc;
    }
  }
  return 0;
}

// Sec. III-B / Alg. 1: confidence of a token = largest probability of softmax(z_t)
//   = 1 / sum_v exp(z_tv - max_v z_tv).
int oracle_token_confidence(const float* lm_logits, int T, int V, float* conf) {
  if (!lm_logits || !conf || T < 0 || V <= 0) return -1;
  for (int t = 0; t < T; ++t) {
    const float* z = lm_logits + (size_t)t * V;
    double m = -std::numeric_limits<double>::infinity();
    for (int v = 0; v < V; ++v) m = std::fmax(m, (double)z[v]);
    double s = 0.0;
    for (int v = 0; v < V; ++v) s += std::exp((double)z[v] - m);
    conf[t] = (float)(1.0 / s);
  }
  return 0;
}

// Alg. 1 (test max(p) > gamma) + Sec. III-A (K vs K/2 experts) + Sec. II-A (routing weights).
//   important[t] = !(conf[t] > gamma)   (conf == NULL: every token important)
//   k_t[t]       = important ? k_big : k_little
//   idx[t][j]    = j-th expert of token t in the order (logit descending, index ascending),
//                  j < k_t; -1 beyond
//   w[t][j]      = softmax over ALL E logits, taken at idx[t][j]; with renorm != 0 divided
//                  by the sum over the k_t selected; 0 beyond k_t
int oracle_route(const float* logits, const float* conf, float gamma, int T, int E, int k_big,
                 int k_little, int renorm, int32_t* idx, float* w, uint8_t* important,
                 int32_t* k_t) {
  if (!logits || !idx || !w || !important || !k_t) return -1;
  if (T < 0 || E <= 0 || k_little < 1 || k_little > k_big || k_big > E) return -1;
  const double ninf = -std::numeric_limits<double>::infinity();
  for (int t = 0; t < T; ++t) {
    const float* row = logits + (size_t)t * E;
    const bool imp = conf ? !(conf[t] > gamma) : true;
    important[t] = imp ? 1 : 0;
    const int k = imp ? k_big : k_little;
    k_t[t] = k;

    // softmax over all experts
    std::vector<double> p(E);
    double m = ninf;
    for (int e = 0; e < E; ++e) m = std::fmax(m, clean_logit(row[e]));
    double s = 0.0;
    for (int e = 0; e < E; ++e) {
      p[e] = (m == ninf) ? 0.0 : std::exp(clean_logit(row[e]) - m);
      s += p[e];
    }
    for (int e = 0; e < E; ++e) p[e] = (s > 0.0) ? p[e] / s : 0.0;

    // plain selection: k rounds of "best expert not taken yet"
    std::vector<char> taken(E, 0);
    double wsum = 0.0;
    for (int j = 0; j < k_big; ++j) {
      if (j >= k) {
        idx[(size_t)t * k_big + j] = -1;
        w[(size_t)t * k_big + j] = 0.0f;
        continue;
      }
      int best = -1;
      for (int e = 0; e < E; ++e) {
        if (taken[e]) continue;
        if (best < 0 || clean_logit(row[e]) > clean_logit(row[best])) best = e;  // ties keep lower e
      }
      taken[best] = 1;
      idx[(size_t)t * k_big + j] = best;
      wsum += p[best];
    }
    for (int j = 0; j < k; ++j) {
      double v = p[idx[(size_t)t * k_big + j]];
      if (renorm) v = (wsum > 0.0) ? v / wsum : 0.0;
      w[(size_t)t * k_big + j] = (float)v;
    }
  }
  return 0;
}

// Execution stage needs the (token, rank) pairs grouped per expert.  The order is fixed:
// expert ascending, then token ascending (a token names an expert at most once).
//   offsets[E+1]      exclusive prefix of per-expert pair counts, offsets[E] = P
//   sorted_token[p]   token of the pair at position p      (-1 for p >= P)
//   sorted_rank[p]    its rank j in the token's selection  (-1 for p >= P)
//   inv_pos[t][j]     position of pair (t, j)              (-1 for j >= k_t)
// Dispatch of the ranks j_lo <= j < k_t[t] only.  j_lo = 0 is the dispatch of a whole step; j_lo =
// k_little is the re-do of a token whose little result was rejected (Alg. 1, Sec. III-B) when the
// experts of ranks below k_little have been computed already: the big model's expert set is the
// little one's plus the ranks k_little .. K-1 (Sec. III-A: same router, K instead of K/2 experts).
int oracle_dispatch_from(const int32_t* idx, const int32_t* k_t, int j_lo, int T, int E, int K,
                         int32_t* offsets, int32_t* sorted_token, int32_t* sorted_rank, int32_t* inv_pos) {
  if (!idx || !k_t || !offsets || !sorted_token || !sorted_rank || !inv_pos || j_lo < 0) return -1;
  for (size_t i = 0; i < (size_t)T * K; ++i) {
    sorted_token[i] = -1;
    sorted_rank[i] = -1;
    inv_pos[i] = -1;
  }
  int pos = 0;
  for (int e = 0; e < E; ++e) {
    offsets[e] = pos;
    for (int t = 0; t < T; ++t) {
      for (int j = j_lo; j < k_t[t]; ++j) {
        if (idx[(size_t)t * K + j] == e) {
          sorted_token[pos] = t;
          sorted_rank[pos] = j;
          inv_pos[(size_t)t * K + j] = pos;
          ++pos;
        }
      }
    }
  }
  offsets[E] = pos;
  return 0;
}

int oracle_dispatch(const int32_t* idx, const int32_t* k_t, int T, int E, int K, int32_t* offsets,
                    int32_t* sorted_token, int32_t* sorted_rank, int32_t* inv_pos) {
  if (!idx || !k_t || !offsets || !sorted_token || !sorted_rank || !inv_pos) return -1;
  for (size_t i = 0; i < (size_t)T * K; ++i) {
    sorted_token[i] = -1;
    sorted_rank[i] = -1;
    inv_pos[i] = -1;
  }
  int pos = 0;
  for (int e = 0; e < E; ++e) {
    offsets[e] = pos;
    for (int t = 0; t < T; ++t) {
      for (int j = 0; j < k_t[t]; ++j) {
        if (idx[(size_t)t * K + j] == e) {
          sorted_token[pos] = t;
          sorted_rank[pos] = j;
          inv_pos[(size_t)t * K + j] = pos;
          ++pos;
        }
      }
    }
  }
  offsets[E] = pos;
  return 0;
}

// SwiGLU feed-forward of one expert on a list of token rows.
//   blob = [W_gate I x H | W_up I x H | W_down H x I], each row-major, in `dtype`
//   for row r (token tok[r], or r itself when tok == NULL):
//     g_i = sum_h W_gate[i][h] x[h];  u_i = sum_h W_up[i][h] x[h]
//     a_i = g_i / (1 + exp(-g_i)) * u_i
//     y[r][c] = sum_i W_down[c][i] a_i
// y is double [n,H].
int oracle_swiglu_rows(const void* x, int dtype, int H, int I, const void* blob,
                       const int32_t* tok, int n, double* y) {
  if (!x || !blob || !y || H <= 0 || I <= 0 || n < 0) return -1;
  const char* base = static_cast<const char*>(blob);
  const void* Wgate = base;
  const void* Wup = base + (size_t)I * H * elem_size(dtype);
  const void* Wdown = base + 2 * (size_t)I * H * elem_size(dtype);
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < n; ++r) {
    const size_t t = tok ? (size_t)tok[r] : (size_t)r;
    std::vector<double> a(I);
    for (int i = 0; i < I; ++i) {
      double g = 0.0, u = 0.0;
      for (int h = 0; h < H; ++h) {
        const double xv = load_elem(x, t * H + h, dtype);
        g += load_elem(Wgate, (size_t)i * H + h, dtype) * xv;
        u += load_elem(Wup, (size_t)i * H + h, dtype) * xv;
      }
      a[i] = g / (1.0 + std::exp(-g)) * u;
    }
    for (int c = 0; c < H; ++c) {
      double acc = 0.0;
      for (int i = 0; i < I; ++i) acc += load_elem(Wdown, (size_t)c * I + i, dtype) * a[i];
      y[(size_t)r * H + c] = acc;
    }
  }
  return 0;
}

// The same feed-forward with the expert's weights stored in 8 bits (weight-only quantisation,
// activations in `xdtype`):
//   blob = [Q_gate I x H | Q_up I x H | Q_down H x I] one E4M3 byte per weight, followed by the
//          fp32 row scales [s_gate I | s_up I | s_down H];  W[r][k] = s[r] * e4m3(Q[r][k])
int oracle_swiglu_rows_w8(const void* x, int xdtype, int H, int I, const void* blob,
                          const int32_t* tok, int n, double* y) {
  if (!x || !blob || !y || H <= 0 || I <= 0 || n < 0) return -1;
  const uint8_t* q = static_cast<const uint8_t*>(blob);
  const uint8_t* Qgate = q;
  const uint8_t* Qup = q + (size_t)I * H;
  const uint8_t* Qdown = q + 2 * (size_t)I * H;
  std::vector<float> sc(2 * (size_t)I + H);
  std::memcpy(sc.data(), q + 3 * (size_t)I * H, sc.size() * sizeof(float));
  const float* s_gate = sc.data();
  const float* s_up = sc.data() + I;
  const float* s_down = sc.data() + 2 * (size_t)I;
  double value_of[256];                      // the 256 codes, decoded once
  for (int b = 0; b < 256; ++b) value_of[b] = e4m3_value((uint8_t)b);
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < n; ++r) {
    const size_t t = tok ? (size_t)tok[r] : (size_t)r;
    std::vector<double> a(I);
    for (int i = 0; i < I; ++i) {
      double g = 0.0, u = 0.0;
      for (int h = 0; h < H; ++h) {
        const double xv = load_elem(x, t * H + h, xdtype);
        g += (double)s_gate[i] * value_of[Qgate[(size_t)i * H + h]] * xv;
        u += (double)s_up[i] * value_of[Qup[(size_t)i * H + h]] * xv;
      }
      a[i] = g / (1.0 + std::exp(-g)) * u;
    }
    for (int c = 0; c < H; ++c) {
      double acc = 0.0;
      for (int i = 0; i < I; ++i) acc += (double)s_down[c] * value_of[Qdown[(size_t)c * I + i]] * a[i];
      y[(size_t)r * H + c] = acc;
    }
  }
  return 0;
}

// The same feed-forward with the expert's weights in MXFP4 (OCP microscaling: 4-bit E2M1 elements
// that share one E8M0 scale per block of 32 along the contraction; weight-only, activations in
// `xdtype`):
//   blob = [Q_gate I x H/2 | Q_up I x H/2 | Q_down H x I/2] bytes of two codes (even k low),
//          followed by the scales [S_gate I x H/32 | S_up I x H/32 | S_down H x I/32], one byte each;
//   W[r][k] = e8m0(S[r][k / 32]) * e2m1(Q[r][k]).  H and I are multiples of 32.
int oracle_swiglu_rows_mx4(const void* x, int xdtype, int H, int I, const void* blob,
                           const int32_t* tok, int n, double* y) {
  if (!x || !blob || !y || H <= 0 || I <= 0 || n < 0 || H % 32 || I % 32) return -1;
  const uint8_t* q = static_cast<const uint8_t*>(blob);
  const size_t HI = (size_t)H * I;
  const uint8_t* Qgate = q;
  const uint8_t* Qup = q + HI / 2;
  const uint8_t* Qdown = q + HI;
  const uint8_t* Sgate = q + 3 * HI / 2;
  const uint8_t* Sup = Sgate + HI / 32;
  const uint8_t* Sdown = Sup + HI / 32;
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < n; ++r) {
    const size_t t = tok ? (size_t)tok[r] : (size_t)r;
    std::vector<double> a(I);
    for (int i = 0; i < I; ++i) {
      double g = 0.0, u = 0.0;
      for (int h = 0; h < H; ++h) {
        const double xv = load_elem(x, t * H + h, xdtype);
        g += mx4_elem(Qgate, Sgate, i, h, H) * xv;
        u += mx4_elem(Qup, Sup, i, h, H) * xv;
      }
      a[i] = g / (1.0 + std::exp(-g)) * u;
    }
    for (int c = 0; c < H; ++c) {
      double acc = 0.0;
      for (int i = 0; i < I; ++i) acc += mx4_elem(Qdown, Sdown, c, i, I) * a[i];
      y[(size_t)r * H + c] = acc;
    }
  }
  return 0;
}

// Values of n E2M1 codes (one per byte, low four bits) and of n E8M0 scales.
int oracle_e2m1_decode(const uint8_t* codes, int n, double* out) {
  if (!codes || !out || n < 0) return -1;
  for (int i = 0; i < n; ++i) out[i] = e2m1_value(codes[i] & 15u);
  return 0;
}
int oracle_e8m0_decode(const uint8_t* scales, int n, double* out) {
  if (!scales || !out || n < 0) return -1;
  for (int i = 0; i < n; ++i) out[i] = e8m0_value(scales[i]);
  return 0;
}

int oracle_e4m3_decode(const uint8_t* codes, int n, double* out) {
  if (!codes || !out || n < 0) return -1;
  for (int i = 0; i < n; ++i) out[i] = e4m3_value(codes[i]);
  return 0;
}

// Execution stage over the dispatched pairs: expert e processes positions
// offsets[e] .. offsets[e+1]-1.  expert_w[e] points at expert e's blob (host memory).
// w8 == 1: the blobs hold 8-bit weights with row scales (oracle_swiglu_rows_w8); w8 == 2: MXFP4
// weights (oracle_swiglu_rows_mx4).
int oracle_expert_ffn(const void* x, int dtype, int H, int I, int E, const int32_t* offsets,
                      const int32_t* sorted_token, const void* const* expert_w, int w8, double* y) {
  if (!offsets || !sorted_token || !expert_w) return -1;
  for (int e = 0; e < E; ++e) {
    const int b = offsets[e], n = offsets[e + 1] - b;
    if (n == 0) continue;
    int rc = w8 == 2 ? oracle_swiglu_rows_mx4(x, dtype, H, I, expert_w[e], sorted_token + b, n, y + (size_t)b * H)
             : w8 ? oracle_swiglu_rows_w8(x, dtype, H, I, expert_w[e], sorted_token + b, n, y + (size_t)b * H)
                  : oracle_swiglu_rows(x, dtype, H, I, expert_w[e], sorted_token + b, n,
                                       y + (size_t)b * H);
    if (rc) return rc;
  }
  return 0;
}

// "finally summed": out[t][c] = sum_{j<k_t} w[t][j] * y[inv_pos[t][j]][c]  (j ascending)
//                              + sum_s shared[s][t][c]
// shared: n_shared stacked [T,H] double arrays (always-on experts, weight 1) or NULL.
int oracle_combine(const double* y, const float* w, const int32_t* inv_pos, const int32_t* k_t,
                   const double* shared, int n_shared, int T, int H, int K, double* out) {
  if (!w || !inv_pos || !k_t || !out) return -1;
  for (int t = 0; t < T; ++t) {
    for (int c = 0; c < H; ++c) {
      double acc = 0.0;
      for (int j = 0; j < k_t[t]; ++j)
        acc += (double)w[(size_t)t * K + j] * y[(size_t)inv_pos[(size_t)t * K + j] * H + c];
      for (int s = 0; s < n_shared; ++s) acc += shared[((size_t)s * T + t) * H + c];
      out[(size_t)t * H + c] = acc;
    }
  }
  return 0;
}

// out[t] += sum_{j_lo <= j < k_t[t]} w[t][j] * y[inv_pos[t][j]]: the ranks that the big model adds on
// top of a little result (routing weights not renormalised, so the ranks below j_lo keep their
// weights).  Tokens with k_t[t] <= j_lo are left as they are.
int oracle_combine_add(const double* y, const float* w, const int32_t* inv_pos, const int32_t* k_t,
                       int j_lo, int T, int H, int K, double* out) {
  if (!w || !inv_pos || !k_t || !out || j_lo < 0) return -1;
  for (int t = 0; t < T; ++t) {
    for (int c = 0; c < H; ++c) {
      double acc = out[(size_t)t * H + c];
      for (int j = j_lo; j < k_t[t]; ++j)
        acc += (double)w[(size_t)t * K + j] * y[(size_t)inv_pos[(size_t)t * K + j] * H + c];
      out[(size_t)t * H + c] = acc;
    }
  }
  return 0;
}

// Threads the OpenMP loops over independent rows use from now on (timing of the oracle on one
// core and on all of them; the arithmetic does not depend on it).  n <= 0: leave as is.
int oracle_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
  return 0;
}

int oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp single
    n = omp_get_num_threads();
  }
#endif
  return n;
}

}  // extern "C"
