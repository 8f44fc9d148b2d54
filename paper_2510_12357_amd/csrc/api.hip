// C-ABI entry points: host-side validation and kernel sequencing.  Every shape is checked here
// against what the kernels and their grids assume before anything is enqueued.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "internal.h"

// Scratch of moe_expert_ffn_static: the SwiGLU activations of one step, for callers that cannot
// allocate.  One copy per GPU the library runs on, held until the process ends.  In host code the
// name below is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
#define MOE_STATIC_SCRATCH_BYTES (8u << 20)
static __device__ __align__(256) unsigned char scratch[MOE_STATIC_SCRATCH_BYTES];

namespace mm {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

int hip_fail(hipError_t e, const char* what) {
  if (e == hipSuccess) return MOE_OK;
  return fail(MOE_E_HIP, "%s: %s", what, hipGetErrorString(e));
}

// ---- per-kernel timing ------------------------------------------------------------------------
namespace {
struct ProfState {
  bool on = false;
  std::vector<hipEvent_t> ev;      // 2 per record: begin, end
  std::vector<int> kind;           // per record
  size_t used = 0;                 // records in use
  static constexpr size_t kMaxRecords = 1 << 15;
} g_prof;
}  // namespace

void prof_mark(int kind, bool begin, hipStream_t s) {
  if (!g_prof.on) return;
  if (begin) {
    if (g_prof.used >= ProfState::kMaxRecords) return;
    if (g_prof.used * 2 >= g_prof.ev.size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { g_prof.on = false; return; }
      g_prof.ev.push_back(a); g_prof.ev.push_back(b);
      g_prof.kind.push_back(kind);
    }
    g_prof.kind[g_prof.used] = kind;
    (void)hipEventRecord(g_prof.ev[2 * g_prof.used], s);
  } else {
    if (g_prof.used >= ProfState::kMaxRecords || g_prof.used * 2 >= g_prof.ev.size()) return;
    (void)hipEventRecord(g_prof.ev[2 * g_prof.used + 1], s);
    g_prof.used++;
  }
}

int device_cu_count() {
  static thread_local int cached_dev = -1, cached_cu = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (dev != cached_dev) {
    int cu = 0;
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0) cu = 256;
    cached_dev = dev; cached_cu = cu;
  }
  return cached_cu;
}

// Steps of this many tokens and more run the LDS-tiled kernels (bf16 activations).
constexpr int kTiledMinT = 256;

int validate_config(const moe_config* c) {
  if (!c) return fail(MOE_E_BADARG, "config is NULL");
  if (c->dtype != MOE_BF16 && c->dtype != MOE_FP32 && c->dtype != MOE_BF16_W8 && c->dtype != MOE_BF16_MXFP4)
    return fail(MOE_E_BADARG, "dtype %d", c->dtype);
  if (c->T < 0 || c->H <= 0 || c->E <= 0 || c->I <= 0) return fail(MOE_E_SHAPE, "T=%d H=%d E=%d I=%d", c->T, c->H, c->E, c->I);
  if (c->k_little < 1 || c->k_little > c->k_big || c->k_big > c->E)
    return fail(MOE_E_SHAPE, "need 1 <= k_little (%d) <= k_big (%d) <= E (%d)", c->k_little, c->k_big, c->E);
  if (c->E > MOE_MAX_EXPERTS) return fail(MOE_E_UNSUPPORTED, "E=%d above %d", c->E, MOE_MAX_EXPERTS);
  if (c->k_big > MOE_MAX_TOPK) return fail(MOE_E_UNSUPPORTED, "k_big=%d above %d", c->k_big, MOE_MAX_TOPK);
  if (c->n_shared < 0 || c->n_shared > MOE_MAX_SHARED) return fail(MOE_E_UNSUPPORTED, "n_shared=%d outside [0,%d]", c->n_shared, MOE_MAX_SHARED);
  if (c->H % 8 || c->I % 8) return fail(MOE_E_UNSUPPORTED, "H=%d and I=%d must be multiples of 8", c->H, c->I);
  int maxdim = c->H > c->I ? c->H : c->I;
  for (int s = 0; s < c->n_shared; ++s) {
    if (c->shared_I[s] <= 0 || c->shared_I[s] % 8) return fail(MOE_E_UNSUPPORTED, "shared_I[%d]=%d must be a positive multiple of 8", s, c->shared_I[s]);
    if (c->shared_I[s] > maxdim) maxdim = c->shared_I[s];
  }
  if ((long long)c->T * c->k_big * (long long)maxdim >= (1ll << 31))
    return fail(MOE_E_UNSUPPORTED, "T*k_big*max(H,I) = %lld does not fit 31 bits", (long long)c->T * c->k_big * maxdim);
  // every tensor the kernels address through a 32-bit buffer offset must stay below 2 GiB
  const long long eb = (long long)elem_bytes(c->dtype);
  const long long biggest = eb * maxdim * (long long)(3 * c->H > c->T * c->k_big ? 3 * c->H : c->T * c->k_big);
  const long long act = eb * (long long)c->T * (c->H > maxdim ? c->H : maxdim);
  const long long gate = eb * (long long)c->E * c->H;
  if (biggest >= (1ll << 31) || act >= (1ll << 31) || gate >= (1ll << 31))
    return fail(MOE_E_UNSUPPORTED, "a tensor of this layer reaches 2 GiB (expert blob, activations or gate matrix)");
  if (c->dtype == MOE_BF16_W8) {
    // the kernels move 16 codes of a weight row at a time
    bool ok = c->H % 16 == 0 && c->I % 16 == 0;
    for (int s = 0; s < c->n_shared; ++s) ok = ok && c->shared_I[s] % 16 == 0;
    if (!ok) return fail(MOE_E_UNSUPPORTED, "8-bit expert weights need H, I and every shared_I to be multiples of 16");
  }
  if (c->dtype == MOE_BF16_MXFP4) {
    // a scale block is 32 weights along the contraction; the kernel fetches the scale bytes of a
    // row 16 at a time with 4-byte aligned loads, so a row must hold a multiple of 4 of them
    bool ok = c->H % 128 == 0 && c->I % 128 == 0;
    for (int s = 0; s < c->n_shared; ++s) ok = ok && c->shared_I[s] % 128 == 0;
    if (!ok) return fail(MOE_E_UNSUPPORTED, "MXFP4 expert weights need H, I and every shared_I to be multiples of 128");
  }
  if (!(c->gamma == c->gamma)) return fail(MOE_E_BADARG, "gamma is NaN");
  return MOE_OK;
}

SlabPlan slab_plan(const moe_config& c) {
  SlabPlan P = {};
  const int target = c.I > 1024 ? c.I : 1024;          // chunk about as long as a routed expert's I
  for (int s = 0; s < c.n_shared; ++s) {
    const int Is = c.shared_I[s];
    int n = (Is + target - 1) / target;
    if (n > kMaxKSplit) n = kMaxKSplit;
    // MXFP4: a chunk starts on a multiple of 128 weights, so that the scale bytes of a row (one
    // per 32 weights) stay 4-byte aligned behind it
    const int round = c.dtype == MOE_BF16_MXFP4 ? 128 : 32;
    int chunk = ((Is + n - 1) / n + round - 1) / round * round;
    n = (Is + chunk - 1) / chunk;
    P.kchunk[s] = chunk;
    for (int k = 0; k < n; ++k) {
      P.slab_shared[P.n_slabs] = s;
      P.slab_chunk[P.n_slabs] = k;
      P.n_slabs++;
    }
  }
  return P;
}

namespace {
struct FfnLayout {
  size_t h_routed, h_shared[MOE_MAX_SHARED], total;
};
FfnLayout ffn_layout(const moe_config& c) {
  FfnLayout L;
  size_t off = 0;
  const size_t eb = elem_bytes(c.dtype);
  L.h_routed = off;
  off += align256((size_t)c.T * c.k_big * c.I * eb);
  for (int s = 0; s < MOE_MAX_SHARED; ++s) {
    L.h_shared[s] = off;
    if (s < c.n_shared) off += align256((size_t)c.T * c.shared_I[s] * eb);
  }
  L.total = off < 256 ? 256 : off;
  return L;
}
}  // namespace

}  // namespace mm

using namespace mm;

extern "C" const char* moe_last_error(void) { return g_err; }

extern "C" int moe_profile_enable(int on) {
  g_prof.on = on != 0;
  g_prof.used = 0;
  return MOE_OK;
}

extern "C" int moe_profile_read(int kind, int64_t* launches, double* total_ms) {
  if (kind < 0 || kind >= kProfKinds || !launches || !total_ms) return fail(MOE_E_BADARG, "moe_profile_read: kind %d", kind);
  int64_t n = 0;
  double ms = 0.0;
  for (size_t i = 0; i < g_prof.used; ++i) {
    if (g_prof.kind[i] != kind) continue;
    MM_HIP(hipEventSynchronize(g_prof.ev[2 * i + 1]));
    float t = 0.f;
    MM_HIP(hipEventElapsedTime(&t, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]));
    ms += t; ++n;
  }
  *launches = n; *total_ms = ms;
  return MOE_OK;
}

extern "C" int moe_device_info(int32_t* n_cu, int32_t* is_gfx950) {
  int dev = 0;
  MM_HIP(hipGetDevice(&dev));
  hipDeviceProp_t p;
  MM_HIP(hipGetDeviceProperties(&p, dev));
  if (n_cu) *n_cu = p.multiProcessorCount;
  if (is_gfx950) *is_gfx950 = (strncmp(p.gcnArchName, "gfx950", 6) == 0) ? 1 : 0;
  return MOE_OK;
}

extern "C" int moe_route(const moe_config* cfg, const void* x, const void* Wg, const float* gate_bias,
                         const float* conf, float* logits, int logits_given, int32_t* topk_idx,
                         float* topk_w, uint8_t* important, int32_t* k_t, void* stream) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  if (cfg->T == 0) return MOE_OK;
  if (!logits || !topk_idx || !topk_w || !important || !k_t)
    return fail(MOE_E_BADARG, "moe_route: logits/topk_idx/topk_w/important/k_t must not be NULL");
  if (!logits_given && (!x || !Wg)) return fail(MOE_E_BADARG, "moe_route: x and Wg are needed unless logits_given");
  hipStream_t s = static_cast<hipStream_t>(stream);
  // decode sizes: plain-FMA GEMV spread over many waves; larger T: MFMA router GEMM
  constexpr int kGemvMaxT = 256;
  // decode batches: logits and selection of a token in one workgroup, one launch
  constexpr int kOneLaunchMaxT = 64;
  if (!logits_given && cfg->T <= kOneLaunchMaxT) {
    ProfScope ps(kProfRouteTopk, s);
    return launch_gate_route(*cfg, x, Wg, gate_bias, conf, logits, topk_idx, topk_w, important, k_t, s);
  }
  if (!logits_given) {
    ProfScope ps(kProfRouterGemm, s);
    if (cfg->T <= kGemvMaxT) {
      rc = launch_gate_gemv(*cfg, x, Wg, gate_bias, logits, s);
    } else {
      StreamArgs a = {};
      a.T = cfg->T; a.H = cfg->H; a.E = cfg->E; a.I = cfg->I;
      a.x = x; a.Wg = Wg; a.bias = gate_bias; a.logits = logits;
      rc = launch_stream(kRouter, cfg->dtype, a, s);
    }
    if (rc) return rc;
  }
  ProfScope ps(kProfRouteTopk, s);
  return launch_route(*cfg, conf, logits, topk_idx, topk_w, important, k_t, s);
}

extern "C" int moe_token_confidence(const float* lm_logits, int32_t T, int32_t V, float* conf, void* stream) {
  if (T < 0 || V <= 0) return fail(MOE_E_SHAPE, "moe_token_confidence: T=%d V=%d", T, V);
  if (T > 0 && (!lm_logits || !conf)) return fail(MOE_E_BADARG, "moe_token_confidence: null pointer");
  ProfScope ps(kProfConfidence, static_cast<hipStream_t>(stream));
  return launch_confidence(lm_logits, T, V, conf, static_cast<hipStream_t>(stream));
}

extern "C" size_t moe_dispatch_workspace_bytes(const moe_config* cfg) {
  if (validate_config(cfg)) return 0;
  return align256(sizeof(int32_t) * (size_t)cfg->E * (size_t)(dispatch_chunks(cfg->T) + 1));
}

extern "C" int moe_dispatch(const moe_config* cfg, const int32_t* topk_idx, const int32_t* k_t,
                            int32_t* expert_offsets, int32_t* sorted_token, int32_t* sorted_rank,
                            int32_t* inv_pos, void* ws, size_t ws_bytes, void* stream) {
  return moe_dispatch_from(cfg, topk_idx, k_t, 0, expert_offsets, sorted_token, sorted_rank, inv_pos, ws, ws_bytes,
                           stream);
}

extern "C" int moe_dispatch_from(const moe_config* cfg, const int32_t* topk_idx, const int32_t* k_t,
                                 int32_t j_lo, int32_t* expert_offsets, int32_t* sorted_token,
                                 int32_t* sorted_rank, int32_t* inv_pos, void* ws, size_t ws_bytes,
                                 void* stream) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  if (j_lo < 0 || j_lo > cfg->k_big) return fail(MOE_E_BADARG, "moe_dispatch_from: j_lo=%d outside [0, k_big=%d]", j_lo, cfg->k_big);
  if (!expert_offsets) return fail(MOE_E_BADARG, "moe_dispatch: expert_offsets is NULL");
  if (cfg->T > 0 && (!topk_idx || !k_t || !sorted_token || !sorted_rank || !inv_pos))
    return fail(MOE_E_BADARG, "moe_dispatch: null tensor");
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < moe_dispatch_workspace_bytes(cfg))
    return fail(MOE_E_WORKSPACE, "moe_dispatch: workspace %p of %zu bytes (need %zu, 256-byte aligned)", ws,
                ws_bytes, moe_dispatch_workspace_bytes(cfg));
  ProfScope ps(kProfDispatch, static_cast<hipStream_t>(stream));
  return launch_dispatch(*cfg, topk_idx, k_t, j_lo, expert_offsets, sorted_token, sorted_rank, inv_pos,
                         static_cast<int32_t*>(ws), static_cast<hipStream_t>(stream));
}

extern "C" int32_t moe_shared_out_slabs(const moe_config* cfg) {
  if (validate_config(cfg)) return -1;
  return slab_plan(*cfg).n_slabs;
}

extern "C" size_t moe_expert_blob_bytes(const moe_config* cfg, int32_t I) {
  if (validate_config(cfg) || I <= 0 || I % 8) return 0;
  return expert_blob_bytes(cfg->dtype, cfg->H, I);
}

extern "C" size_t moe_expert_ffn_workspace_bytes(const moe_config* cfg) {
  if (validate_config(cfg)) return 0;
  return ffn_layout(*cfg).total;
}

extern "C" int moe_expert_ffn(const moe_config* cfg, const void* x, const int32_t* expert_offsets,
                              const int32_t* sorted_token, const void* const* expert_w,
                              const void* const* shared_w, int run_routed, int run_shared, float* y,
                              float* shared_out, void* ws, size_t ws_bytes, void* stream) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  const bool routed = run_routed != 0;
  const bool shared = run_shared != 0 && cfg->n_shared > 0;
  if (cfg->T == 0 || (!routed && !shared)) return MOE_OK;
  if (!x) return fail(MOE_E_BADARG, "moe_expert_ffn: x is NULL");
  if (routed && (!expert_offsets || !sorted_token || !expert_w || !y))
    return fail(MOE_E_BADARG, "moe_expert_ffn: routed part needs expert_offsets, sorted_token, expert_w, y");
  if (shared && (!shared_w || !shared_out))
    return fail(MOE_E_BADARG, "moe_expert_ffn: shared part needs shared_w and shared_out");
  if (shared)
    for (int s = 0; s < cfg->n_shared; ++s)
    {
      if (!shared_w[s]) return fail(MOE_E_BADARG, "moe_expert_ffn: shared_w[%d] is NULL", s);
      // expert blobs are read in 16-byte pieces (the routed experts' pointers live on the device
      // and cannot be checked here)
      if ((uintptr_t)shared_w[s] & 15) return fail(MOE_E_BADARG, "moe_expert_ffn: shared_w[%d] is not 16-byte aligned", s);
    }
  const FfnLayout L = ffn_layout(*cfg);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < L.total)
    return fail(MOE_E_WORKSPACE, "moe_expert_ffn: workspace %p of %zu bytes (need %zu, 256-byte aligned)", ws,
                ws_bytes, L.total);

  StreamArgs a = {};
  a.T = cfg->T; a.H = cfg->H; a.E = cfg->E; a.I = cfg->I;
  a.n_routed = routed ? cfg->E : 0;
  a.n_shared = shared ? cfg->n_shared : 0;
  a.expert_w = expert_w; a.offsets = expert_offsets; a.sorted_token = sorted_token;
  a.max_pairs = cfg->T * cfg->k_big;
  a.x = x; a.y = y; a.shared_out = shared_out;
  char* wsb = static_cast<char*>(ws);
  a.h_routed = wsb + L.h_routed;
  const SlabPlan plan = slab_plan(*cfg);
  for (int s = 0; s < a.n_shared; ++s) {
    a.shared_I[s] = cfg->shared_I[s];
    a.shared_kchunk[s] = plan.kchunk[s];
    a.shared_w[s] = shared_w[s];
    a.h_shared[s] = wsb + L.h_shared[s];
  }
  a.n_slabs = shared ? plan.n_slabs : 0;
  for (int i = 0; i < a.n_slabs; ++i) { a.slab_shared[i] = plan.slab_shared[i]; a.slab_chunk[i] = plan.slab_chunk[i]; }
  hipStream_t s = static_cast<hipStream_t>(stream);
  // Regime: with many tokens per step the experts see enough rows for LDS-tiled MFMA GEMMs;
  // below that the weights are streamed once through the skinny kernel.
  const bool tiled = cfg->dtype != MOE_FP32 && cfg->T >= kTiledMinT;
  const int wfmt = cfg->dtype == MOE_BF16_W8 ? 1 : (cfg->dtype == MOE_BF16_MXFP4 ? 0 : 2);
  {
    ProfScope ps(kProfFfnGateUp, s);
    rc = tiled ? launch_tiled(kGateUp, wfmt, a, s) : launch_stream(kGateUp, cfg->dtype, a, s);
    if (rc) return rc;
  }
  ProfScope ps(kProfFfnDown, s);
  return tiled ? launch_tiled(kDown, wfmt, a, s) : launch_stream(kDown, cfg->dtype, a, s);
}

extern "C" int moe_combine(const moe_config* cfg, const float* y, const float* topk_w,
                           const int32_t* inv_pos, const int32_t* k_t, const float* shared_out, void* out,
                           void* stream) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  if (cfg->T == 0) return MOE_OK;
  if (!y || !topk_w || !inv_pos || !k_t || !out) return fail(MOE_E_BADARG, "moe_combine: null tensor");
  if (cfg->n_shared > 0 && !shared_out) return fail(MOE_E_BADARG, "moe_combine: shared_out is NULL but n_shared=%d", cfg->n_shared);
  ProfScope ps(kProfCombine, static_cast<hipStream_t>(stream));
  return launch_combine(*cfg, y, topk_w, inv_pos, k_t, shared_out, out, static_cast<hipStream_t>(stream));
}

extern "C" int moe_combine_add(const moe_config* cfg, const float* y, const float* topk_w,
                               const int32_t* inv_pos, const int32_t* k_t, int32_t j_lo, void* out,
                               void* stream) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  if (cfg->renorm)
    return fail(MOE_E_UNSUPPORTED, "moe_combine_add: with renormalised routing weights the ranks below j_lo "
                                   "change their weights too; recompute the token with moe_combine");
  if (j_lo < 0 || j_lo > cfg->k_big) return fail(MOE_E_BADARG, "moe_combine_add: j_lo=%d outside [0, k_big=%d]", j_lo, cfg->k_big);
  if (cfg->T == 0) return MOE_OK;
  if (!y || !topk_w || !inv_pos || !k_t || !out) return fail(MOE_E_BADARG, "moe_combine_add: null tensor");
  ProfScope ps(kProfCombine, static_cast<hipStream_t>(stream));
  return launch_combine_add(*cfg, y, topk_w, inv_pos, k_t, j_lo, out, static_cast<hipStream_t>(stream));
}

// ---- one decode step in one launch --------------------------------------------------------------
namespace {
int validate_decode(const moe_config* cfg) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  if (cfg->dtype == MOE_FP32) return fail(MOE_E_UNSUPPORTED, "moe_layer_decode: bf16 activations only (use the separate calls for fp32)");
  if (cfg->dtype == MOE_BF16_MXFP4) return fail(MOE_E_UNSUPPORTED, "moe_layer_decode: bf16 or 8-bit expert weights only (use the separate calls for MXFP4)");
  if (cfg->T > kDecodeMaxTokens) return fail(MOE_E_UNSUPPORTED, "moe_layer_decode: T=%d above %d tokens (use the separate calls)", cfg->T, kDecodeMaxTokens);
  if ((long long)cfg->T * cfg->k_big * cfg->H * 4 >= (1ll << 31)) return fail(MOE_E_UNSUPPORTED, "moe_layer_decode: y reaches 2 GiB");
  return MOE_OK;
}
}  // namespace

extern "C" size_t moe_layer_decode_workspace_bytes(const moe_config* cfg) {
  if (validate_decode(cfg)) return 0;
  return decode_sync_bytes() + ffn_layout(*cfg).total;
}

extern "C" int moe_layer_decode_init(void* ws, size_t ws_bytes, void* stream) {
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < decode_sync_bytes())
    return fail(MOE_E_WORKSPACE, "moe_layer_decode_init: workspace %p of %zu bytes", ws, ws_bytes);
  return launch_decode_sync_clear(ws, static_cast<hipStream_t>(stream));
}

extern "C" int moe_layer_decode_status(const void* ws, int32_t* timed_out_waits) {
  if (!ws || !timed_out_waits) return fail(MOE_E_BADARG, "moe_layer_decode_status: null argument");
  int32_t v = 0;
  MM_HIP(hipMemcpy(&v, static_cast<const int32_t*>(ws) + decode_sync_error_word(), sizeof v, hipMemcpyDeviceToHost));
  *timed_out_waits = v;
  return MOE_OK;
}

extern "C" int moe_layer_decode(const moe_config* cfg, const void* x, const void* Wg, const float* gate_bias,
                                const float* conf, const void* const* expert_w, const void* const* shared_w,
                                float* logits, int logits_given, int32_t* topk_idx, float* topk_w,
                                uint8_t* important, int32_t* k_t, int32_t* expert_offsets, int32_t* sorted_token,
                                int32_t* sorted_rank, int32_t* inv_pos, float* y, float* shared_out, void* out,
                                void* ws, size_t ws_bytes, void* stream) {
  int rc = validate_decode(cfg);
  if (rc) return rc;
  if (cfg->T == 0) return MOE_OK;
  if (!x || !expert_w || !logits || !topk_idx || !topk_w || !important || !k_t || !expert_offsets || !sorted_token ||
      !sorted_rank || !inv_pos || !y || !out)
    return fail(MOE_E_BADARG, "moe_layer_decode: null tensor");
  if (!logits_given && !Wg) return fail(MOE_E_BADARG, "moe_layer_decode: Wg is needed unless logits_given");
  if (cfg->n_shared > 0 && (!shared_w || !shared_out)) return fail(MOE_E_BADARG, "moe_layer_decode: shared_w / shared_out missing");
  for (int s = 0; s < cfg->n_shared; ++s)
    if (!shared_w[s] || ((uintptr_t)shared_w[s] & 15)) return fail(MOE_E_BADARG, "moe_layer_decode: shared_w[%d] null or not 16-byte aligned", s);
  const FfnLayout L = ffn_layout(*cfg);
  const size_t sync_bytes = decode_sync_bytes();
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < sync_bytes + L.total)
    return fail(MOE_E_WORKSPACE, "moe_layer_decode: workspace %p of %zu bytes (need %zu, 256-byte aligned)", ws, ws_bytes,
                sync_bytes + L.total);
  DecodeLaunch D = {};
  D.x = x; D.Wg = Wg; D.gate_bias = gate_bias; D.conf = conf; D.expert_w = expert_w;
  char* wsb = static_cast<char*>(ws) + sync_bytes;
  for (int s = 0; s < cfg->n_shared; ++s) { D.shared_w[s] = shared_w[s]; D.h_shared[s] = wsb + L.h_shared[s]; }
  D.logits_given = logits_given != 0;
  D.logits = logits; D.topk_idx = topk_idx; D.topk_w = topk_w; D.important = important; D.k_t = k_t;
  D.expert_offsets = expert_offsets; D.sorted_token = sorted_token; D.sorted_rank = sorted_rank; D.inv_pos = inv_pos;
  D.h_routed = wsb + L.h_routed; D.y = y; D.shared_out = shared_out; D.out = out;
  D.sync = ws;
  D.spin_limit = 1 << 18;                 // a good tenth of a second of polling: far beyond any wait of a healthy step
  ProfScope ps(kProfDecodeStep, static_cast<hipStream_t>(stream));
  return launch_decode_step(*cfg, D, static_cast<hipStream_t>(stream));
}

// ---- the execution stage without any allocation ------------------------------------------------
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of this GPU's copy of `scratch`, looked up once per device (with it current).
int static_scratch(void** out) {
  int dev = 0;
  MM_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(MOE_E_UNSUPPORTED, "moe_expert_ffn_static: device ordinal %d", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    MM_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p & 255)) return fail(MOE_E_HIP, "moe_expert_ffn_static: scratch symbol at %p", p);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MOE_OK;
}
}  // namespace

extern "C" size_t moe_expert_ffn_static_max_bytes(void) { return MOE_STATIC_SCRATCH_BYTES; }

extern "C" int moe_expert_ffn_static(const moe_config* cfg, const void* x, const int32_t* expert_offsets,
                                     const int32_t* sorted_token, const void* const* expert_w,
                                     const void* const* shared_w, int run_routed, int run_shared, float* y,
                                     float* shared_out, void* stream) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  const size_t need = ffn_layout(*cfg).total;
  if (need > MOE_STATIC_SCRATCH_BYTES)
    return fail(MOE_E_WORKSPACE, "moe_expert_ffn_static: the step needs %zu bytes of scratch, the built-in buffer holds %u; "
                                 "use moe_expert_ffn with a workspace", need, MOE_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc) return rc;
  // Nothing in the buffer has to start at zero: every activation row a down projection reads was
  // written by the gate/up projection of the same call.
  return moe_expert_ffn(cfg, x, expert_offsets, sorted_token, expert_w, shared_w, run_routed, run_shared, y,
                        shared_out, ws, need, stream);
}
