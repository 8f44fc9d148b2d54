// Internal declarations shared by the translation units of libmobile_moe.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mobile_moe.h"

namespace mm {

// ---- error reporting (thread-local message behind moe_last_error) -------------------------
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int hip_fail(hipError_t e, const char* what);
#define MM_HIP(expr)                                   \
  do {                                                 \
    hipError_t _e = (expr);                            \
    if (_e != hipSuccess) return ::mm::hip_fail(_e, #expr); \
  } while (0)

int validate_config(const moe_config* cfg);

// ---- optional per-kernel timing (moe_profile_*): an event pair around each launch site -------
enum ProfKind { kProfRouterGemm = 0, kProfRouteTopk, kProfDispatch, kProfFfnGateUp, kProfFfnDown,
                kProfCombine, kProfConfidence, kProfDecodeStep, kProfKinds };
void prof_mark(int kind, bool begin, hipStream_t s);
struct ProfScope {
  int kind; hipStream_t s;
  ProfScope(int k, hipStream_t st) : kind(k), s(st) { prof_mark(kind, true, s); }
  ~ProfScope() { prof_mark(kind, false, s); }
};
int device_cu_count();

inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }
// bytes of an activation / router-matrix element, and of an expert weight
inline size_t elem_bytes(int dtype) { return dtype == MOE_FP32 ? 4 : 2; }
// one expert: [W_gate I x H | W_up I x H | W_down H x I] (+ the fp32 row scales of 8-bit weights,
// or the block scales of MXFP4 weights: one byte per 32 weights)
inline size_t expert_blob_bytes(int dtype, int H, int I) {
  const size_t n = (size_t)3 * H * I;
  switch (dtype) {
    case MOE_FP32: return n * 4;
    case MOE_BF16_W8: return n + (size_t)4 * (2 * (size_t)I + H);
    case MOE_BF16_MXFP4: return n / 2 + n / 32;
    default: return n * 2;
  }
}

// ---- skinny grouped GEMM  D[r][n] = sum_k W[n][k] * B[r][k]  (weights streamed once) --------
// Three uses: router logits, gate/up projection with fused SwiGLU, down projection.
enum StreamMode { kRouter = 0, kGateUp = 1, kDown = 2 };

// The down projection of a wide shared expert is cut along its contraction into chunks that
// are computed as independent groups and written to separate [T,H] slabs of shared_out.
constexpr int kMaxKSplit = 4;
constexpr int kMaxSlabs = MOE_MAX_SHARED * kMaxKSplit;
struct SlabPlan {
  int n_slabs;
  int kchunk[MOE_MAX_SHARED];          // chunk length per shared expert (multiple of 32)
  int slab_shared[kMaxSlabs];          // slab -> shared expert
  int slab_chunk[kMaxSlabs];           // slab -> chunk index within that expert
};
SlabPlan slab_plan(const moe_config& c);

struct StreamArgs {
  int T, H, E, I;
  int n_routed;                       // E when the routed experts are run, else 0
  int n_shared;                       // shared experts run by this launch
  int shared_I[MOE_MAX_SHARED];
  int shared_kchunk[MOE_MAX_SHARED];
  int n_slabs;                        // groups of the shared down projection
  int slab_shared[kMaxSlabs];
  int slab_chunk[kMaxSlabs];
  const void* shared_w[MOE_MAX_SHARED];
  const void* const* expert_w;        // device table [E]
  const int32_t* offsets;             // device [E+1]
  const int32_t* sorted_token;        // device [T*k_big]
  int max_pairs;                      // T * k_big
  const void* x;                      // [T,H]
  void* h_routed;                     // [T*k_big, I]   SwiGLU activations (storage dtype)
  void* h_shared[MOE_MAX_SHARED];     // [T, I_s]
  float* y;                           // [T*k_big, H]
  float* shared_out;                  // [n_slabs, T, H]
  const void* Wg;                     // router: [E,H]
  const float* bias;                  // router: [E] or null
  float* logits;                      // router: [T,E]
};

int launch_stream(StreamMode mode, int dtype, const StreamArgs& a, hipStream_t s);
// kGateUp / kDown on bf16 activations with the weights (2 bytes: bf16, 1 byte: E4M3 + row
// scales) streamed through an LDS ring (stream_lds.hip)
// weight_format: 2 = bf16, 1 = 8-bit codes with row scales, 0 = MXFP4
int launch_stream_lds(StreamMode mode, int weight_format, const StreamArgs& a, hipStream_t s);

// ---- large-m grouped GEMM on LDS-tiled MFMA (prefill regime; bf16 activations) ---------------
// weight_format: 2 = bf16, 1 = 8-bit codes with row scales, 0 = MXFP4
int launch_tiled(StreamMode mode, int weight_format, const StreamArgs& a, hipStream_t s);

// ---- a whole decode step in one launch (decode_step.hip) -------------------------------------
constexpr int kDecodeMaxTokens = 64;
struct DecodeLaunch {
  const void* x; const void* Wg; const float* gate_bias; const float* conf;
  const void* const* expert_w;            // device table [E]
  const void* shared_w[MOE_MAX_SHARED];
  int logits_given;
  float* logits; int32_t* topk_idx; float* topk_w; uint8_t* important; int32_t* k_t;
  int32_t* expert_offsets; int32_t* sorted_token; int32_t* sorted_rank; int32_t* inv_pos;
  void* h_routed; void* h_shared[MOE_MAX_SHARED];
  float* y; float* shared_out; void* out;
  void* sync;                             // decode_sync_bytes() of counters, zero between steps
  int spin_limit;                         // polls after which a wait inside the kernel gives up
};
size_t decode_sync_bytes();
int decode_sync_error_word();             // index (in ints) of the error word inside the counters
int launch_decode_sync_clear(void* sync, hipStream_t s);
int launch_decode_step(const moe_config& c, const DecodeLaunch& L, hipStream_t s);

// ---- selection, dispatch, combine -----------------------------------------------------------
int launch_route(const moe_config& c, const float* conf, const float* logits, int32_t* idx,
                 float* w, uint8_t* important, int32_t* k_t, hipStream_t s);
int launch_gate_gemv(const moe_config& c, const void* x, const void* Wg, const float* bias, float* logits,
                     hipStream_t s);
int launch_gate_route(const moe_config& c, const void* x, const void* Wg, const float* bias, const float* conf,
                      float* logits, int32_t* idx, float* w, uint8_t* important, int32_t* k_t, hipStream_t s);
int launch_confidence(const float* z, int T, int V, float* conf, hipStream_t s);
int dispatch_chunks(int T);          // workgroups (token chunks) of the large-T dispatch
// pairs (t, j) with j_lo <= j < k_t[t]
int launch_dispatch(const moe_config& c, const int32_t* idx, const int32_t* k_t, int j_lo, int32_t* offsets,
                    int32_t* sorted_token, int32_t* sorted_rank, int32_t* inv_pos, int32_t* counts,
                    hipStream_t s);
int launch_combine(const moe_config& c, const float* y, const float* w, const int32_t* inv_pos,
                   const int32_t* k_t, const float* shared_out, void* out, hipStream_t s);
// out[t] += sum over the ranks j_lo <= j < k_t[t]; tokens without such ranks are not written
int launch_combine_add(const moe_config& c, const float* y, const float* w, const int32_t* inv_pos,
                       const int32_t* k_t, int j_lo, void* out, hipStream_t s);

}  // namespace mm
