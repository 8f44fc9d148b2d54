/*
 * mobile_moe.h -- C ABI of the big-little Mixture-of-Experts layer hot path for AMD MI355X
 * (gfx950), after "MoBiLE: Efficient Mixture-of-Experts Inference on Consumer GPU with
 * Mixture of Big Little Experts" (arXiv 2510.12357).
 *
 * One decode or prefill step of one MoE layer is the call sequence
 *
 *     moe_route  ->  moe_dispatch  ->  [expert_cache_fetch]  ->  moe_expert_ffn  ->  moe_combine
 *
 * which follows the paper's two stages (Sec. II-A): a selection stage in which the router
 * picks experts and produces routing weights, and an execution stage in which the hidden
 * states pass through every selected expert and are summed.  The big-little rule (Sec. III-A,
 * Alg. 1) makes the number of experts a per-token quantity: a token whose confidence
 * max(p) is above the threshold gamma keeps the "little" selection of k_little = K/2 experts,
 * every other ("important") token falls back to the "big" selection of k_big = K experts.
 * When expert weights live in host DRAM (Sec. II-B, III-B) expert_cache_fetch brings the
 * needed experts into a small HBM slot cache, on demand or ahead of time from the router
 * outputs of an earlier pass.
 *
 * General conventions
 *   - Every function returns 0 (MOE_OK) or a negative MOE_E_* code; moe_last_error() gives a
 *     thread-local message for the last failure.  Arguments are validated on the host before
 *     anything is enqueued; a failed call enqueues nothing.
 *   - "device" pointers are HBM addresses owned by the caller; "host" pointers are ordinary
 *     process memory.  The library never allocates or frees caller tensors.  Scratch memory is
 *     passed in (`ws`, size from the matching *_workspace_bytes query, 256-byte aligned).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued asynchronously on it; no call synchronises with the host except where stated.
 *   - Tensors are row-major and dense.  dtype MOE_BF16: activations / weights are bf16,
 *     products accumulate in fp32.  dtype MOE_FP32: fp32 storage and arithmetic.
 *     dtype MOE_BF16_W8 (not in the paper): as MOE_BF16, but the expert weights are stored in
 *     8 bits with one fp32 scale per weight row, which halves the bytes a decode step streams
 *     from HBM and the memory a layer takes.  It needs H, I and every shared_I to be multiples
 *     of 16.
 *     dtype MOE_BF16_MXFP4 (not in the paper): as MOE_BF16, but
 *     the expert weights are stored in the OCP microscaling format MXFP4 (4-bit elements with one
 *     power-of-two scale per 32 weights along the contraction): 4.25 bits per weight.  It needs
 *     H, I and every shared_I to be multiples of 128; moe_layer_decode does not take it.
 *   - Shape limits: H % 8 == 0, I % 8 == 0, every shared_I % 8 == 0, 1 <= k_little <= k_big
 *     <= min(E, MOE_MAX_TOPK), E <= MOE_MAX_EXPERTS, n_shared <= MOE_MAX_SHARED,
 *     T * k_big < 2^31 / max(H, I).  Violations give MOE_E_SHAPE / MOE_E_UNSUPPORTED.
 *   - Expert weight blob (one per routed or shared expert, contiguous, 16-byte aligned):
 *         [ W_gate : I x H | W_up : I x H | W_down : H x I ]      (each row-major)
 *     so that one expert is one host-to-device copy.  The feed-forward is SwiGLU:
 *         y = W_down ( silu(W_gate x) * (W_up x) ).
 *     MOE_BF16_W8: the three matrices hold one E4M3 code per weight (OCP 8-bit floating point
 *     "e4m3fn": 1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities), followed by
 *     the fp32 row scales [ s_gate : I | s_up : I | s_down : H ];  W[r][k] = s[r] * e4m3(Q[r][k]).
 *     The codes are widened exactly to bf16, the products accumulate in fp32, and the row's scale
 *     multiplies the sum.
 *     MOE_BF16_MXFP4: the three matrices hold one E2M1 code per weight (1 sign, 2 exponent bits
 *     with bias 1, 1 mantissa bit: 0, 0.5, 1, 1.5, 2, 3, 4, 6 and their negatives), two per byte
 *     with the weight of the even k in the low four bits, followed by the scales
 *     [ S_gate : I x H/32 | S_up : I x H/32 | S_down : H x I/32 ], one E8M0 byte each (2^(b-127);
 *     255 = NaN);  W[r][k] = e8m0(S[r][k/32]) * e2m1(Q[r][k]).  Code times scale is widened
 *     exactly to bf16 (as long as it stays in bf16's range), the products accumulate in fp32.
 *     moe_expert_blob_bytes gives the size of a blob.
 */
#ifndef MOBILE_MOE_H_
#define MOBILE_MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_MAX_SHARED 4
#define MOE_MAX_EXPERTS 256
#define MOE_MAX_TOPK 16

enum { MOE_BF16 = 0, MOE_FP32 = 1, MOE_BF16_W8 = 2, MOE_BF16_MXFP4 = 3 };

enum {
  MOE_OK = 0,
  MOE_E_BADARG = -1,      /* null pointer, negative size, bad enum */
  MOE_E_SHAPE = -2,       /* sizes inconsistent with each other */
  MOE_E_UNSUPPORTED = -3, /* valid but outside the limits listed above */
  MOE_E_HIP = -4,         /* a HIP runtime call failed (message holds its error string) */
  MOE_E_CACHE_FULL = -5,  /* a DEMAND fetch names more experts than the cache has slots */
  MOE_E_WORKSPACE = -6    /* workspace missing, misaligned or too small */
};

/* Layer description shared by all calls of a step. */
typedef struct moe_config {
  int32_t T;        /* tokens in this step (T == 0 is legal: nothing is enqueued)          */
  int32_t H;        /* hidden size                                                          */
  int32_t E;        /* routed experts                                                       */
  int32_t I;        /* intermediate size of a routed expert                                 */
  int32_t k_big;    /* experts of an important token: the model's default K (Sec. III-A)    */
  int32_t k_little; /* experts of every other token: K/2 in the paper, any 1..k_big here    */
  int32_t n_shared; /* always-on shared experts (weight 1, every token); 0 = none           */
  int32_t shared_I[MOE_MAX_SHARED]; /* their intermediate sizes                             */
  int32_t dtype;    /* MOE_BF16 | MOE_FP32: storage of x, Wg, expert blobs, out;
                       MOE_BF16_W8: bf16 x, Wg, out with 8-bit expert blobs;
                       MOE_BF16_MXFP4: bf16 x, Wg, out with MXFP4 expert blobs               */
  int32_t renorm;   /* 0: routing weight = softmax over all E; 1: renormalised over the k_t
                       selected experts                                                     */
  float gamma;      /* fallback threshold of Alg. 1 (paper default 0.7)                     */
} moe_config;

const char* moe_last_error(void);

/* Number of compute units of the current device and the library's build tag (diagnostics). */
int moe_device_info(int32_t* n_cu, int32_t* is_gfx950);

/* Per-kernel timing for measurement runs (not thread-safe; off by default).  While enabled, every
 * kernel launch site of the calls below is bracketed by a pair of HIP events on the call's stream.
 * moe_profile_enable(1) also clears earlier records.  moe_profile_read waits for the events of
 * one kind and returns how many launch sites were recorded and their summed duration.
 * Kinds: 0 router GEMM, 1 softmax/top-k/importance, 2 dispatch, 3 FFN gate+up (SwiGLU),
 * 4 FFN down, 5 combine, 6 token confidence, 7 whole decode step (moe_layer_decode). */
int moe_profile_enable(int on);
int moe_profile_read(int kind, int64_t* launches, double* total_ms);

/* Measurement aid, not part of the method: one kernel that reads `bytes` bytes of the device
 * buffer `buf` (16-byte aligned) once and does nothing else, enqueued on `stream`.  Timing it gives
 * the read bandwidth the device delivers to a plain streaming kernel, the yardstick next to the
 * published peak.  `sink` is a device int32 the kernel may write (it does not for ordinary data). */
int moe_profile_plain_read(const void* buf, size_t bytes, int32_t* sink, void* stream);

/* ------------------------------------------------------------------------------------------
 * Selection stage (Sec. II-A) with the big-little rule (Sec. III-A, Alg. 1).
 *
 *   logits[t][e] = sum_h x[t][h] * Wg[e][h] + gate_bias[e]              (skipped if logits_given)
 *   important[t] = !(conf[t] > gamma)      (equality and NaN fall back; conf NULL: all important)
 *   k_t[t]       = important[t] ? k_big : k_little
 *   topk_idx[t][j], j < k_t[t]: experts in the order (logit descending, expert id ascending),
 *                  taken on the fp32 logits; a NaN logit counts as -inf; -1 for j >= k_t[t]
 *   topk_w[t][j] = softmax over all E logits at topk_idx[t][j] (divided by the sum over the
 *                  k_t selected if cfg->renorm); 0 for j >= k_t[t]
 *
 * Because the little selection is a prefix of the big one, a token's fallback re-run with
 * k_big experts reuses the first k_little experts of its little pass (Sec. III-A).
 *
 * x        device [T,H] dtype          Wg        device [E,H] dtype
 * gate_bias device [E] fp32 or NULL    conf      device [T] fp32 or NULL
 * logits   device [T,E] fp32: output, or input when logits_given != 0 (x, Wg may then be NULL)
 * topk_idx device [T,k_big] int32      topk_w    device [T,k_big] fp32
 * important device [T] uint8           k_t       device [T] int32
 */
int moe_route(const moe_config* cfg, const void* x, const void* Wg, const float* gate_bias,
              const float* conf, float* logits, int logits_given, int32_t* topk_idx,
              float* topk_w, uint8_t* important, int32_t* k_t, void* stream);

/* Confidence of Alg. 1 / Sec. III-B: the largest probability of the model's output
 * distribution, conf[t] = max_v softmax(lm_logits[t])_v = 1 / sum_v exp(z_tv - max_v z_tv).
 * lm_logits device [T,V] fp32, conf device [T] fp32. */
int moe_token_confidence(const float* lm_logits, int32_t T, int32_t V, float* conf, void* stream);

/* ------------------------------------------------------------------------------------------
 * Token-to-expert dispatch with a variable expert count per token: the (t, j < k_t[t]) pairs
 * are put in the unique order (expert ascending, token ascending) the execution stage
 * (Sec. II-A) consumes.  P = sum_t k_t[t].
 *
 *   expert_offsets device [E+1] int32  exclusive prefix of pairs per expert; [E] = P
 *   sorted_token   device [T*k_big]    token of the pair at each position, -1 beyond P
 *   sorted_rank    device [T*k_big]    rank j of that pair,                -1 beyond P
 *   inv_pos        device [T,k_big]    position of pair (t,j),             -1 for j >= k_t[t]
 * Integer-only and deterministic: the order comes from scans and prefix sums (the only atomics
 * are LDS integer additions into histograms, whose result does not depend on their order).
 * Precondition: the experts topk_idx names for one token (ranks below k_t) are distinct, as
 * moe_route produces them; for a selection that repeats an expert within a token the positions of
 * the repeated entries are unspecified.
 */
size_t moe_dispatch_workspace_bytes(const moe_config* cfg);
int moe_dispatch(const moe_config* cfg, const int32_t* topk_idx, const int32_t* k_t,
                 int32_t* expert_offsets, int32_t* sorted_token, int32_t* sorted_rank,
                 int32_t* inv_pos, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Execution stage (Sec. II-A): grouped SwiGLU feed-forward over the dispatched pairs, plus
 * the always-on shared experts.
 *
 *   for every routed expert e with expert_w[e] != NULL and position p in
 *   [expert_offsets[e], expert_offsets[e+1]):     y[p][:] = FFN_e( x[sorted_token[p]][:] )
 *   for every shared expert s and token t:        FFN_s( x[t][:] ) is written as one or more partial
 *            sums over slices of the intermediate dimension, one [T,H] slab of shared_out each;
 *            the sum of all S = moe_shared_out_slabs(cfg) slabs is sum_s FFN_s(x[t]).
 *
 * expert_w   DEVICE array of E device pointers to expert blobs.  A NULL entry skips that
 *            expert (its rows of y are left untouched): this is how a step is run in several
 *            waves when the HBM cache holds fewer experts than the step needs.
 * shared_w   HOST array of n_shared device pointers (ignored when run_shared == 0)
 * y          device [T*k_big, H] fp32 (rows >= P untouched)
 * shared_out device [S, T, H] fp32, S = moe_shared_out_slabs(cfg) >= n_shared (NULL allowed when
 *            nothing shared is run)
 * run_routed / run_shared  select which of the two parts this call computes
 * ws         device scratch holding the SwiGLU activations
 * The number of pairs per expert is read on the device; the host never waits for it.
 */
size_t moe_expert_ffn_workspace_bytes(const moe_config* cfg);
/* Bytes of one expert blob with intermediate size I (cfg->I for a routed expert, cfg->shared_I[s]
 * for a shared one) in cfg->dtype; 0 on a bad config or I. */
size_t moe_expert_blob_bytes(const moe_config* cfg, int32_t I);
int32_t moe_shared_out_slabs(const moe_config* cfg); /* 0 without shared experts; -1 on a bad config */
int moe_expert_ffn(const moe_config* cfg, const void* x, const int32_t* expert_offsets,
                   const int32_t* sorted_token, const void* const* expert_w,
                   const void* const* shared_w, int run_routed, int run_shared, float* y,
                   float* shared_out, void* ws, size_t ws_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): moe_expert_ffn with the SwiGLU activations kept in a
 * buffer that is built into the library (device memory of moe_expert_ffn_static_max_bytes() =
 * 8 MiB per GPU, held until the process ends) instead of a caller workspace.  Same arguments,
 * results and errors as moe_expert_ffn otherwise; it calls no allocating routine.  A step whose
 * moe_expert_ffn_workspace_bytes(cfg) exceeds the built-in buffer gets MOE_E_WORKSPACE and
 * enqueues nothing.  All calls on one GPU share the buffer: calls that may overlap on that GPU
 * (different streams without ordering between them) race; calls on one stream are safe. */
size_t moe_expert_ffn_static_max_bytes(void);
int moe_expert_ffn_static(const moe_config* cfg, const void* x, const int32_t* expert_offsets,
                          const int32_t* sorted_token, const void* const* expert_w,
                          const void* const* shared_w, int run_routed, int run_shared, float* y,
                          float* shared_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * "... and finally summed" (Sec. II-A):
 *   out[t][:] = sum_{j < k_t[t]} topk_w[t][j] * y[inv_pos[t][j]][:]  +  sum_s shared_out[s][t][:]
 * with s over the S slabs that moe_expert_ffn wrote; summed in fp32 in ascending j, then ascending
 * s, rounded once.   out device [T,H] dtype.
 */
int moe_combine(const moe_config* cfg, const float* y, const float* topk_w,
                const int32_t* inv_pos, const int32_t* k_t, const float* shared_out, void* out,
                void* stream);

/* ------------------------------------------------------------------------------------------
 * One decode step of the layer in ONE kernel launch: moe_route + moe_dispatch + moe_expert_ffn +
 * moe_combine (selection and execution stage of Sec. II-A with the per-token expert count of
 * Sec. III-A / Alg. 1) for steps of at most 64 tokens, dtype MOE_BF16 or MOE_BF16_W8.  Same
 * arithmetic and the same outputs as the four calls: logits, topk_idx, topk_w, important, k_t,
 * expert_offsets, sorted_token, sorted_rank, inv_pos, y, shared_out and out are all written and
 * have the layouts documented above.  A decode step only streams 0.1 .. 1 GB of weights, so the
 * launch gaps and pipeline ramps of five dependent kernels are a large part of it; here the
 * shared experts (which need nothing from the router) stream while the selection is computed,
 * and the down projections, the final sum and the next weights overlap inside one persistent
 * kernel whose workgroups hand results over through device memory.
 *
 * expert_w  DEVICE array of E device pointers; every expert the step selects must be non-NULL
 *           (an expert with a NULL entry is skipped and its rows of y keep their old contents)
 * shared_w  HOST array of n_shared device pointers
 * ws        device workspace of moe_layer_decode_workspace_bytes(cfg) bytes, 256-byte aligned.
 *           It starts with the kernel's hand-over counters: call moe_layer_decode_init on it once
 *           before its first use (enqueues a clear on `stream`); every step leaves them at zero.
 *           Steps that share a workspace must not overlap (one stream, or ordered streams).
 * Every wait inside the kernel is bounded; moe_layer_decode_status (synchronous, for tests and
 * diagnostics) returns how many waits have ever given up on this workspace: 0 in a healthy run.
 * Errors: MOE_E_UNSUPPORTED for fp32 layers and for T > 64 (use the separate calls).
 */
size_t moe_layer_decode_workspace_bytes(const moe_config* cfg);
int moe_layer_decode_init(void* ws, size_t ws_bytes, void* stream);
int moe_layer_decode_status(const void* ws, int32_t* timed_out_waits);
int moe_layer_decode(const moe_config* cfg, const void* x, const void* Wg, const float* gate_bias,
                     const float* conf, const void* const* expert_w, const void* const* shared_w,
                     float* logits, int logits_given, int32_t* topk_idx, float* topk_w,
                     uint8_t* important, int32_t* k_t, int32_t* expert_offsets, int32_t* sorted_token,
                     int32_t* sorted_rank, int32_t* inv_pos, float* y, float* shared_out, void* out,
                     void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Second pass of Alg. 1 at layer level.  Alg. 1 runs the little model (k_little experts per token)
 * and, for a token whose result is rejected (confidence not above gamma), the big model
 * (k_big experts, Sec. III-A: same router).  With routing weights that are not renormalised
 * (cfg->renorm == 0) the big model's layer output is the little one's plus the experts of ranks
 * k_little .. k_big-1, so the re-do only has to compute those:
 *
 *   pass 1  moe_route (conf = NULL is NOT little: pass a confidence above gamma for every token),
 *           moe_dispatch, moe_expert_ffn, moe_combine                    -> out = little output
 *   pass 2  moe_route(logits_given = 1, conf = the tokens' confidences)  -> k_t = k_big where rejected
 *           moe_dispatch_from(j_lo = k_little)    pairs (t, j) with j_lo <= j < k_t[t] only;
 *                                                 inv_pos = -1 for every other rank
 *           moe_expert_ffn(run_shared = 0)        the shared experts are part of pass 1
 *           moe_combine_add(j_lo = k_little)      out[t] += sum_{j_lo <= j < k_t[t]} w[t][j] y[inv_pos[t][j]]
 *
 * moe_dispatch_from has the arguments, outputs and workspace of moe_dispatch; moe_dispatch is
 * j_lo = 0.  moe_combine_add reads and rewrites out [T,H] (storage dtype; fp32 sum in ascending j,
 * one more rounding) for the tokens with k_t[t] > j_lo and leaves the others untouched; it
 * returns MOE_E_UNSUPPORTED when cfg->renorm != 0, because then the weights of the ranks below
 * j_lo differ between the two models.  0 <= j_lo <= k_big, else MOE_E_BADARG.
 */
int moe_dispatch_from(const moe_config* cfg, const int32_t* topk_idx, const int32_t* k_t, int32_t j_lo,
                      int32_t* expert_offsets, int32_t* sorted_token, int32_t* sorted_rank,
                      int32_t* inv_pos, void* ws, size_t ws_bytes, void* stream);
int moe_combine_add(const moe_config* cfg, const float* y, const float* topk_w, const int32_t* inv_pos,
                    const int32_t* k_t, int32_t j_lo, void* out, void* stream);

/* ------------------------------------------------------------------------------------------
 * Fallback fetch and prefetch of expert weights (Sec. II-B: experts stay in host DRAM and are
 * loaded when the router asks for them; Sec. III-B: for a token that falls back, the router
 * outputs of its discarded little pass name the experts of the big pass ahead of time, for
 * any number of layers ahead).
 *
 * The cache is a set of n_slots HBM slots of blob_bytes each, filled by hipMemcpyAsync from a
 * pinned host arena holding all E blobs back to back, on two side streams of default priority
 * (one carries the DEMAND copies, one the PREFETCH copies, so that a copy a step waits for does
 * not queue behind copies started on a prediction).
 * Policy (deterministic, host-side integers only; it depends on the sequence of calls alone):
 *   - every call advances a logical clock; every expert the call names that is resident
 *     afterwards gets that time stamp
 *   - MOE_FETCH_DEMAND: n <= n_slots distinct experts.  Resident ones are hits.  Misses are
 *     loaded in ascending expert id; the victim is the least recently stamped slot that holds
 *     no expert of this call, lowest slot id first among equals (empty slots are oldest).
 *     The compute stream is made to wait for the copies, and the device pointer table
 *     (moe_cache_expert_table) is rewritten on the compute stream so that exactly the experts
 *     of this call point at their slots and all others are NULL.
 *   - MOE_FETCH_PREFETCH: any n, experts in priority order.  Resident ones are re-stamped.
 *     A miss is loaded only if a victim exists that is neither named by this call nor part of
 *     the most recent DEMAND call; otherwise it is dropped (slot_of = -1; nothing is queued for
 *     later).  moe_cache_set_prefetch_limit bounds the copies one PREFETCH call may start; misses
 *     beyond the bound are dropped too.  The pointer table and the compute stream are not touched.
 *   - Ordering against the compute stream: the kernels that read the slots handed out by a DEMAND
 *     call must be enqueued on compute_stream before the NEXT DEMAND call on the cache (PREFETCH
 *     calls may come at any time in between).  A copy that replaces a slot's expert starts only
 *     after the work that was on the compute stream at the time of that next DEMAND call has
 *     finished, and after any earlier copy into the same slot.
 */
typedef struct moe_cache moe_cache_t;

enum { MOE_FETCH_DEMAND = 0, MOE_FETCH_PREFETCH = 1 };

typedef struct moe_fetch_stats {
  int32_t hits;       /* named experts already resident                 */
  int32_t misses;     /* experts copied by this call                    */
  int32_t dropped;    /* PREFETCH only: misses without an evictable slot */
  int32_t reserved;
  uint64_t bytes_h2d; /* misses * blob_bytes                            */
} moe_fetch_stats;

/* host_blobs: pinned host memory, E * blob_bytes, must outlive the cache.
 * device_slots: device memory, n_slots * blob_bytes, caller-owned, 256-byte aligned.
 * Creates the side stream and the events; returns NULL on failure (see moe_last_error). */
moe_cache_t* moe_cache_create(int32_t E, size_t blob_bytes, int32_t n_slots,
                              const void* host_blobs, void* device_slots);
void moe_cache_destroy(moe_cache_t* cache);

/* DEVICE array of E device pointers, owned by the cache: pass it as expert_w. */
const void* const* moe_cache_expert_table(moe_cache_t* cache);

/* expert_ids host [n]; slot_of host [n] out (slot index, or -1 when dropped); stats may be NULL.
 * compute_stream: the stream the consuming kernels run on. */
int expert_cache_fetch(moe_cache_t* cache, const int32_t* expert_ids, int32_t n, int32_t mode,
                       int32_t* slot_of, moe_fetch_stats* stats, void* compute_stream);

/* The execution stage of one step when the routed experts live in host DRAM (Sec. II-B): copies
 * expert_offsets to the host and WAITS for it (the one host synchronisation of such a step: the
 * router decides which experts must be loaded), then runs the shared experts and, in waves of at
 * most n_slots experts (resident ones first), expert_cache_fetch(DEMAND) + the grouped FFN of
 * that wave's experts.  Arguments as moe_expert_ffn; total (sum of the waves' statistics) and
 * n_waves may be NULL. */
int moe_expert_ffn_cached(const moe_config* cfg, moe_cache_t* cache, const void* x,
                          const int32_t* expert_offsets, const int32_t* sorted_token,
                          const void* const* shared_w, float* y, float* shared_out, void* ws,
                          size_t ws_bytes, moe_fetch_stats* total, int32_t* n_waves, void* stream);

/* Host-side view of the cache state (tests, metrics): resident_expert host [n_slots] out,
 * -1 for an empty slot.  Returns n_slots. */
int moe_cache_snapshot(moe_cache_t* cache, int32_t* resident_expert);

/* Blocks the host until every copy issued so far has landed (tests, shutdown). */
int moe_cache_sync(moe_cache_t* cache);

/* Depth of the prefetch queue (Sec. III-B: how far ahead experts are loaded is adjustable): a
 * PREFETCH call starts at most max_copies_per_call copies and drops its other misses; negative =
 * no bound (the default). */
int moe_cache_set_prefetch_limit(moe_cache_t* cache, int32_t max_copies_per_call);

/* Measurement aid: emulates a slower host link (the paper's system loads over PCIe 4.0).  Every
 * copy of this cache is followed by a hold of blob_bytes / gb_per_s, and all emulated copies of a
 * device, whichever cache and copy stream carries them, run one after the other in the order in
 * which they were issued (one link, one queue), so that the link delivers
 * 1 / (1/link + 1/gb_per_s).  0 = off (the default). */
int moe_cache_emulate_link(moe_cache_t* cache, double gb_per_s);

/* ---- Prefetch scheduler over a stack of layers (Sec. III-B) -----------------------------------
 * When a token's little pass is rejected, the router outputs of that pass are known for all
 * layers, and the big pass that follows will most likely select the same experts; they are
 * requested `distance` layers ahead of the layer that is being computed (one layer ahead on a
 * fast link, two or three on a slow one).  The scheduler owns no cache and no stream: it turns
 * router logits into one request list per layer and issues expert_cache_fetch(PREFETCH) calls on
 * the layers' caches at the points of a pass the caller reports.  Host-side object; calls on one
 * scheduler are not thread-safe. */
typedef struct moe_prefetcher moe_prefetcher_t;

/* caches: host array of n_layers caches (kept by pointer; they must outlive the scheduler and
 * all hold the same number of experts).  k_big: experts predicted per rejected token and layer.
 * Returns NULL on error. */
moe_prefetcher_t* moe_prefetcher_create(int32_t n_layers, moe_cache_t* const* caches, int32_t k_big);
void moe_prefetcher_destroy(moe_prefetcher_t* p);

/* Bound on the PREFETCH copies in flight over all layers (the depth of the prefetch queue): an
 * advance call starts at most as many copies as keep the number of prefetch copies that have not
 * landed yet within the bound, and drops the rest.  Negative = no bound (the default).  With a
 * bound, what a call starts depends on how far earlier copies have come. */
int moe_prefetcher_set_in_flight_limit(moe_prefetcher_t* p, int32_t max_copies_in_flight);

/* With on != 0, a request made while a DEMAND copy of any of the layers is still in flight starts
 * no copy (it runs under the bound 0: resident experts of the list are kept fresh, missing ones
 * are dropped), so that a copy the step is waiting for never shares the link with a copy started
 * on a prediction.  Off by default.  Like the bound above, it makes what a call starts depend on
 * timing. */
int moe_prefetcher_set_yield_to_demand(moe_prefetcher_t* p, int32_t on);

/* New prediction from one pass's router states.  layer_logits: host array of n_layers DEVICE
 * pointers to that pass's router logits [T, E] fp32 (as moe_route wrote them); rejected: host
 * [n_rejected], the tokens of the pass whose little result was dropped.  Copies the logits to the
 * host on `stream` and WAITS for them.  The request list of a layer is the rejected tokens'
 * selection under the layer's own rule (k_big experts; logit descending, expert id ascending, NaN
 * as -infinity), rank by rank (every token's first choice, then every token's second, ...), each
 * expert once.  n_rejected == 0 clears the prediction (no copy, no wait). */
int moe_prefetcher_predict(moe_prefetcher_t* p, const float* const* layer_logits, int32_t T,
                           const int32_t* rejected, int32_t n_rejected, void* stream);

/* The request list of a layer: ids host [E] out; returns its length (or a negative error). */
int moe_prefetcher_predicted(moe_prefetcher_t* p, int32_t layer, int32_t* ids);

/* A point of the pass that follows the prediction.  layer == -1: the pass starts (the lists of
 * layers 0 .. distance-1 are requested); layer == l >= 0: layer l is about to run (the list of
 * layer l + distance is requested, if there is such a layer).  distance == 0 requests nothing.
 * Layers with an empty list are skipped.  Per request made, in order: issued_layers[i] (the
 * layer), limits_used[i] (the bound on copies the call ran under, negative = none) and
 * issued_stats[i]; each host [n_layers] out or NULL.  compute_stream as in expert_cache_fetch.
 * Returns the number of requests made (>= 0) or a negative error. */
int moe_prefetcher_advance(moe_prefetcher_t* p, int32_t layer, int32_t distance, int32_t* issued_layers,
                           int32_t* limits_used, moe_fetch_stats* issued_stats, void* compute_stream);

#ifdef __cplusplus
}
#endif
#endif /* MOBILE_MOE_H_ */
