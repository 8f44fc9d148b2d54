// Weighted sum that closes the execution stage (Sec. II-A: the outputs of the selected experts
// are "finally summed"):
//   out[t][:] = sum_{j < k_t[t]} topk_w[t][j] * y[inv_pos[t][j]][:] + sum_s shared_out[s][t][:]
// where s runs over the slabs of shared_out (partial sums of the shared experts' outputs),
// accumulated in fp32 in ascending j, then ascending s, and rounded once to the storage dtype.
// Pure streaming: each thread owns four consecutive columns (16-byte loads, 8/16-byte stores).
#include "internal.h"

namespace mm {
namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
constexpr int kThreads = 256;

template <bool OUT_BF16>
__global__ __launch_bounds__(kThreads) void combine_kernel(
    const float* __restrict__ y, const float* __restrict__ w, const int32_t* __restrict__ inv_pos,
    const int32_t* __restrict__ k_t, const float* __restrict__ shared_out, int n_shared, int T, int H,
    int K, int max_pairs, void* __restrict__ out) {
  const int t = blockIdx.x;
  const int c = (blockIdx.y * kThreads + threadIdx.x) * 4;
  if (c >= H) return;
  int kt = k_t[t];
  kt = kt < 0 ? 0 : (kt > K ? K : kt);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int j = 0; j < kt; ++j) {
    const int p = inv_pos[(size_t)t * K + j];
    if (p < 0 || p >= max_pairs) continue;
    const float wj = w[(size_t)t * K + j];
    const f32x4 v = *reinterpret_cast<const f32x4*>(y + (size_t)p * H + c);
    acc += wj * v;
  }
  for (int s = 0; s < n_shared; ++s)
    acc += *reinterpret_cast<const f32x4*>(shared_out + ((size_t)s * T + t) * H + c);
  if (OUT_BF16) {
    bf16x4 o = {(__bf16)acc[0], (__bf16)acc[1], (__bf16)acc[2], (__bf16)acc[3]};
    *reinterpret_cast<bf16x4*>(static_cast<uint16_t*>(out) + (size_t)t * H + c) = o;
  } else {
    *reinterpret_cast<f32x4*>(static_cast<float*>(out) + (size_t)t * H + c) = acc;
  }
}

// Second pass of Alg. 1 at layer level: a token whose little result was rejected gets the big
// model's layer output.  Both use the same router and weights that are not renormalised, so the
// big output is the little output plus the experts of ranks k_little .. k_t-1:
//   out[t][:] = out[t][:] + sum_{j_lo <= j < k_t[t]} topk_w[t][j] * y[inv_pos[t][j]][:]
// in fp32, ascending j, rounded once more to the storage dtype.  Tokens with k_t <= j_lo are
// not touched.
template <bool OUT_BF16>
__global__ __launch_bounds__(kThreads) void combine_add_kernel(
    const float* __restrict__ y, const float* __restrict__ w, const int32_t* __restrict__ inv_pos,
    const int32_t* __restrict__ k_t, int j_lo, int H, int K, int max_pairs, void* __restrict__ out) {
  const int t = blockIdx.x;
  const int c = (blockIdx.y * kThreads + threadIdx.x) * 4;
  if (c >= H) return;
  int kt = k_t[t];
  kt = kt < 0 ? 0 : (kt > K ? K : kt);
  if (kt <= j_lo) return;
  f32x4 acc;
  if (OUT_BF16) {
    const bf16x4 o = *reinterpret_cast<const bf16x4*>(static_cast<const uint16_t*>(out) + (size_t)t * H + c);
    acc = f32x4{(float)o[0], (float)o[1], (float)o[2], (float)o[3]};
  } else {
    acc = *reinterpret_cast<const f32x4*>(static_cast<const float*>(out) + (size_t)t * H + c);
  }
  for (int j = j_lo; j < kt; ++j) {
    const int p = inv_pos[(size_t)t * K + j];
    if (p < 0 || p >= max_pairs) continue;
    const float wj = w[(size_t)t * K + j];
    const f32x4 v = *reinterpret_cast<const f32x4*>(y + (size_t)p * H + c);
    acc += wj * v;
  }
  if (OUT_BF16) {
    bf16x4 o = {(__bf16)acc[0], (__bf16)acc[1], (__bf16)acc[2], (__bf16)acc[3]};
    *reinterpret_cast<bf16x4*>(static_cast<uint16_t*>(out) + (size_t)t * H + c) = o;
  } else {
    *reinterpret_cast<f32x4*>(static_cast<float*>(out) + (size_t)t * H + c) = acc;
  }
}

}  // namespace

int launch_combine_add(const moe_config& c, const float* y, const float* w, const int32_t* inv_pos,
                       const int32_t* k_t, int j_lo, void* out, hipStream_t s) {
  if (c.T == 0) return MOE_OK;
  const dim3 grid((unsigned)c.T, (unsigned)((c.H / 4 + kThreads - 1) / kThreads));
  if (c.dtype != MOE_FP32)
    hipLaunchKernelGGL(combine_add_kernel<true>, grid, dim3(kThreads), 0, s, y, w, inv_pos, k_t, j_lo, c.H,
                       c.k_big, c.T * c.k_big, out);
  else
    hipLaunchKernelGGL(combine_add_kernel<false>, grid, dim3(kThreads), 0, s, y, w, inv_pos, k_t, j_lo, c.H,
                       c.k_big, c.T * c.k_big, out);
  return hip_fail(hipGetLastError(), "combine_add_kernel launch");
}

int launch_combine(const moe_config& c, const float* y, const float* w, const int32_t* inv_pos,
                   const int32_t* k_t, const float* shared_out, void* out, hipStream_t s) {
  if (c.T == 0) return MOE_OK;
  const dim3 grid((unsigned)c.T, (unsigned)((c.H / 4 + kThreads - 1) / kThreads));
  const int ns = shared_out ? slab_plan(c).n_slabs : 0;
  if (c.dtype != MOE_FP32)
    hipLaunchKernelGGL(combine_kernel<true>, grid, dim3(kThreads), 0, s, y, w, inv_pos, k_t, shared_out,
                       ns, c.T, c.H, c.k_big, c.T * c.k_big, out);
  else
    hipLaunchKernelGGL(combine_kernel<false>, grid, dim3(kThreads), 0, s, y, w, inv_pos, k_t, shared_out,
                       ns, c.T, c.H, c.k_big, c.T * c.k_big, out);
  return hip_fail(hipGetLastError(), "combine_kernel launch");
}

}  // namespace mm
