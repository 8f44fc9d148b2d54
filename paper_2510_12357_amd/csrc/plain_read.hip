// Measurement aid: a plain streaming read of a device buffer, the yardstick for what the
// memory system of the device delivers to a kernel that does nothing but read.  The shape is the
// best of those tried on MI355X: one workgroup of four waves per compute unit, every lane 16
// loads of 16 bytes in flight with the non-temporal policy, all workgroups moving through the
// buffer side by side (7.2 TB/s; without the policy 6.4, with 8192 workgroups 6.4, with two
// workgroups per compute unit 6.1 .. 6.6).
#include "internal.h"

namespace mm {
namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4;
constexpr int kLoads = 16;
constexpr int kThreadsR = 256;

__global__ __launch_bounds__(kThreadsR) void plain_read_kernel(const i32x4* __restrict__ p, size_t n16, int32_t* sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  i32x4 acc = {0, 0, 0, 0};
  for (; i + (kLoads - 1) * stride < n16; i += kLoads * stride) {
    i32x4 v[kLoads];
#pragma unroll
    for (int u = 0; u < kLoads; ++u) v[u] = __builtin_nontemporal_load(p + i + u * stride);
#pragma unroll
    for (int u = 0; u < kLoads; ++u) acc ^= v[u];
  }
  for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(p + i);
  // every load feeds the value that decides about the store, so none can be dropped
  const int x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
  if (x == 0x5ca1ab1e) sink[0] = x;
}

}  // namespace
}  // namespace mm

extern "C" int moe_profile_plain_read(const void* buf, size_t bytes, int32_t* sink, void* stream) {
  using namespace mm;
  if (!buf || !sink || ((uintptr_t)buf & 15) || bytes < 16) return fail(MOE_E_BADARG, "moe_profile_plain_read: buf %p (16-byte aligned), %zu bytes, sink %p", buf, bytes, (void*)sink);
  const size_t n16 = bytes / 16;
  size_t grid = (n16 + (size_t)kThreadsR * kLoads - 1) / ((size_t)kThreadsR * kLoads);
  const size_t cus = (size_t)device_cu_count();
  if (grid > cus) grid = cus;
  hipLaunchKernelGGL(plain_read_kernel, dim3((unsigned)grid), dim3(kThreadsR), 0, static_cast<hipStream_t>(stream),
                     static_cast<const i32x4*>(buf), n16, sink);
  return hip_fail(hipGetLastError(), "plain_read_kernel launch");
}
