// Measurement aids: a plain streaming copy and a plain streaming read (with and
// without the non-temporal hint), 16 bytes per lane.  They give the achievable HBM rate of the box the roofline
// fraction is quoted next to, and a dispatch of known size against which
// hardware byte counters can be scaled.
#include "common.h"

namespace moe {
namespace {

__global__ __launch_bounds__(256) void probe_copy_kernel(uint4* __restrict__ dst,
                                                         const uint4* __restrict__ src, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// NT: the loads carry the non-temporal hint (lines are not kept in L2), as the
// weight streams of the FFN kernels do.
template <bool NT>
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ src, size_t n,
                                                         uint32_t* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  uint32_t acc = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4* q = reinterpret_cast<const u32x4*>(src + i);
    const u32x4 v = NT ? __builtin_nontemporal_load(q) : *q;
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  // data-dependent, practically never true: keeps the loads alive
  if (acc == 0x9e3779b9u) sink[0] = acc;
}

template <bool NT>
moe_status launch_probe_read(const void* src, size_t bytes, void* sink4, void* stream) {
  const size_t n = bytes / 16;
  if (n == 0) return MOE_OK;
  const int blocks = (int)((n + 255) / 256 < 256 * 32 ? (n + 255) / 256 : 256 * 32);
  hipLaunchKernelGGL(probe_read_kernel<NT>, dim3(blocks), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(src), n,
                     static_cast<uint32_t*>(sink4));
  MOE_HIP(hipGetLastError());
  return MOE_OK;
}

}  // namespace
}  // namespace moe

extern "C" moe_status moe_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
  MOE_REQUIRE(dst && src && bytes % 16 == 0, "moe_probe_copy: NULL pointer or size not a multiple of 16");
  const size_t n = bytes / 16;
  if (n == 0) return MOE_OK;
  const int blocks = (int)((n + 255) / 256 < 256 * 32 ? (n + 255) / 256 : 256 * 32);
  hipLaunchKernelGGL(moe::probe_copy_kernel, dim3(blocks), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<uint4*>(dst),
                     static_cast<const uint4*>(src), n);
  MOE_HIP(hipGetLastError());
  return MOE_OK;
}

extern "C" moe_status moe_probe_read(const void* src, size_t bytes, void* sink4, void* stream) {
  MOE_REQUIRE(src && sink4 && bytes % 16 == 0, "moe_probe_read: NULL pointer or size not a multiple of 16");
  return moe::launch_probe_read<false>(src, bytes, sink4, stream);
}

extern "C" moe_status moe_probe_read_nt(const void* src, size_t bytes, void* sink4, void* stream) {
  MOE_REQUIRE(src && sink4 && bytes % 16 == 0,
              "moe_probe_read_nt: NULL pointer or size not a multiple of 16");
  return moe::launch_probe_read<true>(src, bytes, sink4, stream);
}
