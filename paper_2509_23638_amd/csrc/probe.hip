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
// weight streams of the FFN kernels do, and a wavefront has eight 1 KiB loads
// in flight over 8 KiB in a row -- the shape that reads fastest on this part.
template <bool NT>
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ src, size_t n,
                                                         uint32_t* __restrict__ sink) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  uint32_t acc = 0;
  if (NT) {
    constexpr int kBurst = 8;
    const int lane = threadIdx.x & 63;
    const size_t waves = (size_t)gridDim.x * (blockDim.x >> 6);
    const size_t wave = (size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const size_t chunks = n / (64 * kBurst);          // whole 8 KiB chunks
    for (size_t c = wave; c < chunks; c += waves) {
      u32x4 v[kBurst];
#pragma unroll
      for (int q = 0; q < kBurst; ++q)
        v[q] = __builtin_nontemporal_load(
            reinterpret_cast<const u32x4*>(src + (c * kBurst + q) * 64 + lane));
#pragma unroll
      for (int q = 0; q < kBurst; ++q) acc ^= v[q].x ^ v[q].y ^ v[q].z ^ v[q].w;
    }
    // the tail that does not fill a chunk
    for (size_t i = chunks * 64 * kBurst + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x) {
      const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + i));
      acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
  } else {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
      const uint4 v = src[i];
      acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
  }
  // data-dependent, practically never true: keeps the loads alive
  if (acc == 0x9e3779b9u) sink[0] = acc;
}

template <bool NT>
moe_status launch_probe_read(const void* src, size_t bytes, void* sink4, void* stream) {
  const size_t n = bytes / 16;
  if (n == 0) return MOE_OK;
  // plain: many small steps; bursts: two workgroups per compute unit
  const int cap = NT ? 512 : 256 * 32;
  const int blocks = (int)((n + 255) / 256 < (size_t)cap ? (n + 255) / 256 : cap);
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
