// One-time re-layout of an expert matrix for the matrix cores (bf16 storage).
//
// The paper fixes no memory layout for the three matrices of an expert
// (Section 4.4 only names them).  Row-major [N, K] makes a wavefront that feeds
// v_mfma_f32_16x16x32_bf16 touch 16 rows x 64 bytes per load instruction; the
// tiled layout stores every 16-row x 32-column MFMA operand tile as one
// contiguous KiB, lane by lane, so the same load reads 1 KiB in a row:
//
//   tile (n16, ks)  at element offset  (n16 * (K/32) + ks) * 512
//   inside a tile, lane l = r + 16 g (r = row in the tile, g = 8-column group)
//   holds W[16 n16 + r][32 ks + 8 g .. 8 g + 7]  at element offset 8 l.
//
// A tile's bytes are exactly what lane l of a wavefront needs as its A operand.
#include "common.h"

namespace moe {
namespace {

__global__ __launch_bounds__(256) void pack_kernel(const uint4* __restrict__ src,
                                                   uint4* __restrict__ dst, int N, int K) {
  // one thread per 16-byte unit of the destination
  const size_t units = (size_t)N * K / 8;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const int ksteps = K / 32;
  for (size_t u = (size_t)blockIdx.x * blockDim.x + threadIdx.x; u < units; u += stride) {
    const int lane = (int)(u & 63);
    const size_t tile = u >> 6;
    const int ks = (int)(tile % ksteps);
    const size_t n16 = tile / ksteps;
    const int r = lane & 15, g = lane >> 4;
    const size_t row = n16 * 16 + r;
    dst[u] = src[(row * K + (size_t)ks * 32 + g * 8) / 8];
  }
}

}  // namespace
}  // namespace moe

extern "C" moe_status moe_pack_weights(const void* src, void* dst, int32_t N, int32_t K,
                                       void* stream) {
  MOE_REQUIRE(src && dst && src != dst, "moe_pack_weights: NULL pointer or in-place request");
  MOE_REQUIRE(N > 0 && K > 0 && N % 16 == 0 && K % 32 == 0,
              "moe_pack_weights: N must be a multiple of 16 and K of 32 (N=%d K=%d)", N, K);
  const size_t units = (size_t)N * K / 8;
  const int blocks = (int)((units + 255) / 256 < 65536 ? (units + 255) / 256 : 65536);
  hipLaunchKernelGGL(moe::pack_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(src), static_cast<uint4*>(dst), N, K);
  MOE_HIP(hipGetLastError());
  return MOE_OK;
}
