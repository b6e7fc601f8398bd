// Glue between the layers of a stack of MoE blocks: weightless RMS
// normalisation of the residual stream, x / sqrt(mean(x^2) + eps), computed in
// float32 and rounded once to the storage dtype.  (The paper's block takes the
// already normalised attention output; a stack of MoE blocks alone needs this
// to keep the residual stream finite.)
#include "common.h"

namespace moe {
namespace {

template <bool BF16>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const void* __restrict__ X,
                                                      void* __restrict__ out, int H, float eps) {
  __shared__ float s_part[4];
  const int t = blockIdx.x;
  const int lane = threadIdx.x & (MOE_WAVE - 1), wave = threadIdx.x / MOE_WAVE;
  float ss = 0.f;
  for (int h = threadIdx.x; h < H; h += blockDim.x) {
    const float v = BF16 ? bf16_bits_to_f32(static_cast<const uint16_t*>(X)[(size_t)t * H + h])
                         : static_cast<const float*>(X)[(size_t)t * H + h];
    ss = fmaf(v, v, ss);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, MOE_WAVE);
  if (lane == 0) s_part[wave] = ss;
  __syncthreads();
  const float tot = s_part[0] + s_part[1] + s_part[2] + s_part[3];
  const float scale = 1.0f / sqrtf(tot / (float)H + eps);
  for (int h = threadIdx.x; h < H; h += blockDim.x) {
    if (BF16) {
      const float v = bf16_bits_to_f32(static_cast<const uint16_t*>(X)[(size_t)t * H + h]);
      static_cast<uint16_t*>(out)[(size_t)t * H + h] = f32_to_bf16_bits(v * scale);
    } else {
      static_cast<float*>(out)[(size_t)t * H + h] = static_cast<const float*>(X)[(size_t)t * H + h] * scale;
    }
  }
}

}  // namespace
}  // namespace moe

extern "C" moe_status moe_rmsnorm(const moe_shape* shape, const void* X, void* out, float eps,
                                  void* stream) {
  moe_status st = moe::check_shape(shape, "moe_rmsnorm");
  if (st != MOE_OK) return st;
  if (shape->T == 0) return MOE_OK;
  MOE_REQUIRE(X && out, "moe_rmsnorm: NULL pointer argument");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (shape->dtype == MOE_BF16)
    hipLaunchKernelGGL(moe::rmsnorm_kernel<true>, dim3(shape->T), dim3(256), 0, s, X, out, shape->H, eps);
  else
    hipLaunchKernelGGL(moe::rmsnorm_kernel<false>, dim3(shape->T), dim3(256), 0, s, X, out, shape->H, eps);
  MOE_HIP(hipGetLastError());
  return MOE_OK;
}
