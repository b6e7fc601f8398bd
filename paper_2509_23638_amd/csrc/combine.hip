// Weighted combine back to token order (paper Section 2.1:
// x' = sum_j w_j * Expert_j(a)), plus the unweighted shared-expert rows and an
// optional residual.  A gather-sum in float32 in a fixed order (slot 0..k-1,
// then shared experts, then the residual): no atomics, one rounding to the
// storage dtype at the end.  The rows of Y are float32, or (YB) bf16 rows that
// moe_layer_forward keeps at prefill sizes: widened exactly, same order of sums.
#include "common.h"

namespace moe {
namespace {

template <bool YB>
__device__ __forceinline__ float4 load_y4(const void* Y, size_t at) {
  if (YB) {
    const uint2 r = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(Y) + at);
    return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u),
                       __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xffff0000u));
  }
  return *reinterpret_cast<const float4*>(static_cast<const float*>(Y) + at);
}

template <bool BF16, bool YB>
__global__ __launch_bounds__(256) void combine_kernel(const void* __restrict__ Y,
                                                      const float* __restrict__ topk_w,
                                                      const int32_t* __restrict__ inv_perm,
                                                      const void* __restrict__ residual,
                                                      void* __restrict__ out, int T, int H, int k,
                                                      int S) {
  const int t = blockIdx.x;            // tokens along x: the only grid dimension that can hold 2^24
  const int h4 = (blockIdx.y * blockDim.x + threadIdx.x) * 4;
  if (h4 >= H) return;
  const int A = T * k;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int j = 0; j < k; ++j) {
    const int p = inv_perm[t * k + j];
    if (p < 0) continue;
    const float w = topk_w[t * k + j];
    const float4 y = load_y4<YB>(Y, (size_t)p * H + h4);
    acc.x = fmaf(w, y.x, acc.x);
    acc.y = fmaf(w, y.y, acc.y);
    acc.z = fmaf(w, y.z, acc.z);
    acc.w = fmaf(w, y.w, acc.w);
  }
  for (int s = 0; s < S; ++s) {
    const float4 y = load_y4<YB>(Y, (size_t)(A + s * T + t) * H + h4);
    acc.x += y.x; acc.y += y.y; acc.z += y.z; acc.w += y.w;
  }
  if (BF16) {
    if (residual) {
      const uint2 r = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(residual) + (size_t)t * H + h4);
      acc.x += __uint_as_float(r.x << 16);
      acc.y += __uint_as_float(r.x & 0xffff0000u);
      acc.z += __uint_as_float(r.y << 16);
      acc.w += __uint_as_float(r.y & 0xffff0000u);
    }
    uint2 o;
    o.x = pack_bf16x2(acc.x, acc.y);
    o.y = pack_bf16x2(acc.z, acc.w);
    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(out) + (size_t)t * H + h4) = o;
  } else {
    if (residual) {
      const float4 r = *reinterpret_cast<const float4*>(static_cast<const float*>(residual) + (size_t)t * H + h4);
      acc.x += r.x; acc.y += r.y; acc.z += r.z; acc.w += r.w;
    }
    *reinterpret_cast<float4*>(static_cast<float*>(out) + (size_t)t * H + h4) = acc;
  }
}

}  // namespace

moe_status launch_combine(const moe_shape& s, const void* Y, const float* topk_w,
                          const int32_t* inv_perm, const void* residual, void* out,
                          hipStream_t stream, bool y_bf16) {
  if (s.T == 0) return MOE_OK;
  if (y_bf16 && s.dtype != MOE_BF16) return fail(MOE_ERR_UNSUPPORTED, "bf16 rows of Y need bf16 storage");
  dim3 grid(s.T, (s.H / 4 + 255) / 256), block(256);
  if (y_bf16)
    hipLaunchKernelGGL((combine_kernel<true, true>), grid, block, 0, stream, Y, topk_w, inv_perm, residual,
                       out, s.T, s.H, s.k, s.S);
  else if (s.dtype == MOE_BF16)
    hipLaunchKernelGGL((combine_kernel<true, false>), grid, block, 0, stream, Y, topk_w, inv_perm, residual,
                       out, s.T, s.H, s.k, s.S);
  else
    hipLaunchKernelGGL((combine_kernel<false, false>), grid, block, 0, stream, Y, topk_w, inv_perm,
                       residual, out, s.T, s.H, s.k, s.S);
  MOE_HIP(hipGetLastError());
  return MOE_OK;
}

}  // namespace moe

extern "C" moe_status moe_combine(const moe_shape* shape, const float* Y, const float* topk_w,
                                  const int32_t* inv_perm, const void* residual, void* out,
                                  void* stream) {
  moe_status st = moe::check_shape(shape, "moe_combine");
  if (st != MOE_OK) return st;
  if (shape->T == 0) return MOE_OK;
  MOE_REQUIRE(Y && topk_w && inv_perm && out, "moe_combine: NULL pointer argument");
  return moe::launch_combine(*shape, Y, topk_w, inv_perm, residual, out,
                             static_cast<hipStream_t>(stream), false);
}
