// Gate of the MoE block (paper Section 2.1, "e_i, w_i = Gate(a)"): router GEMM
// with float64 accumulation, k rounds of wave-level arg-max with lowest-index
// tie-break, softmax weights renormalised over the selected experts.
//
// Work split: one workgroup of four wavefronts handles TPB tokens.  Wave w owns
// the experts e with e % 4 == w; every lane covers 8 consecutive hidden
// positions per step, so X and Wr are read with 16-byte (bf16) coalesced loads.
// Per-lane partial sums are reduced over the wave with a butterfly, the logits
// meet in LDS, and wave tk then selects for token tk with one candidate slot
// per lane (two when E > 64).
#include "common.h"

namespace moe {
namespace {

constexpr int kRouteWaves = 4;

template <typename T> struct Load8;

template <> struct Load8<uint16_t> {  // bf16 bits
  static __device__ __forceinline__ void load(const void* base, size_t idx, double (&v)[8]) {
    const uint4 raw = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + idx);
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = (double)__uint_as_float(w[i] << 16);
      v[2 * i + 1] = (double)__uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

template <> struct Load8<float> {
  static __device__ __forceinline__ void load(const void* base, size_t idx, double (&v)[8]) {
    const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + idx);
    const float4 a = p[0], b = p[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, MOE_WAVE);
  return v;
}

// EPW = compile-time bound on experts per wave (keeps accumulators in VGPRs)
template <typename ST, int TPB, int EPW>
__global__ __launch_bounds__(kRouteWaves* MOE_WAVE) void route_kernel(
    const void* __restrict__ X, const void* __restrict__ Wr, const float* __restrict__ bias,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, double* __restrict__ logits_out,
    int T, int H, int E, int k) {
  __shared__ double s_logit[TPB][MOE_MAX_E];

  const int lane = threadIdx.x & (MOE_WAVE - 1);
  const int wave = threadIdx.x / MOE_WAVE;
  const int t0 = blockIdx.x * TPB;

  double acc[EPW][TPB];
#pragma unroll
  for (int i = 0; i < EPW; ++i)
#pragma unroll
    for (int j = 0; j < TPB; ++j) acc[i][j] = 0.0;

  for (int hc = lane * 8; hc < H; hc += MOE_WAVE * 8) {
    double xv[TPB][8];
#pragma unroll
    for (int j = 0; j < TPB; ++j) {
      const int t = min(t0 + j, T - 1);  // clamp: rows past T are never written
      Load8<ST>::load(X, (size_t)t * H + hc, xv[j]);
    }
#pragma unroll
    for (int i = 0; i < EPW; ++i) {
      const int e = wave + i * kRouteWaves;
      if (e < E) {
        double wv[8];
        Load8<ST>::load(Wr, (size_t)e * H + hc, wv);
#pragma unroll
        for (int j = 0; j < TPB; ++j)
#pragma unroll
          for (int q = 0; q < 8; ++q) acc[i][j] = fma(xv[j][q], wv[q], acc[i][j]);
      }
    }
  }

#pragma unroll
  for (int i = 0; i < EPW; ++i) {
    const int e = wave + i * kRouteWaves;
    if (e < E) {
      const double b = bias ? (double)bias[e] : 0.0;
#pragma unroll
      for (int j = 0; j < TPB; ++j) {
        const double s = wave_sum(acc[i][j]) + b;
        if (lane == 0) s_logit[j][e] = s;
      }
    }
  }
  __syncthreads();

  // wave tk selects for token t0 + tk
  for (int tk = wave; tk < TPB; tk += kRouteWaves) {
    const int t = t0 + tk;
    if (t >= T) continue;
    const double ninf = -__builtin_huge_val();
    const double c0 = lane < E ? s_logit[tk][lane] : ninf;
    const double c1 = lane + MOE_WAVE < E ? s_logit[tk][lane + MOE_WAVE] : ninf;
    if (logits_out) {
      if (lane < E) logits_out[(size_t)t * E + lane] = c0;
      if (lane + MOE_WAVE < E) logits_out[(size_t)t * E + lane + MOE_WAVE] = c1;
    }
    bool taken0 = !(lane < E), taken1 = !(lane + MOE_WAVE < E);
    double first = 0.0, mine = 0.0;  // lane j keeps the j-th selected logit
    int my_idx = 0;
    float denom = 0.f;
    for (int j = 0; j < k; ++j) {
      double v;
      int idx;
      if (!taken0 && (taken1 || c0 >= c1)) { v = c0; idx = lane; }
      else if (!taken1) { v = c1; idx = lane + MOE_WAVE; }
      else { v = ninf; idx = 0x7fffffff; }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        const double ov = __shfl_xor(v, off, MOE_WAVE);
        const int oi = __shfl_xor(idx, off, MOE_WAVE);
        if (ov > v || (ov == v && oi < idx)) { v = ov; idx = oi; }
      }
      if (idx == lane) taken0 = true;
      if (idx == lane + MOE_WAVE) taken1 = true;
      if (j == 0) first = v;
      // softmax over all experts renormalised over the selected ones equals a
      // softmax over the selected logits; the largest one is the shift
      const float p = expf((float)(v - first));
      denom += p;
      if (lane == j) { mine = v; my_idx = idx; }
    }
    if (lane < k) {
      topk_idx[(size_t)t * k + lane] = my_idx;
      topk_w[(size_t)t * k + lane] = expf((float)(mine - first)) / denom;
    }
  }
}

template <typename ST, int TPB>
void launch_typed(const moe_shape& s, const void* X, const void* Wr, const float* bias,
                  int32_t* topk_idx, float* topk_w, double* logits_out, hipStream_t stream) {
  const int blocks = (s.T + TPB - 1) / TPB;
  const int epw = (s.E + kRouteWaves - 1) / kRouteWaves;
  dim3 grid(blocks), block(kRouteWaves * MOE_WAVE);
#define ROUTE_LAUNCH(EPW)                                                               \
  hipLaunchKernelGGL((route_kernel<ST, TPB, EPW>), grid, block, 0, stream, X, Wr, bias, \
                     topk_idx, topk_w, logits_out, s.T, s.H, s.E, s.k)
  if (epw <= 2) ROUTE_LAUNCH(2);
  else if (epw <= 8) ROUTE_LAUNCH(8);
  else if (epw <= 16) ROUTE_LAUNCH(16);
  else ROUTE_LAUNCH(32);
#undef ROUTE_LAUNCH
}

}  // namespace

moe_status launch_route(const moe_shape& s, const void* X, const void* Wr, const float* bias,
                        int32_t* topk_idx, float* topk_w, double* logits_out,
                        hipStream_t stream) {
  if (s.T == 0) return MOE_OK;
  // many tokens: four tokens share each router-weight load
  const bool many = s.T >= 512 && s.E <= 64;
  if (s.dtype == MOE_BF16) {
    if (many) launch_typed<uint16_t, 4>(s, X, Wr, bias, topk_idx, topk_w, logits_out, stream);
    else launch_typed<uint16_t, 1>(s, X, Wr, bias, topk_idx, topk_w, logits_out, stream);
  } else {
    if (many) launch_typed<float, 4>(s, X, Wr, bias, topk_idx, topk_w, logits_out, stream);
    else launch_typed<float, 1>(s, X, Wr, bias, topk_idx, topk_w, logits_out, stream);
  }
  MOE_HIP(hipGetLastError());
  return MOE_OK;
}

}  // namespace moe

extern "C" moe_status moe_route(const moe_shape* shape, const void* X, const void* Wr,
                                const float* bias, int32_t* topk_idx, float* topk_w,
                                double* logits_out, void* stream) {
  moe_status st = moe::check_shape(shape, "moe_route");
  if (st != MOE_OK) return st;
  if (shape->T == 0) return MOE_OK;
  MOE_REQUIRE(X && Wr && topk_idx && topk_w, "moe_route: NULL pointer argument");
  return moe::launch_route(*shape, X, Wr, bias, topk_idx, topk_w, logits_out,
                           static_cast<hipStream_t>(stream));
}
