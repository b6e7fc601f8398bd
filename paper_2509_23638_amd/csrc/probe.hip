// Measurement aids: a plain streaming copy and a plain streaming read (with and
// without the non-temporal hint), 16 bytes per lane, and the stage loop of the
// tiled FFN kernels on its own.  They give the achievable HBM rate of the box the roofline
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

// The stage loop of the tiled FFN kernels and nothing else: what a compute unit
// can take in while it streams weights.  One workgroup of eight waves per
// compute unit; per stage it fetches 16 KiB of "weights" (its own stream through
// `w`, one KiB per instruction, non-temporal) and NTOK x 8 KiB of "token rows"
// (8 rows x 128 B per instruction out of a 2 MiB matrix of 256 rows that stays in
// L2) with the direct-to-LDS load, into a ring of three buffers with two stages
// in flight, behind a counted vmcnt wait and a bare barrier.  Nothing is
// multiplied.  Loads complete in order, so "at most one stage's loads
// outstanding" says the stage at hand has landed.
constexpr int kStageWaves = 8;
constexpr int kStageWorkgroups = 256;
constexpr size_t kStageTokenBytes = 256 * 8192;

template <int NTOK>
__global__ __launch_bounds__(kStageWaves * 64, 1) void probe_stage_kernel(const unsigned char* __restrict__ w,
                                                                          size_t w_stride,
                                                                          const unsigned char* __restrict__ tok,
                                                                          int stages) {
  extern __shared__ __attribute__((aligned(16))) unsigned char ring[];
  constexpr int PER = 2 + NTOK;                       // loads per wave and stage
  constexpr int SLOT = PER * kStageWaves * 1024;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const unsigned char* wp = w + (size_t)blockIdx.x * w_stride + (size_t)wave * 2048 + lane * 16;
  const unsigned char* tp[NTOK > 0 ? NTOK : 1];
#pragma unroll
  for (int q = 0; q < NTOK; ++q) {
    const int grp = (wave + 8 * q + blockIdx.x) & 31;   // 8 of the 256 rows
    tp[q] = tok + (size_t)(grp * 8 + (lane >> 3)) * 8192 + (lane & 7) * 16;
  }
  auto issue = [&](int st) {
    unsigned char* base = ring + (st % 3) * SLOT + wave * PER * 1024;
#pragma unroll
    for (int q = 0; q < 2; ++q)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(wp + (size_t)st * (kStageWaves * 2048) + q * 1024),
          (__attribute__((address_space(3))) void*)(base + q * 1024), 16, 0, 2);
#pragma unroll
    for (int q = 0; q < NTOK; ++q)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(tp[q] + (st & 63) * 128),
          (__attribute__((address_space(3))) void*)(base + (2 + q) * 1024), 16, 0, 0);
  };
  issue(0);
  issue(1);
  for (int st = 0; st < stages; ++st) {
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(PER) : "memory");
    issue(st + 2 < stages ? st + 2 : stages - 1);     // the tail re-reads the last stage: equal counts
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <int NTOK>
moe_status launch_probe_stage(const void* w, size_t w_stride, const void* tok, int stages, hipStream_t stream) {
  const int lds = 3 * (2 + NTOK) * kStageWaves * 1024;
  MOE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&probe_stage_kernel<NTOK>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  hipLaunchKernelGGL(probe_stage_kernel<NTOK>, dim3(kStageWorkgroups), dim3(kStageWaves * 64), lds, stream,
                     static_cast<const unsigned char*>(w), w_stride, static_cast<const unsigned char*>(tok),
                     stages);
  MOE_HIP(hipGetLastError());
  return MOE_OK;
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

extern "C" moe_status moe_probe_stage(const void* weights, size_t weight_bytes, const void* tokens,
                                      size_t token_bytes, int32_t token_fetches, int32_t stages,
                                      void* stream) {
  MOE_REQUIRE(weights && tokens, "moe_probe_stage: NULL pointer argument");
  MOE_REQUIRE(token_fetches >= 0 && token_fetches <= 4, "moe_probe_stage: token_fetches must be 0..4");
  MOE_REQUIRE(stages >= 2 && stages <= (1 << 20), "moe_probe_stage: stages must be 2..2^20");
  // every workgroup walks its own stages x 16 KiB; the token matrix is 256 rows of 8 KiB
  const size_t w_stride = (size_t)stages * moe::kStageWaves * 2048;
  MOE_REQUIRE(weight_bytes >= w_stride * moe::kStageWorkgroups,
              "moe_probe_stage: weights must hold 256 x stages x 16 KiB");
  MOE_REQUIRE(token_bytes >= moe::kStageTokenBytes, "moe_probe_stage: tokens must hold 2 MiB");
  hipStream_t s = static_cast<hipStream_t>(stream);
  switch (token_fetches) {
    case 0: return moe::launch_probe_stage<0>(weights, w_stride, tokens, stages, s);
    case 1: return moe::launch_probe_stage<1>(weights, w_stride, tokens, stages, s);
    case 2: return moe::launch_probe_stage<2>(weights, w_stride, tokens, stages, s);
    case 3: return moe::launch_probe_stage<3>(weights, w_stride, tokens, stages, s);
    default: return moe::launch_probe_stage<4>(weights, w_stride, tokens, stages, s);
  }
}
