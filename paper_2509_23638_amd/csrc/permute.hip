// Bucketing of the routed assignments by expert: the per-expert pending-token
// counts the paper's scheduler sorts experts by (Section 4.3.2, Premise 1),
// their exclusive scan, and the stable permutation the grouped FFN consumes.
//
// One workgroup of 16 wavefronts walks the A = T*k flat assignment ids in
// tiles of 1024.  Pass 1 builds the histogram with LDS integer atomics; a
// serial scan over <= 128 experts gives the offsets; pass 2 ranks every
// assignment inside its wavefront with ballots (lanes of equal expert id),
// stitches the wavefronts together through per-wave counts in LDS and writes
// perm / inv_perm.  All integer work: the result is unique and bit-exact.
#include "common.h"

namespace moe {
namespace {

constexpr int kPermThreads = 1024;
constexpr int kPermWaves = kPermThreads / MOE_WAVE;

__global__ __launch_bounds__(kPermThreads) void permute_kernel(
    const int32_t* __restrict__ topk_idx, int32_t* __restrict__ count,
    int32_t* __restrict__ offset, int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
    int A, int E) {
  __shared__ int s_hist[MOE_MAX_E];
  __shared__ int s_base[MOE_MAX_E];               // next free position per expert
  __shared__ int s_wave[kPermWaves][MOE_MAX_E];   // per-wave counts, then offsets

  const int tid = threadIdx.x;
  const int lane = tid & (MOE_WAVE - 1);
  const int wave = tid / MOE_WAVE;

  for (int e = tid; e < E; e += kPermThreads) s_hist[e] = 0;
  __syncthreads();
  for (int i = tid; i < A; i += kPermThreads) {
    const int x = topk_idx[i];
    if (x >= 0 && x < E) atomicAdd(&s_hist[x], 1);
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int e = 0; e < E; ++e) {
      const int c = s_hist[e];
      s_base[e] = run;
      offset[e] = run;
      count[e] = c;
      run += c;
    }
    offset[E] = run;
  }
  __syncthreads();

  const int tiles = (A + kPermThreads - 1) / kPermThreads;
  for (int tile = 0; tile < tiles; ++tile) {
    for (int j = tid; j < kPermWaves * MOE_MAX_E; j += kPermThreads) (&s_wave[0][0])[j] = 0;
    const int i = tile * kPermThreads + tid;
    int x = -1;
    if (i < A) {
      x = topk_idx[i];
      if (x < 0 || x >= E) x = -1;
    }
    // rank among the lanes of this wave that carry the same expert id
    unsigned long long todo = __ballot(x >= 0);
    int rank = 0, group = 0;
    bool leader = false;
    while (todo) {
      const int first = __ffsll((long long)todo) - 1;
      const int lx = __shfl(x, first, MOE_WAVE);
      const unsigned long long same = __ballot(x == lx);
      if (x == lx) {
        rank = __popcll(same & ((1ull << lane) - 1ull));
        group = __popcll(same);
        leader = (lane == first);
      }
      todo &= ~same;
    }
    __syncthreads();  // zeroing done
    if (leader) s_wave[wave][x] = group;
    __syncthreads();
    for (int e = tid; e < E; e += kPermThreads) {
      int run = s_base[e];
      for (int w = 0; w < kPermWaves; ++w) {
        const int c = s_wave[w][e];
        s_wave[w][e] = run;
        run += c;
      }
      s_base[e] = run;
    }
    __syncthreads();
    if (i < A) {
      if (x >= 0) {
        const int pos = s_wave[wave][x] + rank;
        perm[pos] = i;
        inv_perm[i] = pos;
      } else {
        inv_perm[i] = -1;
      }
    }
    __syncthreads();
  }
}

}  // namespace

moe_status launch_permute(const moe_shape& s, const int32_t* topk_idx, int32_t* count,
                          int32_t* offset, int32_t* perm, int32_t* inv_perm,
                          hipStream_t stream) {
  hipLaunchKernelGGL(permute_kernel, dim3(1), dim3(kPermThreads), 0, stream, topk_idx, count,
                     offset, perm, inv_perm, s.T * s.k, s.E);
  MOE_HIP(hipGetLastError());
  return MOE_OK;
}

}  // namespace moe

extern "C" moe_status moe_permute(const moe_shape* shape, const int32_t* topk_idx,
                                  int32_t* count, int32_t* offset, int32_t* perm,
                                  int32_t* inv_perm, void* stream) {
  moe_status st = moe::check_shape(shape, "moe_permute");
  if (st != MOE_OK) return st;
  MOE_REQUIRE(count && offset, "moe_permute: NULL count/offset");
  MOE_REQUIRE(shape->T == 0 || (topk_idx && perm && inv_perm), "moe_permute: NULL pointer argument");
  return moe::launch_permute(*shape, topk_idx, count, offset, perm, inv_perm,
                             static_cast<hipStream_t>(stream));
}
