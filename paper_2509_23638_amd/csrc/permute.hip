// Bucketing of the routed assignments by expert: the per-expert pending-token
// counts the paper's scheduler sorts experts by (Section 4.3.2, Premise 1),
// their exclusive scan, and the stable permutation the grouped FFN consumes.
//
// One workgroup per expert, so the experts' buckets are built in parallel on
// different compute units with no hand-over between them: workgroup e scans all
// A = T*k flat assignment ids (a few tens of KB, L2-resident), counting with
// ballots how many name an expert below e (that is offset[e]) and how many
// name e (count[e]); a second scan writes perm / inv_perm for the ids that
// name e.  Each wavefront (four, or sixteen from 4096 ids) owns a contiguous
// share of the ids, so ranks ascend with the id and the order inside a bucket
// is stable.  All integer work: the result is unique and bit-exact.
#include "common.h"

namespace moe {
namespace {

constexpr int kPermMaxWaves = 16;
constexpr int kPermUnroll = 16;

__global__ __launch_bounds__(kPermMaxWaves * MOE_WAVE) void permute_kernel(
    const int32_t* __restrict__ topk_idx, int32_t* __restrict__ count,
    int32_t* __restrict__ offset, int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
    int A, int E) {
  __shared__ int s_eq[kPermMaxWaves], s_less[kPermMaxWaves];
  const int e = blockIdx.x;
  const int lane = threadIdx.x & (MOE_WAVE - 1);
  const int wave = threadIdx.x / MOE_WAVE, n_waves = blockDim.x / MOE_WAVE;
  // share of the ids owned by this wave, a multiple of the wave width
  const int per = ((A + n_waves - 1) / n_waves + MOE_WAVE - 1) / MOE_WAVE * MOE_WAVE;
  const int lo = min(wave * per, A), hi = min(lo + per, A);   // lo == hi: nothing to scan

  // kPermUnroll independent loads are issued before any of them is used, so a
  // scan costs one memory round trip per 1024 ids instead of one per 64
  int eq = 0, less = 0;
  for (int base = lo; base < hi; base += MOE_WAVE * kPermUnroll) {
    int x[kPermUnroll];
#pragma unroll
    for (int u = 0; u < kPermUnroll; ++u) {
      const int i = base + u * MOE_WAVE + lane;
      x[u] = topk_idx[min(i, hi - 1)];
      if (i >= hi) x[u] = -1;
    }
#pragma unroll
    for (int u = 0; u < kPermUnroll; ++u) {
      eq += __popcll(__ballot(x[u] == e));
      less += __popcll(__ballot(x[u] >= 0 && x[u] < e));
    }
  }
  if (lane == 0) {
    s_eq[wave] = eq;
    s_less[wave] = less;
  }
  __syncthreads();
  int start = 0, total = 0, n = 0;  // bucket start; ids naming e in earlier shares; bucket size
  for (int w = 0; w < n_waves; ++w) {
    start += s_less[w];
    if (w < wave) total += s_eq[w];
    n += s_eq[w];
  }
  if (threadIdx.x == 0) {
    count[e] = n;
    offset[e] = start;
    if (e == E - 1) offset[E] = start + n;
  }
  int run = start + total;
  for (int base = lo; base < hi; base += MOE_WAVE * kPermUnroll) {
    int x[kPermUnroll];
#pragma unroll
    for (int u = 0; u < kPermUnroll; ++u) {
      const int i = base + u * MOE_WAVE + lane;
      x[u] = topk_idx[min(i, hi - 1)];
      if (i >= hi) x[u] = e + 1;   // padding lanes match nothing
    }
#pragma unroll
    for (int u = 0; u < kPermUnroll; ++u) {
      const int i = base + u * MOE_WAVE + lane;
      const unsigned long long m = __ballot(x[u] == e);
      if (x[u] == e) {
        const int pos = run + __popcll(m & ((1ull << lane) - 1ull));
        perm[pos] = i;
        inv_perm[i] = pos;
      } else if (e == 0 && i < hi && (x[u] < 0 || x[u] >= E)) {
        inv_perm[i] = -1;   // out-of-range index: in no bucket
      }
      run += __popcll(m);
    }
  }
}

}  // namespace

moe_status launch_permute(const moe_shape& s, const int32_t* topk_idx, int32_t* count,
                          int32_t* offset, int32_t* perm, int32_t* inv_perm,
                          hipStream_t stream) {
  // a scan is one memory round trip per 1024 ids and wave: more waves for long lists
  const int waves = s.T * s.k >= 4096 ? kPermMaxWaves : 4;
  hipLaunchKernelGGL(permute_kernel, dim3(s.E), dim3(waves * MOE_WAVE), 0, stream, topk_idx, count,
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
