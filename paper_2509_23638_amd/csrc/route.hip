// Gate of the MoE block (paper Section 2.1, "e_i, w_i = Gate(a)"): router GEMM
// with float64 accumulation, k rounds of wave-level arg-max with lowest-index
// tie-break, softmax weights renormalised over the selected experts.
//
// Work split: one workgroup of NW wavefronts handles TPB tokens.  Wave w owns
// the experts e with e % NW == w; every lane covers 8 consecutive hidden
// positions per step, so X and Wr are read with 16-byte (bf16) coalesced loads,
// several steps' loads in flight at once.  Per-lane partial sums are folded to
// one value per 16-lane row with DPP moves, the four row partials meet in LDS,
// and wave tk then selects for token tk by rank: lane e counts the experts
// that beat expert e (two candidates per lane when E > 64) -- no cross-lane
// traffic at all in the selection.
#include "common.h"

namespace moe {
namespace {


// Eight consecutive stored values: fetched raw (so that many fetches can be in
// flight in few registers) and widened to float64 only when they are used.
template <typename T> struct Load8;

template <> struct Load8<uint16_t> {  // bf16 bits
  typedef uint4 Raw;
  static __device__ __forceinline__ Raw fetch(const void* base, size_t idx) {
    return *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + idx);
  }
  static __device__ __forceinline__ void widen(const Raw& raw, double (&v)[8]) {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = (double)__uint_as_float(w[i] << 16);
      v[2 * i + 1] = (double)__uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

template <> struct Load8<float> {
  struct Raw { float4 a, b; };
  static __device__ __forceinline__ Raw fetch(const void* base, size_t idx) {
    const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + idx);
    Raw r;
    r.a = p[0];
    r.b = p[1];
    return r;
  }
  static __device__ __forceinline__ void widen(const Raw& r, double (&v)[8]) {
    v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w;
    v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
  }
};

// Sum over the 16 lanes of a DPP row, left in every lane of the row: xor-1 and
// xor-2 inside quads, then the mirrored half-row and row.  Fixed tree, so the
// float64 result is the same from run to run.
__device__ __forceinline__ double dpp_f64(double v, const int ctrl_tag) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  switch (ctrl_tag) {
    case 0: lo = __builtin_amdgcn_update_dpp(0, lo, 0xB1, 0xF, 0xF, false);
            hi = __builtin_amdgcn_update_dpp(0, hi, 0xB1, 0xF, 0xF, false); break;   // quad_perm [1,0,3,2]
    case 1: lo = __builtin_amdgcn_update_dpp(0, lo, 0x4E, 0xF, 0xF, false);
            hi = __builtin_amdgcn_update_dpp(0, hi, 0x4E, 0xF, 0xF, false); break;   // quad_perm [2,3,0,1]
    case 2: lo = __builtin_amdgcn_update_dpp(0, lo, 0x141, 0xF, 0xF, false);
            hi = __builtin_amdgcn_update_dpp(0, hi, 0x141, 0xF, 0xF, false); break;  // row_half_mirror
    default: lo = __builtin_amdgcn_update_dpp(0, lo, 0x140, 0xF, 0xF, false);
             hi = __builtin_amdgcn_update_dpp(0, hi, 0x140, 0xF, 0xF, false); break; // row_mirror
  }
  return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double row16_sum(double v) {
  v += dpp_f64(v, 0);
  v += dpp_f64(v, 1);
  v += dpp_f64(v, 2);
  v += dpp_f64(v, 3);
  return v;
}

// Rank of candidate c (expert index e) among the E logits of one token: the
// number of experts that beat it, where o beats e if its logit is larger, or
// equal with a lower index -- the order k rounds of arg-max with lowest-index
// ties produce.  The logits are read from LDS eight at a time so that the
// reads overlap instead of costing one LDS round trip each.
__device__ __forceinline__ void ranks_of(const double* logit, int E, double c0, int e0, double c1,
                                         int e1, int& r0, int& r1) {
  r0 = 0;
  r1 = 0;
  for (int ob = 0; ob < E; ob += 8) {
    double v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = logit[min(ob + u, E - 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int o = ob + u;
      const bool in = o < E;
      r0 += (in && (v[u] > c0 || (v[u] == c0 && o < e0))) ? 1 : 0;
      r1 += (in && (v[u] > c1 || (v[u] == c1 && o < e1))) ? 1 : 0;
    }
  }
}

// NW  = wavefronts per workgroup; wave w owns the experts e with e % NW == w
// TPB = tokens per workgroup (they share every router-weight fetch)
// EPW = compile-time bound on experts per wave (keeps accumulators in VGPRs)
// UNR = hidden-dimension steps (512 positions each) whose fetches are issued together
template <typename ST, int NW, int TPB, int EPW, int UNR>
__global__ __launch_bounds__(NW* MOE_WAVE) void route_kernel(
    const void* __restrict__ X, const void* __restrict__ Wr, const float* __restrict__ bias,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, double* __restrict__ logits_out,
    int T, int H, int E, int k) {
  __shared__ double s_row[TPB][MOE_MAX_E][4];   // one partial per 16-lane row
  __shared__ double s_logit[TPB][MOE_MAX_E];
  __shared__ double s_sel[TPB][MOE_MAX_K];

  const int lane = threadIdx.x & (MOE_WAVE - 1);
  const int wave = threadIdx.x / MOE_WAVE;
  const int t0 = blockIdx.x * TPB;

  double acc[EPW][TPB];
#pragma unroll
  for (int i = 0; i < EPW; ++i)
#pragma unroll
    for (int j = 0; j < TPB; ++j) acc[i][j] = 0.0;

  for (int base = 0; base < H; base += UNR * MOE_WAVE * 8) {
    // Every fetch of this step is issued before anything is used (raw form:
    // 4 registers per 8 bf16 values), so the step costs one round trip to
    // memory.  No branch on the expert index: a wave's slots past E re-read
    // the last expert's row and accumulate a value nobody stores, which keeps
    // the body straight-line.
    typename Load8<ST>::Raw xraw[UNR][TPB], wraw[UNR][EPW];
    bool live[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int hc = base + u * MOE_WAVE * 8 + lane * 8;
      live[u] = hc < H;
      const size_t at = live[u] ? hc : 0;   // dead lanes re-read column 0 and are zeroed below
#pragma unroll
      for (int j = 0; j < TPB; ++j)
        xraw[u][j] = Load8<ST>::fetch(X, (size_t)min(t0 + j, T - 1) * H + at);
#pragma unroll
      for (int i = 0; i < EPW; ++i)
        wraw[u][i] = Load8<ST>::fetch(Wr, (size_t)min(wave + i * NW, E - 1) * H + at);
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      double xv[TPB][8];
#pragma unroll
      for (int j = 0; j < TPB; ++j) {
        Load8<ST>::widen(xraw[u][j], xv[j]);
        if (!live[u])
#pragma unroll
          for (int q = 0; q < 8; ++q) xv[j][q] = 0.0;
      }
#pragma unroll
      for (int i = 0; i < EPW; ++i) {
        double wv[8];
        Load8<ST>::widen(wraw[u][i], wv);
#pragma unroll
        for (int j = 0; j < TPB; ++j)
#pragma unroll
          for (int q = 0; q < 8; ++q) acc[i][j] = fma(xv[j][q], wv[q], acc[i][j]);
      }
    }
  }

  // lane partials -> one partial per 16-lane row -> LDS
#pragma unroll
  for (int i = 0; i < EPW; ++i) {
    const int e = wave + i * NW;
    if (e < E) {
#pragma unroll
      for (int j = 0; j < TPB; ++j) {
        const double r = row16_sum(acc[i][j]);
        if ((lane & 15) == 0) s_row[j][e][lane >> 4] = r;
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < TPB * E; i += NW * MOE_WAVE) {
    const int j = TPB == 1 ? 0 : i / E, e = i - j * E;
    const double b = bias ? (double)bias[e] : 0.0;
    const double v = ((s_row[j][e][0] + s_row[j][e][1]) + (s_row[j][e][2] + s_row[j][e][3])) + b;
    s_logit[j][e] = v;
    if (logits_out && t0 + j < T) logits_out[(size_t)(t0 + j) * E + e] = v;
  }
  __syncthreads();

  // wave tk selects for token t0 + tk: lane e ranks expert e (and e + 64)
  const int tk = wave;
  const bool mine = tk < TPB && t0 + tk < T;
  if (mine) {
    const double ninf = -__builtin_huge_val();
    const int e0 = lane, e1 = lane + MOE_WAVE;
    const double c0 = e0 < E ? s_logit[tk][e0] : ninf;
    const double c1 = e1 < E ? s_logit[tk][e1] : ninf;
    int r0, r1;
    ranks_of(s_logit[tk], E, c0, e0, c1, e1, r0, r1);
    const size_t t = (size_t)(t0 + tk);
    if (e0 < E && r0 < k) { s_sel[tk][r0] = c0; topk_idx[t * k + r0] = e0; }
    if (e1 < E && r1 < k) { s_sel[tk][r1] = c1; topk_idx[t * k + r1] = e1; }
  }
  __syncthreads();
  if (mine && lane < k) {
    // softmax over all experts renormalised over the selected ones equals a
    // softmax over the selected logits; the largest one is the shift
    const double first = s_sel[tk][0];
    float denom = 0.f;
    for (int j = 0; j < k; ++j) denom += expf((float)(s_sel[tk][j] - first));
    topk_w[(size_t)(t0 + tk) * k + lane] = expf((float)(s_sel[tk][lane] - first)) / denom;
  }
}

template <typename ST>
void launch_typed(const moe_shape& s, const void* X, const void* Wr, const float* bias,
                  int32_t* topk_idx, float* topk_w, double* logits_out, hipStream_t stream) {
#define ROUTE_LAUNCH(NW, TPB, EPW, UNR)                                                        \
  hipLaunchKernelGGL((route_kernel<ST, NW, TPB, EPW, UNR>), dim3((s.T + TPB - 1) / TPB),       \
                     dim3(NW * MOE_WAVE), 0, stream, X, Wr, bias, topk_idx, topk_w, logits_out, \
                     s.T, s.H, s.E, s.k)
  // float32 rows take twice the registers per fetch: half the steps in flight
  constexpr int W = sizeof(ST) == 2 ? 2 : 1;
  if (s.T >= 512 && s.E <= 64) {
    // many tokens: throughput matters; two tokens share each router-weight fetch
    if (s.E <= 8) ROUTE_LAUNCH(4, 2, 2, 2 * W);
    else if (s.E <= 32) ROUTE_LAUNCH(4, 2, 8, W);
    else ROUTE_LAUNCH(4, 2, 16, 1);
  } else {
    // few tokens: latency matters; eight waves per token, as much of the
    // hidden dimension in flight per wave as the registers allow
    if (s.E <= 8) ROUTE_LAUNCH(8, 1, 1, 4 * W);
    else if (s.E <= 32) ROUTE_LAUNCH(8, 1, 4, 2 * W);
    else if (s.E <= 64) ROUTE_LAUNCH(8, 1, 8, 2 * W);
    else ROUTE_LAUNCH(8, 1, 16, W);
  }
#undef ROUTE_LAUNCH
}

}  // namespace

moe_status launch_route(const moe_shape& s, const void* X, const void* Wr, const float* bias,
                        int32_t* topk_idx, float* topk_w, double* logits_out,
                        hipStream_t stream) {
  if (s.T == 0) return MOE_OK;
  if (s.dtype == MOE_BF16) launch_typed<uint16_t>(s, X, Wr, bias, topk_idx, topk_w, logits_out, stream);
  else launch_typed<float>(s, X, Wr, bias, topk_idx, topk_w, logits_out, stream);
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
