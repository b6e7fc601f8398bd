// Gate of the MoE block (paper Section 2.1, "e_i, w_i = Gate(a)"): router GEMM
// with float64 accumulation, selection of the k largest logits with
// lowest-index tie-break, softmax weights renormalised over the selected
// experts.
//
// Logits, three forms chosen by shape:
//  * few experts (E <= 8): one workgroup per token, 8 waves x 64 lanes split
//    the hidden dimension, and the same launch selects;
//  * few tokens, many experts: blocks of (4 or 16) tokens x 4 experts, so that
//    every workgroup reads only its rows of Wr and the router matrix is spread
//    over the chip instead of being pulled whole into every compute unit;
//    inside a wave the four 16-lane rows hold four token sets and a row's 16
//    lanes split the hidden dimension (256 contiguous bytes per row and fetch);
//  * many tokens: 16 x 16 tiles on the float64 matrix cores.
// Per-lane partial sums fold with DPP moves, waves' partials meet in LDS, all
// in a fixed order.  Selection: one wavefront per token, k rounds of arg-max
// over 64-bit sortable keys, reducing only the keys' high words unless lanes
// tie on them.
#include "common.h"

#include <stdlib.h>

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

// Order-preserving map of a finite float64 to an unsigned key: larger value,
// larger key; -0.0 and +0.0 share a key (the +0.0 folds the sign of zero) so
// that they tie like the float64 comparison says.  Every real key is above 0,
// which marks "no candidate".
__device__ __forceinline__ uint64_t sortable_key(double v) {
  const uint64_t u = (uint64_t)__double_as_longlong(v + 0.0);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

// Maximum over the wavefront, returned uniform: xor-1 / xor-2 inside quads,
// mirrored half-row and row (every lane of a 16-lane row then holds the row
// maximum), then the four rows' values are read out and combined as scalars.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false));
  v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false));
  const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
  const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
  const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
  const uint32_t d = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
  return max(max(a, b), max(c, d));
}

__device__ __forceinline__ double readlane_f64(double v, int lane_uniform) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane_uniform);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane_uniform);
  return __hiloint2double(hi, lo);
}

// Selection for one token by one wavefront: k rounds of arg-max with the
// lowest index winning ties (exactly the reference's selection), then the
// renormalised softmax weights.  Lane l offers experts l (logit c0) and l + 64
// (c1) as 64-bit sortable keys, the better of the two per round.  A round
// reduces only the keys' high words over the wave (32-bit maximum through DPP);
// the low words, and then the expert indices, are consulted only when several
// lanes share the leading word -- a wave-uniform, rarely taken branch.  The
// r-th winner's logit and index are parked in lane r, so the weights need one
// expf per lane and no LDS.  Every lane of the wave must call this.
// Where a launch of ONE token also leaves its buckets (count [E], offset
// [E+1], perm [k], inv_perm [k], as permute_kernel writes them); all NULL
// otherwise.
struct OneTokenBuckets {
  int32_t *count, *offset, *perm, *inv_perm;
};

__device__ __forceinline__ void select_topk(double c0, double c1, int E, int k, bool store, size_t t,
                                            int lane, int32_t* __restrict__ topk_idx,
                                            float* __restrict__ topk_w,
                                            OneTokenBuckets one = OneTokenBuckets{nullptr, nullptr, nullptr, nullptr},
                                            int32_t* lds_sel = nullptr) {
  const int e0 = lane, e1 = lane + MOE_WAVE;
  uint64_t key0 = e0 < E ? sortable_key(c0) : 0ull;
  uint64_t key1 = e1 < E ? sortable_key(c1) : 0ull;
  double sel_v = 0.0;
  int32_t sel_i = 0;
  for (int r = 0; r < k; ++r) {
    const bool first = key0 >= key1;                   // equal keys: the lower index
    const uint64_t best = first ? key0 : key1;
    const uint32_t hi = (uint32_t)(best >> 32), lo = (uint32_t)best;
    const uint32_t idx = first ? e0 : e1;
    const uint32_t top = wave_max_u32(hi);
    uint64_t m = __builtin_amdgcn_ballot_w64(hi == top);
    if (__popcll(m) > 1) {
      const bool in = hi == top;
      const uint32_t top_lo = wave_max_u32(in ? lo : 0u);
      m = __builtin_amdgcn_ballot_w64(in && lo == top_lo);
      if (__popcll(m) > 1) {
        const bool in2 = in && lo == top_lo;
        const uint32_t low_idx = wave_max_u32(in2 ? ~idx : 0u);   // largest ~idx = smallest index
        m = __builtin_amdgcn_ballot_w64(in2 && ~idx == low_idx);
      }
    }
    const int winner = __ffsll((unsigned long long)m) - 1;       // uniform; m is never empty
    const double wv = readlane_f64(first ? c0 : c1, winner);
    const int32_t wi = __builtin_amdgcn_readlane((int)idx, winner);
    if (lane == r) { sel_v = wv; sel_i = wi; }
    if (lane == winner) { if (first) key0 = 0ull; else key1 = 0ull; }
  }
  // softmax over all experts renormalised over the selected ones equals a
  // softmax over the selected logits; the largest one (lane 0's) is the shift.
  // k <= 16: the selected values sit in the first 16-lane row.
  const double top_v = readlane_f64(sel_v, 0);
  float ex = lane < k ? expf((float)(sel_v - top_v)) : 0.f;
  float sum = ex;
  sum += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(sum), 0xB1, 0xF, 0xF, false));
  sum += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(sum), 0x4E, 0xF, 0xF, false));
  sum += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(sum), 0x141, 0xF, 0xF, false));
  sum += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(sum), 0x140, 0xF, 0xF, false));
  if (store && lane < k) {
    topk_idx[t * k + lane] = sel_i;
    topk_w[t * k + lane] = ex / sum;
    if (lds_sel) lds_sel[t * k + lane] = sel_i;
  }
  // A batch of one token: its k assignments are the whole list, so the buckets
  // are known here and the bucketing launch is saved (a tenth of a one-token
  // layer's dependent launches).  Lane l answers for experts l and l + 64 and,
  // if l < k, for assignment l: count = assignments naming the expert, offset =
  // assignments naming a lower one, position = assignments that sort before
  // this one (lower expert, or the same expert earlier in the list: stable).
  if (one.count != nullptr) {
    int n0 = 0, n1 = 0, less0 = 0, less1 = 0, pos = 0;
    for (int r = 0; r < k; ++r) {
      const int32_t v = __builtin_amdgcn_readlane(sel_i, r);
      n0 += v == e0;
      n1 += v == e1;
      less0 += v < e0;
      less1 += v < e1;
      pos += v < sel_i || (v == sel_i && r < lane);
    }
    if (e0 < E) {
      one.count[e0] = n0;
      one.offset[e0] = less0;
    }
    if (e1 < E) {
      one.count[e1] = n1;
      one.offset[e1] = less1;
    }
    if (lane == 0) one.offset[E] = k;
    if (lane < k) {
      one.perm[pos] = lane;
      one.inv_perm[lane] = pos;
    }
  }
}

// One 128-position step of a wave: raw fetches of TPL token rows and EPW
// router rows (8 positions per lane).  Rows past the batch or the expert list
// re-read the last valid row (their sums are never stored); lanes past H
// re-read column 0 and contribute zeros.
template <typename ST, int EPW, int TPL> struct RouteStep {
  typename Load8<ST>::Raw x[TPL], w[EPW];
  bool live;
  __device__ __forceinline__ void load(const void* X, const void* Wr, int tl, int e0, int T, int E,
                                       int H, int hc) {
    live = hc < H;
    const size_t at = live ? hc : 0;
#pragma unroll
    for (int j = 0; j < TPL; ++j) x[j] = Load8<ST>::fetch(X, (size_t)min(tl + j, T - 1) * H + at);
#pragma unroll
    for (int i = 0; i < EPW; ++i) w[i] = Load8<ST>::fetch(Wr, (size_t)min(e0 + i, E - 1) * H + at);
  }
  __device__ __forceinline__ void mac(double (&acc)[EPW][TPL]) const {
    double xv[TPL][8];
#pragma unroll
    for (int j = 0; j < TPL; ++j) {
      Load8<ST>::widen(x[j], xv[j]);
      if (!live)
#pragma unroll
        for (int q = 0; q < 8; ++q) xv[j][q] = 0.0;
    }
#pragma unroll
    for (int i = 0; i < EPW; ++i) {
      double wv[8];
      Load8<ST>::widen(w[i], wv);
#pragma unroll
      for (int j = 0; j < TPL; ++j)
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[i][j] = fma(xv[j][q], wv[q], acc[i][j]);
    }
  }
};

// Logits of a block of tokens x experts.
// EPW  = experts per workgroup, TPL = tokens per lane.
// RT   = 4: the four 16-lane rows of a wave hold four token sets (a wave covers
//           4*TPL tokens) and a row's 16 lanes split the hidden dimension, 128
//           positions per step;
//        1: all 64 lanes split the hidden dimension, 512 positions per step
//           (a wave covers TPL tokens) -- more lanes per token, for batches too
//           small to fill the chip otherwise.
// KS   = wavefronts that split the hidden dimension (steps round robin).
// UNR  = steps whose fetches are issued together.  PIPE: instead, the next
//        step's fetches are issued before the current step is multiplied (long
//        per-wave loops of the many-token case).
// FUSE = the workgroup holds all E <= EPW logits of its tokens, so it also
//        selects (wave j for token j): one launch for the whole gate.
template <typename ST, int EPW, int TPL, int RT, int KS, int UNR, bool PIPE, bool FUSE>
__global__ __launch_bounds__(KS* MOE_WAVE) void route_logits_kernel(
    const void* __restrict__ X, const void* __restrict__ Wr, const float* __restrict__ bias,
    double* __restrict__ logits, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, int T,
    int H, int E, int k, OneTokenBuckets one) {
  constexpr int TPW = RT * TPL;                      // tokens per workgroup
  constexpr int NP = KS * (4 / RT);                  // partial sums per (expert, token)
  constexpr int PS = RT == 4 ? 128 : 512;            // positions per step
  static_assert(!FUSE || TPW <= KS, "one selecting wave per token");
  __shared__ double s_part[NP][EPW][TPW];
  __shared__ double s_logit[FUSE ? TPW : 1][FUSE ? EPW : 1];

  const int lane = threadIdx.x & (MOE_WAVE - 1);
  const int wave = threadIdx.x / MOE_WAVE;
  const int row = lane >> 4, col = lane & 15;
  const int t0 = blockIdx.x * TPW, e0 = blockIdx.y * EPW;
  const int tl = t0 + (RT == 4 ? row * TPL : 0);     // this lane's first token
  const int hl = (RT == 4 ? col : lane) * 8;         // this lane's offset inside a step
  constexpr int stride = KS * PS;                    // between a wave's steps

  double acc[EPW][TPL];
#pragma unroll
  for (int i = 0; i < EPW; ++i)
#pragma unroll
    for (int j = 0; j < TPL; ++j) acc[i][j] = 0.0;

  typedef RouteStep<ST, EPW, TPL> Step;
  if constexpr (!PIPE) {
    for (int base = wave * PS; base < H; base += UNR * stride) {
      Step st[UNR];
#pragma unroll
      for (int u = 0; u < UNR; ++u) st[u].load(X, Wr, tl, e0, T, E, H, base + u * stride + hl);
#pragma unroll
      for (int u = 0; u < UNR; ++u) st[u].mac(acc);
    }
  } else {
    Step a, b;
    int base = wave * PS;
    if (base < H) a.load(X, Wr, tl, e0, T, E, H, base + hl);
    while (base < H) {
      if (base + stride < H) b.load(X, Wr, tl, e0, T, E, H, base + stride + hl);
      a.mac(acc);
      base += stride;
      if (base >= H) break;
      if (base + stride < H) a.load(X, Wr, tl, e0, T, E, H, base + stride + hl);
      b.mac(acc);
      base += stride;
    }
  }

#pragma unroll
  for (int i = 0; i < EPW; ++i)
#pragma unroll
    for (int j = 0; j < TPL; ++j) {
      const double r = row16_sum(acc[i][j]);
      if (col == 0) {
        if (RT == 4) s_part[wave][i][row * TPL + j] = r;
        else s_part[wave * 4 + row][i][j] = r;
      }
    }
  __syncthreads();
  for (int p = threadIdx.x; p < EPW * TPW; p += KS * MOE_WAVE) {
    const int i = p / TPW, j = p - i * TPW;
    const int e = e0 + i, t = t0 + j;
    double v = s_part[0][i][j];
#pragma unroll
    for (int w = 1; w < NP; ++w) v += s_part[w][i][j];
    v += (bias && e < E) ? (double)bias[e] : 0.0;
    if (e < E && t < T) logits[(size_t)t * E + e] = v;
    if (FUSE) s_logit[j][i] = v;
  }
  if constexpr (FUSE) {
    __syncthreads();
    if (wave < TPW) {                                // whole wavefronts; no barrier below
      const bool store = t0 + wave < T;
      const double c0 = lane < EPW ? s_logit[wave][lane] : 0.0;
      select_topk(c0, 0.0, E, k, store, (size_t)min(t0 + wave, T - 1), lane, topk_idx, topk_w, one);
    }
  }
}

// Logits on the float64 matrix cores: a wavefront owns a 16-token x 16-expert
// tile and multiplies it with v_mfma_f64_16x16x4_f64 -- lane (r = l % 16,
// g = l / 16) supplies X[token r][k] and Wr[expert r][k] for the four k of its
// group g, and holds D[token 4i + g][expert r] in accumulator element i.  A
// lane fetches 8 consecutive hidden positions at a time (one 16-byte load for
// bf16), which feed 8 MFMAs; the k order inside a 32-position step is
// permuted the same way for both operands, so the sums are unaffected.  Each
// widened value is used by 16 multiply-adds instead of one, which is what
// makes this the many-token form: the conversion work of the vector kernel
// is gone and the float64 multiply-add rate is what is left.  KS waves split
// the hidden dimension into contiguous runs and their partial tiles meet in
// LDS; UNR steps are fetched together, one batch ahead of the batch being
// multiplied.
typedef double d4 __attribute__((ext_vector_type(4)));

template <typename ST, int KS, int UNR>
__global__ __launch_bounds__(KS* MOE_WAVE) void route_logits_mfma_kernel(
    const void* __restrict__ X, const void* __restrict__ Wr, const float* __restrict__ bias,
    double* __restrict__ logits, int T, int H, int E) {
  typedef typename Load8<ST>::Raw Raw;
  __shared__ double s_part[KS][16][17];
  const int lane = threadIdx.x & (MOE_WAVE - 1);
  const int wave = threadIdx.x / MOE_WAVE;
  const int r = lane & 15, g = lane >> 4;
  const int t0 = blockIdx.x * 16, e0 = blockIdx.y * 16;
  const size_t xrow = (size_t)min(t0 + r, T - 1) * H;   // rows past the end re-read the last one
  const size_t wrow = (size_t)min(e0 + r, E - 1) * H;

  const int steps = (H + 31) / 32, per_wave = (steps + KS - 1) / KS;
  const int k_end = min((wave + 1) * per_wave * 32, H);

  d4 acc[4];                                            // independent chains
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = d4{0.0, 0.0, 0.0, 0.0};

  struct Batch {
    Raw xr[UNR], wr[UNR];
    __device__ __forceinline__ void load(const void* X, const void* Wr, size_t xrow, size_t wrow,
                                         int at0, int k_end) {
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int hc = at0 + u * 32;
        const size_t at = hc < k_end ? hc : 0;          // past the run: a valid address, zeroed in mac
        xr[u] = Load8<ST>::fetch(X, xrow + at);
        wr[u] = Load8<ST>::fetch(Wr, wrow + at);
      }
    }
    __device__ __forceinline__ void mac(d4 (&acc)[4], int at0, int k_end) const {
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const bool live = at0 + u * 32 < k_end;
        double xv[8], wv[8];
        Load8<ST>::widen(xr[u], xv);
        Load8<ST>::widen(wr[u], wv);
        // a step past the run multiplies zeros: straight-line code schedules
        // better than a branch around the MFMAs
#pragma unroll
        for (int q = 0; q < 8; ++q)
          acc[q & 3] = __builtin_amdgcn_mfma_f64_16x16x4f64(live ? xv[q] : 0.0, wv[q], acc[q & 3], 0, 0, 0);
      }
    }
  };
  Batch a, b;
  int base = wave * per_wave * 32;
  constexpr int adv = UNR * 32;
  if (base < k_end) a.load(X, Wr, xrow, wrow, base + g * 8, k_end);
  while (base < k_end) {
    if (base + adv < k_end) b.load(X, Wr, xrow, wrow, base + adv + g * 8, k_end);
    a.mac(acc, base + g * 8, k_end);
    base += adv;
    if (base >= k_end) break;
    if (base + adv < k_end) a.load(X, Wr, xrow, wrow, base + adv + g * 8, k_end);
    b.mac(acc, base + g * 8, k_end);
    base += adv;
  }
  const d4 sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
#pragma unroll
  for (int i = 0; i < 4; ++i) s_part[wave][4 * i + g][r] = sum[i];
  __syncthreads();
  for (int p = threadIdx.x; p < 256; p += KS * MOE_WAVE) {
    const int j = p >> 4, i = p & 15;
    const int t = t0 + j, e = e0 + i;
    if (t < T && e < E) {
      double v = s_part[0][j][i];
#pragma unroll
      for (int w = 1; w < KS; ++w) v += s_part[w][j][i];
      logits[(size_t)t * E + e] = v + (bias ? (double)bias[e] : 0.0);
    }
  }
}

constexpr int kSelectWaves = 4;   // tokens per selection workgroup
constexpr long kMfmaTiles = 128;   // 16 x 16 logit tiles from which the matrix-core form is used

// Selection as a launch of its own (E larger than one logits block): one
// wavefront per token.
// With `all` set (the launcher passes it for batches of at most kSelectWaves
// tokens, i.e. a single workgroup, and k <= 16) the workgroup also buckets: the
// waves leave their selections in LDS, and the first wave, one lane per
// assignment (at most 64), counts and ranks them exactly as for a single token
// (see select_topk) -- the bucketing launch is saved for these batches too.
__global__ __launch_bounds__(kSelectWaves* MOE_WAVE) void route_select_kernel(
    const double* __restrict__ logits, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    int T, int E, int k, OneTokenBuckets all) {
  __shared__ int32_t s_sel[MOE_WAVE];
  const int lane = threadIdx.x & (MOE_WAVE - 1);
  const int tk = threadIdx.x / MOE_WAVE;
  const int t = min(blockIdx.x * kSelectWaves + tk, T - 1);
  const bool store = blockIdx.x * kSelectWaves + tk < T;
  const int e0 = lane, e1 = lane + MOE_WAVE;
  const double c0 = e0 < E ? logits[(size_t)t * E + e0] : 0.0;
  const double c1 = e1 < E ? logits[(size_t)t * E + e1] : 0.0;
  select_topk(c0, c1, E, k, store, (size_t)t, lane, topk_idx, topk_w, OneTokenBuckets{},
              all.count != nullptr ? s_sel : nullptr);
  if (all.count == nullptr) return;   // uniform over the launch
  __syncthreads();
  if (tk != 0) return;
  const int A = T * k;                // at most 64
  const int32_t mine = lane < A ? s_sel[lane] : 0x7fffffff;
  int n0 = 0, n1 = 0, less0 = 0, less1 = 0, pos = 0;
  for (int i = 0; i < A; ++i) {
    const int32_t v = __builtin_amdgcn_readlane(mine, i);
    n0 += v == e0;
    n1 += v == e1;
    less0 += v < e0;
    less1 += v < e1;
    pos += v < mine || (v == mine && i < lane);
  }
  if (e0 < E) {
    all.count[e0] = n0;
    all.offset[e0] = less0;
  }
  if (e1 < E) {
    all.count[e1] = n1;
    all.offset[e1] = less1;
  }
  if (lane == 0) all.offset[E] = A;
  if (lane < A) {
    all.perm[pos] = lane;
    all.inv_perm[lane] = pos;
  }
}

// Returns true when the launch also selected (fused form).
template <typename ST>
bool launch_logits(const moe_shape& s, const void* X, const void* Wr, const float* bias,
                   double* logits, int32_t* topk_idx, float* topk_w, hipStream_t stream,
                   OneTokenBuckets one) {
#define LOGITS_LAUNCH(EPW, TPL, RT, KS, UNR, PIPE, FUSE)                                        \
  hipLaunchKernelGGL((route_logits_kernel<ST, EPW, TPL, RT, KS, UNR, PIPE, FUSE>),              \
                     dim3((s.T + RT * TPL - 1) / (RT * TPL), (s.E + EPW - 1) / EPW),            \
                     dim3(KS * MOE_WAVE), 0, stream, X, Wr, bias, logits, topk_idx, topk_w,     \
                     s.T, s.H, s.E, s.k, one)
  constexpr bool wide = sizeof(ST) == 4;   // float32 rows take twice the registers per fetch
  auto blocks = [&](int epw, int tpw) {
    return (long)((s.T + tpw - 1) / tpw) * ((s.E + epw - 1) / epw);
  };
  if (s.E <= 8 && s.T <= 1024) {
    // few experts: one workgroup per token holds all its logits and selects in
    // the same launch; 64 lanes x 8 waves split the hidden dimension
    const int steps = (s.H + 8 * 512 - 1) / (8 * 512);   // per wave
    if constexpr (!wide) {
      if (steps >= 2) { LOGITS_LAUNCH(8, 1, 1, 8, 2, false, true); return true; }
    }
    LOGITS_LAUNCH(8, 1, 1, 8, 1, false, true);
    return true;
  }
  static const char* tune = tune_env("MOE_TUNE_ROUTE_MFMA");   // measurement aid: tile threshold
  if (blocks(16, 16) >= (tune ? atol(tune) : kMfmaTiles)) {
    // many tokens: 16 x 16 tiles on the float64 matrix cores; enough waves
    // along the hidden dimension to give every SIMD two
    const long tiles = blocks(16, 16);
    const dim3 grid((s.T + 15) / 16, (s.E + 15) / 16);
#define MFMA_LAUNCH(KS)                                                                         \
  hipLaunchKernelGGL((route_logits_mfma_kernel<ST, KS, wide ? 2 : 4>), grid,                    \
                     dim3(KS * MOE_WAVE), 0, stream, X, Wr, bias, logits, s.T, s.H, s.E)
    if (tiles * 4 >= 2048 || s.H <= 1024) MFMA_LAUNCH(4);
    else MFMA_LAUNCH(8);
#undef MFMA_LAUNCH
    return false;
  }
  // few tokens: latency.  Eight waves split the hidden dimension and fetch all
  // their steps at once where the registers allow; the tile is the largest
  // that still gives every compute unit a workgroup, so that the router matrix
  // is spread over the chip, else the smallest.
  const int steps = (s.H + 8 * 128 - 1) / (8 * 128);   // per wave
  const int depth = wide ? 1 : (steps >= 4 ? 4 : steps >= 2 ? 2 : 1);
  if (blocks(4, 16) >= 256) {
    if constexpr (!wide) { if (depth >= 2) { LOGITS_LAUNCH(4, 4, 4, 8, 2, false, false); return false; } }
    LOGITS_LAUNCH(4, 4, 4, 8, 1, false, false);
  } else if (blocks(4, 8) >= 256) {
    if constexpr (!wide) {
      if (depth == 4) { LOGITS_LAUNCH(4, 2, 4, 8, 4, false, false); return false; }
      if (depth == 2) { LOGITS_LAUNCH(4, 2, 4, 8, 2, false, false); return false; }
    }
    LOGITS_LAUNCH(4, 2, 4, 8, 1, false, false);
  } else {
    if constexpr (!wide) {
      if (depth == 4) { LOGITS_LAUNCH(4, 1, 4, 8, 4, false, false); return false; }
      if (depth == 2) { LOGITS_LAUNCH(4, 1, 4, 8, 2, false, false); return false; }
    }
    LOGITS_LAUNCH(4, 1, 4, 8, 1, false, false);
  }
  return false;
#undef LOGITS_LAUNCH
}

}  // namespace

// `logits` [T,E] float64 is required: an output the caller wants, or scratch.
// With `one` set (a batch of one token) the selecting launch also writes the buckets.
static moe_status route_impl(const moe_shape& s, const void* X, const void* Wr, const float* bias,
                             int32_t* topk_idx, float* topk_w, double* logits, hipStream_t stream,
                             OneTokenBuckets one) {
  if (s.T == 0) return MOE_OK;
  const bool selected = s.dtype == MOE_BF16
      ? launch_logits<uint16_t>(s, X, Wr, bias, logits, topk_idx, topk_w, stream, one)
      : launch_logits<float>(s, X, Wr, bias, logits, topk_idx, topk_w, stream, one);
  MOE_HIP(hipGetLastError());
  if (!selected) {
    hipLaunchKernelGGL(route_select_kernel, dim3((s.T + kSelectWaves - 1) / kSelectWaves),
                       dim3(kSelectWaves * MOE_WAVE), 0, stream, logits, topk_idx, topk_w, s.T, s.E,
                       s.k, one);
    MOE_HIP(hipGetLastError());
  }
  return MOE_OK;
}

moe_status launch_route(const moe_shape& s, const void* X, const void* Wr, const float* bias,
                        int32_t* topk_idx, float* topk_w, double* logits, hipStream_t stream) {
  return route_impl(s, X, Wr, bias, topk_idx, topk_w, logits, stream, OneTokenBuckets{});
}

// Routing for the whole block: for a batch of one token the selecting launch
// buckets as well (`bucketed` says so), else the caller runs launch_permute.
moe_status launch_route_bucket(const moe_shape& s, const void* X, const void* Wr, const float* bias,
                               int32_t* topk_idx, float* topk_w, double* logits, int32_t* count,
                               int32_t* offset, int32_t* perm, int32_t* inv_perm, hipStream_t stream,
                               bool* bucketed) {
  // the fused router of E <= 8 runs one workgroup per token: a single token only; the selecting
  // launch of its own has one workgroup up to kSelectWaves tokens
  const bool fused = s.E <= 8 && s.T <= 1024;   // as launch_logits decides
  *bucketed = s.k <= 16 && (fused ? s.T == 1 : s.T <= kSelectWaves);
  const OneTokenBuckets one = *bucketed ? OneTokenBuckets{count, offset, perm, inv_perm} : OneTokenBuckets{};
  return route_impl(s, X, Wr, bias, topk_idx, topk_w, logits, stream, one);
}

}  // namespace moe

extern "C" moe_status moe_route(const moe_shape* shape, const void* X, const void* Wr,
                                const float* bias, int32_t* topk_idx, float* topk_w,
                                double* logits_out, void* workspace, void* stream) {
  moe_status st = moe::check_shape(shape, "moe_route");
  if (st != MOE_OK) return st;
  if (shape->T == 0) return MOE_OK;
  MOE_REQUIRE(X && Wr && topk_idx && topk_w, "moe_route: NULL pointer argument");
  double* logits = logits_out;
  if (!logits) {
    if (!workspace)
      return moe::fail(MOE_ERR_WORKSPACE, "moe_route: needs logits_out or a workspace for the logits");
    logits = reinterpret_cast<double*>(static_cast<char*>(workspace) +
                                       moe::workspace_layout(*shape).logits);
  }
  return moe::launch_route(*shape, X, Wr, bias, topk_idx, topk_w, logits,
                           static_cast<hipStream_t>(stream));
}
