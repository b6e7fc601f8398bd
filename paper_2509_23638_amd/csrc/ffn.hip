// Grouped SiLU-gated expert FFN over the active experts (paper Section 4.4: an
// expert is gate_proj, up_proj, down_proj; Section 2.1: only the top-k experts
// of a token run).
//
// bf16 storage -- weight-streaming MFMA kernels
// ---------------------------------------------
// At decode sizes every active expert's weights are read once and used for a
// handful of rows, so the kernels are built around the weight stream:
//   * a wavefront owns 16 weight rows per matrix tile and walks the
//     contraction dimension; lane (r = lane % 16, g = lane / 16) loads the 16
//     bytes W[row0 + r][k0 + 8 g .. +7] straight into the register layout the
//     A operand of v_mfma_f32_16x16x32_bf16 wants -- no LDS hop for weights;
//   * the (few) activation rows are the B operand: a workgroup stages them
//     through LDS one 128-wide k-chunk at a time, double buffered, already in
//     fragment order, so every wave's B read is one linear ds_read_b128;
//   * weights of chunk c+1 are in flight while chunk c multiplies.
// Phase 1 (gate/up): tile 0 = 16 rows of Wg, tile 1 = the same rows of Wu, so
// silu(g) * u happens in registers and h is written once, rounded to bf16.
// Phase 2 (down): tile 0/1 = two neighbouring 16-row tiles of Wd; Y is float32.
// Grid = (row slabs, experts in the launch list, 64-row token blocks); blocks
// whose expert has an empty bucket (or no rows in that token block) exit at
// once and read no weights.
//
// f32 storage -- plain float32 FMA kernels (one wavefront per output element
// of a row block), for the small full-precision configuration.
#include "common.h"

#include <math.h>
#include <stdlib.h>

#include <algorithm>
#include <mutex>
#include <type_traits>

namespace moe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
using ActRsrc = __amdgpu_buffer_rsrc_t;   // buffer resource: base, size, range-checked 32-bit offsets

constexpr int kWaves = 4;           // wavefronts per workgroup
constexpr int kThreads = kWaves * MOE_WAVE;
constexpr int kKStep = 32;          // contraction depth of one MFMA
constexpr int kStepsPerChunk = 4;   // k-steps staged per LDS buffer
constexpr int kChunk = kKStep * kStepsPerChunk;  // 128
constexpr int kFragBytes = MOE_WAVE * 16;        // one B fragment in LDS
// TB = 16-row activation tiles per pass: 4 (64 bucket rows).  One LDS buffer
// holds TB * 4 fragments.  (Passes of 128 rows existed: their register budget
// leaves one workgroup per compute unit, and wherever buckets are that long the
// tiled kernels measured faster.)
constexpr int buf_bytes(int tb) { return tb * kStepsPerChunk * kFragBytes; }

enum { kGateUp = 0, kDown = 1, kDownHalves = 2, kDownNarrow = 3 };

struct FfnArgs {
  const uint16_t* act;    // gate/up: X [T,H]; down: h [rows,F]
  const int32_t* perm;
  const int32_t* offset;
  void* out;              // gate/up: h [rows,N] bf16; down: Y [rows,N] f32
  int T, k, E, A;
  int K;                  // contraction length
  int N;                  // output width
  int tiled;              // weights are in the tiled layout (see moe_weight_layout)
  int interleave;         // tiled kernels: deal work items to the XCDs round-robin (see tile_order)
  int heavy_first;        // stream kernels: walk groups and passes backwards (see ffn_stream_kernel)
  int split_tail;         // eight-wave tiled kernel: cut the items of a partly filled last round (see TileSplit)
};

// Element offset of the 16 bytes lane (r, g) feeds the MFMA with for weight tile
// n16 (rows 16 n16 ..), k-step ks, and the element stride from one k-step to
// the next.  Row-major: row (16 n16 + r), columns 32 ks + 8 g.  Tiled: the
// tile is one contiguous KiB and the lane's share sits at 8 * lane.
__device__ __forceinline__ size_t weight_lane_offset(bool tiled, int n16, int K, int lane) {
  return tiled ? (size_t)n16 * (K / kKStep) * 512 + (size_t)lane * 8
               : (size_t)(n16 * 16 + (lane & 15)) * K + (size_t)(lane >> 4) * 8;
}
__device__ __forceinline__ int weight_kstep_stride(bool tiled) { return tiled ? 512 : kKStep; }

// silu(z) = z / (1 + e^-z) with the hardware exponential and reciprocal (1 ulp
// each): the result is rounded to bfloat16 right after.
__device__ __forceinline__ float silu_f(float z) {
  return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z));
}

// RT = 16-row weight tiles per wave and matrix.  A wave holds NA = 2*RT weight
// tiles: gate/up -> tile 2*rt + m is rows (wave*RT + rt)*16.. of Wg (m = 0) or
// Wu (m = 1); down -> tile a is rows (wave*NA + a)*16.. of Wd.  RT = 1 keeps
// many small workgroups in flight (decode, bound by HBM); RT = 2 reuses every
// activation fragment read from LDS for four MFMAs instead of two, which is
// what a compute-heavy batch (prefill) needs.
//
// kDownNarrow: the down projection with ONE tile per wave (a workgroup owns 64
// rows of Wd): twice the workgroups of half the size, for shapes whose few
// hundred 128-row workgroups would fill the chip's workgroup slots one and a
// bit times (the last, nearly empty round costs as much as a full one).
//
// kDownHalves: the wave's two tiles are the SAME 16 rows of Wd over the first
// and the second half of the contraction, summed at the end.  A workgroup then
// owns 64 rows instead of 128, so a Mixtral-shaped down projection has twice
// the workgroups (two per compute unit, like gate/up) and twice the weight
// bytes in flight.  The halves need different activations: LDS holds both.
template <int MODE, int NT, int TB, int RT, bool ONCE>
struct Streamer {
  static constexpr bool kHalves = MODE == kDownHalves;
  static constexpr int NH = kHalves ? 2 : 1;          // activation positions staged per chunk
  static constexpr int kBufBytes = NH * buf_bytes(TB);
  static constexpr int NA = MODE == kDownNarrow ? 1 : 2 * RT;
  int half_chunks = 0;    // kDownHalves: chunks per half of the contraction
  const FfnArgs& a;
  const uint16_t* w[NA];  // this lane's first element in each weight tile
  unsigned char* lds;
  int lane, wave;
  int wstep;              // elements from one k-step of a weight tile to the next
  size_t act_off[NT];     // element offset of this lane's activation row per tile
  // weight chunks held: c .. c+NS-1 (the one-tile form has the registers for one more in flight)
  static constexpr int NS = MODE == kDownNarrow ? 4 : (RT == 1 && !kHalves) ? 3 : 2;
  bf16x8 wreg[NS][kStepsPerChunk][NA];
  uint4 xreg[NS][NH * NT];   // activation fetches in flight, by chunk modulo NS
  f32x4 acc[NA][NT];

  __device__ __forceinline__ Streamer(const FfnArgs& a_) : a(a_) {}

  template <int SET>
  __device__ __forceinline__ void load_weights(int c) {
#pragma unroll
    for (int s = 0; s < kStepsPerChunk; ++s)
#pragma unroll
      for (int i = 0; i < NA; ++i)
        wreg[SET][s][i] = load_weight(w[i] + (size_t)(c * kStepsPerChunk + s) * wstep);
  }

  // ONCE: no other workgroup reads this weight tile (the expert's bucket fits
  // one pass), so it is loaded non-temporal: it is not kept in L2, where it
  // would only push out lines that are read again.  Measured on a
  // Mixtral-shaped layer the weight stream gains 8-10 % from this; with several
  // passes per expert it loses as much.  (A compile-time choice: given both
  // kinds of load behind a run-time flag the compiler emits the plain one.)
  __device__ __forceinline__ bf16x8 load_weight(const uint16_t* p) const {
    const bf16x8* q = reinterpret_cast<const bf16x8*>(p);
    return ONCE ? __builtin_nontemporal_load(q) : *q;
  }

  // wave w fetches k-step w of every tile of chunk c
  template <int SET>
  __device__ __forceinline__ void load_act(int c) {
#pragma unroll
    for (int hf = 0; hf < NH; ++hf)
#pragma unroll
      for (int t = 0; t < NT; ++t)
        xreg[SET][hf * NT + t] = *reinterpret_cast<const uint4*>(
            a.act + act_off[t] + (size_t)(c + hf * half_chunks) * kChunk + wave * kKStep +
            (lane >> 4) * 8);
  }

  template <int SET>
  __device__ __forceinline__ void store_act(int buf) {
#pragma unroll
    for (int q = 0; q < NH * NT; ++q)
      *reinterpret_cast<uint4*>(lds + buf * kBufBytes +
                                ((q * kStepsPerChunk + wave) * MOE_WAVE + lane) * 16) = xreg[SET][q];
  }

  template <int SET>
  __device__ __forceinline__ void multiply(int buf) {
#pragma unroll
    for (int s = 0; s < kStepsPerChunk; ++s) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        if (kHalves) {
#pragma unroll
          for (int i = 0; i < NA; ++i) {
            const bf16x8 b = *reinterpret_cast<const bf16x8*>(
                lds + buf * kBufBytes + (((i * NT + t) * kStepsPerChunk + s) * MOE_WAVE + lane) * 16);
            acc[i][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[SET][s][i], b, acc[i][t], 0, 0, 0);
          }
        } else {
          const bf16x8 b = *reinterpret_cast<const bf16x8*>(
              lds + buf * kBufBytes + ((t * kStepsPerChunk + s) * MOE_WAVE + lane) * 16);
#pragma unroll
          for (int i = 0; i < NA; ++i)
            acc[i][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[SET][s][i], b, acc[i][t], 0, 0, 0);
        }
      }
    }
  }

  // Chunk c multiplies while the weights of the next NS-1 chunks are in flight.
  // Loads complete in order, so what a wait lets stay in flight is whatever was
  // issued after the thing waited for.  The activations of chunk c+1 are
  // written to LDS at the end of step c; they were fetched a whole step
  // earlier, AHEAD of the weights of chunks c+1 and c+2, so waiting for them
  // leaves both of those weight chunks on their way (fetched in the same step,
  // behind the newest weights, they would drain the pipe down to one chunk at
  // every step).
  template <int SET>
  __device__ __forceinline__ void step(int c, int nchunks) {
    if (c + 2 < nchunks) load_act<(SET + 2) % NS>(c + 2);
    if (c + NS - 1 < nchunks) load_weights<(SET + NS - 1) % NS>(c + NS - 1);
    multiply<SET>(c & 1);
    if (c + 1 < nchunks) store_act<(SET + 1) % NS>((c + 1) & 1);
    __syncthreads();
  }

  __device__ __forceinline__ void run() {
    const int nchunks = kHalves ? half_chunks : a.K / kChunk;
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
      for (int t = 0; t < NT; ++t) acc[i][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    load_act<0>(0);
    load_weights<0>(0);
    if (nchunks > 1) load_act<1>(1);
    if (NS >= 3 && nchunks > 1) load_weights<1>(1);
    if (NS >= 4 && nchunks > 2) load_weights<2 % NS>(2);
    store_act<0>(0);
    __syncthreads();
    int c = 0;
    if (NS == 4) {
      for (; c + 3 < nchunks; c += 4) {
        step<0>(c, nchunks);
        step<1>(c + 1, nchunks);
        step<2 % NS>(c + 2, nchunks);
        step<3 % NS>(c + 3, nchunks);
      }
      if (c < nchunks) step<0>(c, nchunks);
      if (c + 1 < nchunks) step<1>(c + 1, nchunks);
      if (c + 2 < nchunks) step<2 % NS>(c + 2, nchunks);
    } else if (NS == 3) {
      for (; c + 2 < nchunks; c += 3) {
        step<0>(c, nchunks);
        step<1>(c + 1, nchunks);
        step<2 % NS>(c + 2, nchunks);
      }
      if (c < nchunks) step<0>(c, nchunks);
      if (c + 1 < nchunks) step<1>(c + 1, nchunks);
    } else {
      for (; c + 1 < nchunks; c += 2) {
        step<0>(c, nchunks);
        step<1>(c + 1, nchunks);
      }
      if (c < nchunks) step<0>(c, nchunks);
    }
  }
};

// One workgroup: expert `e`, output rows [n0, n0 + rows per WG), bucket rows
// [r0, min(r0 + 16*TB, row_end)).
template <int MODE, int NT, int TB, int RT, bool ONCE>
__device__ __forceinline__ void ffn_block(const FfnArgs& a, const uint16_t* W0, const uint16_t* W1,
                                          int n0, int r0, int row_end, int shared_base,
                                          unsigned char* lds) {
  constexpr int NA = MODE == kDownNarrow ? 1 : 2 * RT;
  Streamer<MODE, NT, TB, RT, ONCE> st(a);
  st.lds = lds;
  st.lane = threadIdx.x & (MOE_WAVE - 1);
  st.wave = threadIdx.x / MOE_WAVE;
  const int r = st.lane & 15, g = st.lane >> 4;
  int nrow[NA];  // first output row of each of this wave's weight tiles
  st.wstep = weight_kstep_stride(a.tiled);
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    if (MODE == kGateUp) {
      nrow[i] = n0 + (st.wave * RT + (i >> 1)) * 16;
      st.w[i] = ((i & 1) ? W1 : W0) + weight_lane_offset(a.tiled, nrow[i] / 16, a.K, st.lane);
    } else if (MODE == kDownNarrow) {
      nrow[i] = n0 + st.wave * 16;
      st.w[i] = W0 + weight_lane_offset(a.tiled, nrow[i] / 16, a.K, st.lane);
    } else if (MODE == kDownHalves) {
      st.half_chunks = a.K / kChunk / 2;
      nrow[i] = n0 + st.wave * 16;
      st.w[i] = W0 + weight_lane_offset(a.tiled, nrow[i] / 16, a.K, st.lane) +
                (size_t)i * st.half_chunks * kStepsPerChunk * st.wstep;
    } else {
      nrow[i] = n0 + (st.wave * NA + i) * 16;
      st.w[i] = W0 + weight_lane_offset(a.tiled, nrow[i] / 16, a.K, st.lane);
    }
  }
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int p = min(r0 + t * 16 + r, row_end - 1);  // clamp; extra columns are dropped
    int src;
    if (MODE == kGateUp) src = shared_base >= 0 ? p - shared_base : a.perm[p] / a.k;
    else src = p;
    st.act_off[t] = (size_t)src * a.K;
  }
  st.run();

  // D layout: lane holds rows 4*g .. 4*g+3 of the 16-row tile, column r
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int p = r0 + t * 16 + r;
    if (p >= row_end) continue;
    if (MODE == kGateUp) {
      uint16_t* h = static_cast<uint16_t*>(a.out);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        float hv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) hv[j] = silu_f(st.acc[2 * rt][t][j]) * st.acc[2 * rt + 1][t][j];
        uint2 pk;
        pk.x = pack_bf16x2(hv[0], hv[1]);
        pk.y = pack_bf16x2(hv[2], hv[3]);
        *reinterpret_cast<uint2*>(h + (size_t)p * a.N + nrow[2 * rt] + 4 * g) = pk;
      }
    } else if (MODE == kDownHalves) {
      float* y = static_cast<float*>(a.out);
      *reinterpret_cast<float4*>(y + (size_t)p * a.N + nrow[0] + 4 * g) =
          make_float4(st.acc[0][t][0] + st.acc[1][t][0], st.acc[0][t][1] + st.acc[1][t][1],
                      st.acc[0][t][2] + st.acc[1][t][2], st.acc[0][t][3] + st.acc[1][t][3]);
    } else {
      float* y = static_cast<float*>(a.out);
#pragma unroll
      for (int i = 0; i < NA; ++i)
        *reinterpret_cast<float4*>(y + (size_t)p * a.N + nrow[i] + 4 * g) =
            make_float4(st.acc[i][t][0], st.acc[i][t][1], st.acc[i][t][2], st.acc[i][t][3]);
    }
  }
}

// rows past the bucket's end are clamped on load and dropped on store, so a
// larger tile count than needed is only wasted arithmetic
template <int MODE, int TB, int RT, bool ONCE>
__device__ __forceinline__ void ffn_block_sized(int nt, const FfnArgs& a, const uint16_t* W0,
                                                const uint16_t* W1, int n0, int r0, int row_end,
                                                int shared_base, unsigned char* lds) {
  static_assert(TB == 4, "the variants below cover passes of up to four tiles");
  switch (nt) {
    case 1: ffn_block<MODE, 1, TB, RT, ONCE>(a, W0, W1, n0, r0, row_end, shared_base, lds); break;
    case 2: ffn_block<MODE, 2, TB, RT, ONCE>(a, W0, W1, n0, r0, row_end, shared_base, lds); break;
    case 3: ffn_block<MODE, 3, TB, RT, ONCE>(a, W0, W1, n0, r0, row_end, shared_base, lds); break;
    default: ffn_block<MODE, 4, TB, RT, ONCE>(a, W0, W1, n0, r0, row_end, shared_base, lds); break;
  }
}

template <int MODE, int TB, int RT>
__global__ __launch_bounds__(kThreads) void ffn_stream_kernel(FfnArgs a, ExpertTable tab,
                                                              GroupList groups) {
  constexpr int kTokBlock = 16 * TB;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * (MODE == kDownHalves ? 2 : 1) * buf_bytes(TB)];
  // Workgroups are handed out in grid order, and the ones that take longest
  // should go first: later passes over a bucket exist only for the fullest
  // buckets, and the shared experts (listed last) see every token.  So when a
  // launch has either, the grid is walked backwards in both of those dimensions
  // (fine-grained layer, 128 tokens: gate/up 80 -> 74 us; with equal experts and
  // a single pass the forward order measured 3 % faster and stays).
  const int e = groups.id[a.heavy_first ? gridDim.y - 1 - blockIdx.y : blockIdx.y];
  const int pass = a.heavy_first ? gridDim.z - 1 - blockIdx.z : blockIdx.z;
  int row_begin, row_end, shared_base = -1;
  if (e < a.E) {
    row_begin = a.offset[e];
    row_end = a.offset[e + 1];
  } else {
    row_begin = a.A + (e - a.E) * a.T;
    row_end = row_begin + a.T;
    shared_base = row_begin;
  }
  const int r0 = row_begin + pass * kTokBlock;
  if (r0 >= row_end) return;
  const int nt = (min(row_end - r0, kTokBlock) + 15) / 16;
  const uint16_t *W0, *W1;
  int n0;
  if (MODE == kGateUp) {
    W0 = static_cast<const uint16_t*>(tab.Wg[e]);
    W1 = static_cast<const uint16_t*>(tab.Wu[e]);
    n0 = blockIdx.x * (kWaves * 16 * RT);
  } else if (MODE == kDownHalves || MODE == kDownNarrow) {
    W0 = W1 = static_cast<const uint16_t*>(tab.Wd[e]);
    n0 = blockIdx.x * (kWaves * 16);
  } else {
    W0 = W1 = static_cast<const uint16_t*>(tab.Wd[e]);
    n0 = blockIdx.x * (kWaves * 32 * RT);
  }
  // whole bucket in this one pass: nobody else reads these weight rows
  if (pass == 0 && row_end - r0 <= kTokBlock)
    ffn_block_sized<MODE, TB, RT, true>(nt, a, W0, W1, n0, r0, row_end, shared_base, lds);
  else
    ffn_block_sized<MODE, TB, RT, false>(nt, a, W0, W1, n0, r0, row_end, shared_base, lds);
}

// ------------------------------------------------ prefill: tiled kernel ----
// Many rows per expert: the FFN is a grouped GEMM and the bound moves from the
// weight stream to the matrix cores and to the bytes that reach a compute unit
// per flop.  One workgroup (four waves as 2 x 2) owns 256 bucket rows x 128
// weight rows (64 gate + 64 up rows, or 128 down rows); a wave keeps 8 x 4 MFMA
// tiles of accumulators.  Both operands go global -> LDS with the
// direct-to-LDS form of the global load (no staging registers), three 64-wide
// k-stages of 48 KiB in a ring, two of them in flight while one multiplies.
//
// Fetch shape.  Measured on this chip, a wave-wide 16-byte load whose lanes
// cover 16 rows x 64 B runs at a third of the rate of one that covers 8 rows x
// 128 B (whole cache lines), even out of L2.  So one fetch instruction takes 8
// rows x 64 k, and a 16-row x 64-k operand block is two of them (2 KiB).  Where
// the rows and chunks of a block sit inside those 2 KiB is chosen for the LDS
// banks (see tile_fetch_row below).
//
// The waves take the token tiles alternately so that a partly filled 256-row
// block is still shared evenly; tiles past the bucket's end are fetched
// (clamped rows) but not multiplied.  Work items are dealt so that each XCD
// (own L2) gets a contiguous run of them.
constexpr int kTileRows = 256;                    // bucket rows per workgroup
constexpr int kTileK = 64;                        // contraction depth of a stage
constexpr int kDblFrag = 2 * kFragBytes;          // 16 rows x 64 k
constexpr int kTileStage = 24 * kDblFrag;         // 16 token + 8 weight blocks = 48 KiB
constexpr int kTileStages = 3;
constexpr int kTileLds = kTileStage * kTileStages;
constexpr int kFetchPerWave = 12;                 // 48 fetches per stage over 4 waves

// The list of 256-row blocks of the experts in a launch.  Every workgroup
// derives it on its own from the bucket offsets (at most 136 groups: cheaper
// than a launch of its own and a round trip through memory): per group its
// first row, its row count and the index of its first block.
struct TilePlan {
  int begin[MOE_MAX_GROUPS], rows[MOE_MAX_GROUPS], first[MOE_MAX_GROUPS + 1];
  int sizes;   // bit c set: some group's (last) block multiplies 4c+1 .. 4c+4 token tiles
};

template <int ROWS = 256>
__device__ __forceinline__ void tile_plan_build(TilePlan& pl, const FfnArgs& a, const GroupList& groups) {
  const int i = threadIdx.x;
  if (i < groups.n) {
    const int e = groups.id[i];
    int b, n;
    if (e < a.E) {
      b = a.offset[e];
      n = a.offset[e + 1] - b;
    } else {
      b = a.A + (e - a.E) * a.T;
      n = a.T;
    }
    pl.begin[i] = b;
    pl.rows[i] = n;
  }
  if (i == 0) pl.sizes = 0;
  __syncthreads();
  if (i < groups.n && pl.rows[i] > 0) {
    const int tiles = (min(pl.rows[i], ROWS) + 15) / 16;
    atomicOr(&pl.sizes, 1 << ((tiles - 1) / 4));
  }
  if (i <= groups.n) {
    int run = 0;
    for (int q = 0; q < i; ++q) run += (pl.rows[q] + ROWS - 1) / ROWS;
    pl.first[i] = run;
  }
  __syncthreads();
}

// Placement of a 16-row x 64-k operand block in LDS (2 KiB = two fetches).
// The direct-to-LDS load puts fetch lane l at base + 16 l, and a fetch should
// cover whole 128-byte lines, so lanes 8 j .. 8 j + 7 take the eight 16-byte
// chunks of one row: row slot j, chunk position i.  Which row sits in which
// slot and which chunk at which position is free, and decides the bank
// behaviour of the MFMA operand read, where lane (r, g) wants row r, chunk
// 4 s + g.  Measured on this chip, a ds_read_b128 runs at the full 256 B/clk
// only if (a) every four consecutive lanes read four different 16-byte slots
// of ONE aligned 64-byte bank group, and (b) the eight such quads of a
// 32-lane half cover the four bank groups evenly; rows of 128 bytes with an
// XOR swizzle, conflict-free by the usual bank arithmetic, break (a) and run at
// half rate.  So: rows 4 q + idx (idx = 0..3) of quad q go to fetch q / 2, row
// slots 2 idx + (q & 1) (same parity = same half of the 256-byte bank line),
// and chunk c sits at position 4 (c & 1) + ((c >> 1) ^ idx): the four rows of
// a quad land in one bank group, g = c & 1 selects which.
__device__ __forceinline__ int tile_fetch_row(int lane, int u) {
  const int j = lane >> 3;
  return 4 * (2 * u + (j & 1)) + (j >> 1);
}
__device__ __forceinline__ int tile_fetch_chunk(int lane) {
  const int j = lane >> 3, i = lane & 7;
  return 2 * ((i & 3) ^ (j >> 1)) + (i >> 2);
}
__device__ __forceinline__ int tile_read_offset(int r, int c) {
  const int q = r >> 2, idx = r & 3;
  return (q >> 1) * kFragBytes + (2 * idx + (q & 1)) * 128 + (4 * (c & 1) + (((c >> 1) ^ idx) & 3)) * 16;
}

// One work item of the tiled kernel: a 256-row block of an expert's bucket
// times one slab of its weight rows.
struct TileItem {
  int e, r0, row_end, slab;
  int single;    // 1: the expert's bucket is this one block (an int: padding bytes made every copy of the
                 // struct go through scratch memory, and the reload waited for every outstanding fetch)
};

template <int ROWS = 256>
__device__ __forceinline__ TileItem tile_item(const GroupList& groups, const TilePlan& pl, int item,
                                              int slabs) {
  const int blk = item / slabs;
  // the one group whose block range holds blk (groups without rows have an
  // empty range): every lane tests a group, a ballot names the hit
  const int lane = threadIdx.x & (MOE_WAVE - 1);
  int g = 0;
  for (int base = 0; base < groups.n; base += MOE_WAVE) {
    const int cand = min(base + lane, groups.n - 1);
    const bool hit = base + lane < groups.n && pl.first[cand] <= blk && blk < pl.first[cand + 1];
    const unsigned long long m = __builtin_amdgcn_ballot_w64(hit);
    if (m) {
      g = base + __ffsll(m) - 1;
      break;
    }
  }
  TileItem it;
  it.slab = item - blk * slabs;
  it.e = groups.id[g];
  it.r0 = pl.begin[g] + (blk - pl.first[g]) * ROWS;
  it.row_end = pl.begin[g] + pl.rows[g];
  it.single = pl.rows[g] <= ROWS;
  return it;
}

// Part `part` of `parts` of an item: the same weight slab over a share of the
// block's token tiles (see TileSplit).  Parts past the block's last tile are
// empty: r0 == row_end, nothing is stored and every load is clamped to the
// bucket's last row.
__device__ __forceinline__ TileItem tile_item_part(TileItem it, int rows_per_block, int part, int parts) {
  const int tiles = (min(it.row_end - it.r0, rows_per_block) + 15) / 16;
  const int per = (tiles + parts - 1) / parts;
  const int block_end = min(it.row_end, it.r0 + rows_per_block);
  it.r0 = min(it.r0 + part * per * 16, block_end);
  it.row_end = min(block_end, it.r0 + per * 16);
  it.single = 0;   // its weights are read by the other parts too
  return it;
}

// Blocks of a stage: 0..15 = token tiles, 16..23 = weight tiles (gate/up:
// 16..19 gate rows n0.., 20..23 the same rows of up).  Every block is two
// fetches (rows 0..7 and 8..15); wave w issues the fetches h = w + 4 q, so its
// fetches q < 8 are token rows and q >= 8 weight rows.
//
// First half of an item's set-up: what names the activation row behind each
// of this lane's eight token fetches (gate/up: a bucket position maps to its
// token through perm -- loads that are issued early and used late).
template <int MODE>
__device__ __forceinline__ void tile_rows(const FfnArgs& a, const TileItem& it, int lane, int wave,
                                          int (&ids)[8]) {
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int h = wave + 4 * q, blk = h >> 1, u = h & 1;
    const int p = min(it.r0 + blk * 16 + tile_fetch_row(lane, u), it.row_end - 1);
    // Unconditional, branch-free loads with no consumer nearby, so that they
    // stay in flight: a shared expert's rows (p >= A) read a valid entry that
    // is ignored later, and the division by k waits until the id is used.
    ids[q] = MODE == kGateUp ? a.perm[min(p, a.A - 1)] : 0;
  }
}

// Second half: the twelve source pointers of this lane (stage 0).
// (NQ = 12; the weights-in-registers form below asks for the token sources only, NQ = 8.)
// SAME_ROWS: the item covers the same row block as the one whose pointers are
// in `cur` (another slab of its weights): the token pointers are taken over,
// no look-up result is touched.
template <int MODE, int NQ, bool SAME_ROWS = false>
__device__ __forceinline__ void tile_sources(const FfnArgs& a, const ExpertTable& tab,
                                             const TileItem& it, const int (&ids)[8], int lane,
                                             int wave, const uint16_t* (&src)[NQ],
                                             const uint16_t* const* cur = nullptr) {
  const int e = it.e;
  const int n0 = it.slab * (MODE == kGateUp ? 64 : 128);
  const int chunk = tile_fetch_chunk(lane);
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int h = wave + 4 * q, blk = h >> 1, u = h & 1;
    const int rr = tile_fetch_row(lane, u);   // row inside the 16-row block
    if (q < 8 && SAME_ROWS) {
      src[q] = cur[q];
      continue;
    }
    if (q < 8) {
      const int p = min(it.r0 + blk * 16 + rr, it.row_end - 1);   // bucket position
      int row = p;                                                 // down: h is in bucket order
      if (MODE == kGateUp) row = e >= a.E ? p - (a.A + (e - a.E) * a.T) : ids[q] / a.k;
      src[q] = a.act + (size_t)row * a.K + chunk * 8;
      continue;
    }
    const int j = blk - 16;
    if (a.tiled) {
      // tiled weights: fetch u is the MFMA tile of k-step 2 st + u, one KiB in a row
      const uint16_t* W;
      int n16;
      if (MODE == kGateUp) {
        W = static_cast<const uint16_t*>(j < 4 ? tab.Wg[e] : tab.Wu[e]);
        n16 = n0 / 16 + (j & 3);
      } else {
        W = static_cast<const uint16_t*>(tab.Wd[e]);
        n16 = n0 / 16 + j;
      }
      src[q] = W + weight_lane_offset(true, n16, a.K, lane) + (size_t)u * 512;
    } else {
      const uint16_t* rowp;
      if (MODE == kGateUp) {
        const uint16_t* W = static_cast<const uint16_t*>(j < 4 ? tab.Wg[e] : tab.Wu[e]);
        rowp = W + (size_t)(n0 + (j & 3) * 16 + rr) * a.K;
      } else {
        rowp = static_cast<const uint16_t*>(tab.Wd[e]) + (size_t)(n0 + j * 16 + rr) * a.K;
      }
      src[q] = rowp + chunk * 8;
    }
  }
  // pin the pointers down here: otherwise their computation (with its waits
  // for table look-ups) sinks in between the fetches, and an in-order wait
  // there stalls on the fetches already issued
#pragma unroll
  for (int q = 0; q < NQ; ++q) asm volatile("" : "+v"(src[q]));
}

// Issue this wave's fetches of stage st into ring buffer st % 3: the first NTOK
// of its eight token fetches (token blocks 0 .. 2 NTOK - 1 of the sixteen) and
// its four weight fetches.  A source pointer advances 64 elements along its row
// per stage, or two KiB tiles for tiled weights.
template <int NTOK>
__device__ __forceinline__ void tile_fetch(const uint16_t* const (&src)[kFetchPerWave], int st,
                                           int w_adv, int wave, unsigned char* ring) {
  unsigned char* base = ring + (st % kTileStages) * kTileStage;
#pragma unroll
  for (int q = 0; q < kFetchPerWave; ++q) {
    if (q >= NTOK && q < 8) continue;
    // weights are read once: marked non-temporal, so that they do not push the
    // token rows (re-read by every slab of a block) out of L2
    if (q >= 8)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(src[q] + (size_t)st * w_adv),
          (__attribute__((address_space(3))) void*)(base + (wave + 4 * q) * kFragBytes), 16, 0, 2);
    else
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(src[q] + (size_t)st * kTileK),
          (__attribute__((address_space(3))) void*)(base + (wave + 4 * q) * kFragBytes), 16, 0, 0);
  }
}

// ---- general form: eight waves --------------------------------------------
// With one wave per SIMD a stage is a serial chain (wait, barrier, fetch issue,
// operand reads, matrix instructions) that nothing overlaps: measured on a
// Mixtral-shaped layer at 256 tokens (blocks of 65-128 rows) the chain took
// 0.75 us per stage whether or not the weights came from HBM, against the 0.64
// us the weight stream needs.  So the general form runs EIGHT waves, two per
// SIMD, as 4 (token tiles wm, wm + 4, ...) x 2 (halves of the weight rows): a
// wave multiplies a quarter of the block's token tiles, and one wave's operand
// reads overlap the other's matrix instructions.  Same ring, same operand
// placement, same order of accumulation along the contraction (same bits).
constexpr int kT8Waves = 8;
constexpr int kT8Threads = kT8Waves * MOE_WAVE;
constexpr int kT8Tok = 4;                 // token fetches per wave and stage, a full 256-row block
constexpr int kT8Fetch = kT8Tok + 2;      // plus two weight fetches

// Wave w issues the token fetches h = w + 8 q (q < 4) and the weight fetches
// h = 32 + w + 8 q' (q' < 2) of the 48 per stage; fetch h is rows 8 (h & 1) .. of
// block h / 2 and lands at stage base + h KiB.
template <int MODE>
__device__ __forceinline__ void tile8_rows(const FfnArgs& a, const TileItem& it, int lane, int wave,
                                           int (&ids)[kT8Tok]) {
#pragma unroll
  for (int q = 0; q < kT8Tok; ++q) {
    const int h = wave + kT8Waves * q, blk = h >> 1, u = h & 1;
    const int p = min(it.r0 + blk * 16 + tile_fetch_row(lane, u), it.row_end - 1);
    ids[q] = MODE == kGateUp ? a.perm[min(p, a.A - 1)] : 0;   // see tile_rows
  }
}

template <int MODE>
__device__ __forceinline__ void tile8_sources(const FfnArgs& a, const ExpertTable& tab,
                                              const TileItem& it, const int (&ids)[kT8Tok], int lane,
                                              int wave, const uint16_t* (&src)[kT8Fetch]) {
  const int e = it.e;
  const int n0 = it.slab * (MODE == kGateUp ? 64 : 128);
  const int chunk = tile_fetch_chunk(lane);
#pragma unroll
  for (int q = 0; q < kT8Fetch; ++q) {
    const int h = q < kT8Tok ? wave + kT8Waves * q : 32 + wave + kT8Waves * (q - kT8Tok);
    const int blk = h >> 1, u = h & 1;
    const int rr = tile_fetch_row(lane, u);   // row inside the 16-row block
    if (q < kT8Tok) {
      const int p = min(it.r0 + blk * 16 + rr, it.row_end - 1);   // bucket position
      int row = p;                                                 // down: h is in bucket order
      if (MODE == kGateUp) row = e >= a.E ? p - (a.A + (e - a.E) * a.T) : ids[q] / a.k;
      src[q] = a.act + (size_t)row * a.K + chunk * 8;
      continue;
    }
    const int j = blk - 16;
    if (a.tiled) {
      const uint16_t* W;
      int n16;
      if (MODE == kGateUp) {
        W = static_cast<const uint16_t*>(j < 4 ? tab.Wg[e] : tab.Wu[e]);
        n16 = n0 / 16 + (j & 3);
      } else {
        W = static_cast<const uint16_t*>(tab.Wd[e]);
        n16 = n0 / 16 + j;
      }
      src[q] = W + weight_lane_offset(true, n16, a.K, lane) + (size_t)u * 512;
    } else {
      const uint16_t* rowp;
      if (MODE == kGateUp) {
        const uint16_t* W = static_cast<const uint16_t*>(j < 4 ? tab.Wg[e] : tab.Wu[e]);
        rowp = W + (size_t)(n0 + (j & 3) * 16 + rr) * a.K;
      } else {
        rowp = static_cast<const uint16_t*>(tab.Wd[e]) + (size_t)(n0 + j * 16 + rr) * a.K;
      }
      src[q] = rowp + chunk * 8;
    }
  }
  // pinned down here, not between the fetches (see tile_sources)
#pragma unroll
  for (int q = 0; q < kT8Fetch; ++q) asm volatile("" : "+v"(src[q]));
}

// This wave's fetches of stage st into ring buffer st % 3: the first NTOK of its
// token fetches (token blocks 0 .. 4 NTOK - 1) and its two weight fetches.
template <int NTOK>
__device__ __forceinline__ void tile8_fetch(const uint16_t* const (&src)[kT8Fetch], int st, int w_adv,
                                            int wave, unsigned char* ring) {
  unsigned char* base = ring + (st % kTileStages) * kTileStage;
#pragma unroll
  for (int q = 0; q < kT8Fetch; ++q) {
    if (q >= NTOK && q < kT8Tok) continue;
    if (q >= kT8Tok)   // weights are read once: non-temporal (see tile_fetch)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(src[q] + (size_t)st * w_adv),
          (__attribute__((address_space(3))) void*)(base + (32 + wave + kT8Waves * (q - kT8Tok)) * kFragBytes),
          16, 0, 2);
    else
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(src[q] + (size_t)st * kTileK),
          (__attribute__((address_space(3))) void*)(base + (wave + kT8Waves * q) * kFragBytes), 16, 0, 0);
  }
}

// One item.  On entry the fetches of its stages 0 and 1 are in flight (issued
// by the previous item, or by the kernel's preamble); before its own epilogue
// it sets up the next item of this workgroup and issues that item's first two
// stages, so the stores of one item and the cold first fetches of the next
// overlap instead of adding up.
// NJ = token tiles per wave that are multiplied (the block's tiles dealt to the
// four wave rows, rounded up): a compile-time bound, so the accumulators stay
// in registers and a short block costs what it uses.
template <int MODE, int NJ>
__device__ __forceinline__ void ffn_tile_block(const FfnArgs& a, const ExpertTable& tab,
                                               const TileItem& it, bool has_next,
                                               const TileItem& nxt,
                                               const uint16_t* (&src)[kT8Fetch],
                                               unsigned char* ring) {
  const int r0 = it.r0, row_end = it.row_end;
  const int lane = threadIdx.x & (MOE_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);
  const int wm = wave & 3, wn = wave >> 2;
  const int n0 = it.slab * (MODE == kGateUp ? 64 : 128);
  const int w_adv = a.tiled ? 1024 : kTileK;
  // where lane (r, g) finds row r, chunk 4 s + g of a block, for k-step s = 0, 1
  int rd[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) rd[ks] = tile_read_offset(lane & 15, 4 * ks + (lane >> 4));
  // tiled weights arrive as whole MFMA tiles: k-step ks is the ks-th KiB of the block
  int rdw[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) rdw[ks] = a.tiled ? ks * kFragBytes + lane * 16 : rd[ks];

  f32x4 acc[4][NJ];   // this wave's token tiles are wm, wm + 4, ...
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  int next_ids[kT8Tok];
#pragma unroll
  for (int q = 0; q < kT8Tok; ++q) next_ids[q] = 0;

  const int ns = a.K / kTileK;
  for (int st = 0; st < ns; ++st) {
    // This wave's fetches of stage st have landed once at most the fetches of
    // the one younger stage already issued are still outstanding (loads complete
    // in order; NJ + 2 per wave and stage, six in the two stages an item
    // inherits, so "all but the newest NJ + 2" is exact or conservative).  A
    // bare barrier, not __syncthreads(): the fence that comes with the latter
    // makes the compiler wait for EVERY outstanding fetch, which would put the
    // whole ring one stage deep.  What the barrier has to order is covered by
    // hand: the vmcnt wait above it (this wave's direct-to-LDS fetches of stage
    // st have been written), and program order (a wave's LDS reads of stage
    // st-1 fed MFMAs it has already issued).
    if (st + 1 < ns) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(NJ + 2) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    // the next item's row look-ups: issued early, needed only after the last stage
    if (st == 1 && has_next) tile8_rows<MODE>(a, nxt, lane, wave, next_ids);
    if (st + 2 < ns) tile8_fetch<NJ>(src, st + 2, w_adv, wave, ring);   // into the buffer stage st-1 used
    const unsigned char* base = ring + (st % kTileStages) * kTileStage;
    bf16x8 wf[2][4], tf[2][NJ];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int blk;
        if (MODE == kGateUp) blk = 16 + (i >> 1) * 4 + wn * 2 + (i & 1);
        else blk = 16 + wn * 4 + i;
        wf[ks][i] = *reinterpret_cast<const bf16x8*>(base + blk * kDblFrag + rdw[ks]);
      }
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        tf[ks][j] = *reinterpret_cast<const bf16x8*>(base + (wm + 4 * j) * kDblFrag + rd[ks]);
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[ks][i], tf[ks][j], acc[i][j], 0, 0, 0);
    if constexpr (NJ >= 2) {
      // order for the scheduler: the first k-step's reads, then its MFMAs with the
      // second k-step's reads slipped in one per two MFMAs, then the rest
      __builtin_amdgcn_sched_group_barrier(0x100, 4 + NJ, 0);
#pragma unroll
      for (int q = 0; q < 4 + NJ; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 8 * NJ - 2 * (4 + NJ), 0);
    }
  }

  // D layout: lane holds rows 4*g .. 4*g+3 of the 16-row weight tile, column r = token
  auto epilogue = [&]() {
    const int r = lane & 15, g = lane >> 4;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int p = r0 + (wm + 4 * j) * 16 + r;
      if (p >= row_end) continue;
      if (MODE == kGateUp) {
        uint16_t* h = static_cast<uint16_t*>(a.out);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          float hv[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) hv[q] = silu_f(acc[i][j][q]) * acc[2 + i][j][q];
          uint2 pk;
          pk.x = pack_bf16x2(hv[0], hv[1]);
          pk.y = pack_bf16x2(hv[2], hv[3]);
          *reinterpret_cast<uint2*>(h + (size_t)p * a.N + n0 + (wn * 2 + i) * 16 + 4 * g) = pk;
        }
      } else {
        float* y = static_cast<float*>(a.out);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          *reinterpret_cast<float4*>(y + (size_t)p * a.N + n0 + (wn * 4 + i) * 16 + 4 * g) =
              make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
      }
    }
  };

  // The ring is free once every wave has read the last stage: start the next
  // item, then write this one's results while those fetches fly.  (The
  // epilogue is written out on both paths: behind the join of a conditional
  // the compiler would first wait for every outstanding fetch.)
  if (has_next) {
    const uint16_t* next_src[kT8Fetch];
    if (ns < 2) tile8_rows<MODE>(a, nxt, lane, wave, next_ids);
    tile8_sources<MODE>(a, tab, nxt, next_ids, lane, wave, next_src);
    asm volatile("s_barrier" ::: "memory");
    tile8_fetch<kT8Tok>(next_src, 0, w_adv, wave, ring);   // in full: the next item's size is not a constant here
    if (ns > 1) tile8_fetch<kT8Tok>(next_src, 1, w_adv, wave, ring);
    epilogue();
#pragma unroll
    for (int q = 0; q < kT8Fetch; ++q) src[q] = next_src[q];
  } else {
    epilogue();
  }
}

// Which work items a workgroup of XCD `xcd` walks: by default XCD x takes the
// x-th contiguous eighth of the list (block-major, slab fastest), so that the
// slabs sharing a block's activation rows sit behind one L2.  With a handful of
// experts that puts one whole expert on each XCD, and the XCD with the fullest
// bucket finishes last.  So when the launcher allows it (the activation matrix
// is small enough to live in every L2 anyway) and the experts' blocks differ in
// size class (TilePlan::sizes), the items are dealt round-robin instead (item i
// to XCD i mod 8) and every XCD gets an eighth of every expert.  With equal
// classes the contiguous order stays: it measured 6 % faster there.
struct TileOrder {
  int base, step, count;
  __device__ __forceinline__ int item(int n) const { return base + n * step; }
};
__device__ __forceinline__ TileOrder tile_order(int total, int xcd, bool interleave) {
  TileOrder o;
  if (interleave) {
    o.base = xcd;
    o.step = 8;
    o.count = (total - xcd + 7) / 8;
  } else {
    const int per_xcd = (total + 7) / 8;
    o.base = xcd * per_xcd;
    o.step = 1;
    o.count = max(0, min(per_xcd, total - o.base));
  }
  return o;
}

// The last round of a persistent loop.  A workgroup of an XCD walks items
// local, local + stride, ...: with `count` items per XCD the last round holds
// count mod stride of them, and costs a whole item's time however few they are
// (880 items of a prefill layer over 256 workgroups: the fourth round is 44 %
// full).  So the items of a partly filled last round are cut into 2 or 4 parts
// along the token tiles of their block (same weights, a share of the rows: the
// variants for short blocks run them), as many as keep the parts within one
// round.  Splitting never changes a sum: every output row is still one
// workgroup's fixed-order accumulation over the whole contraction.
struct TileSplit {
  int full;    // walk positions below this are whole items
  int parts;   // positions from `full` on are parts: item full + (n - full) / parts
  int count;   // walk positions in all
  __device__ __forceinline__ int item(int n) const { return n < full ? n : full + (n - full) / parts; }
  __device__ __forceinline__ int part(int n) const { return n < full ? -1 : (n - full) % parts; }
};
__device__ __forceinline__ TileSplit tile_split(int count, int stride, bool allow) {
  TileSplit sp;
  const int rem = count % stride;
  sp.full = count;
  sp.parts = 1;
  sp.count = count;
  if (allow && rem > 0 && count > stride) {
    // cost of the last round in item times: ceil(parts * rem / stride) / parts
    int best = 4, parts = 1;   // in quarters
    for (int f = 2; f <= 4; f *= 2) {
      const int c = ((f * rem + stride - 1) / stride) * (4 / f);
      if (c < best) {
        best = c;
        parts = f;
      }
    }
    if (parts > 1) {
      sp.full = count - rem;
      sp.parts = parts;
      sp.count = sp.full + parts * rem;
    }
  }
  return sp;
}

// Persistent workgroups, one per compute unit (the 144 KiB ring allows no
// more).  Work items = (row block, weight slab), slab fastest.  Workgroups are
// dealt to the 8 XCDs round-robin by their linear id, and every XCD has its
// own L2: each XCD gets one contiguous eighth of the items, and the
// workgroups behind one L2 walk that run side by side, so the slabs that share
// a row block's activations (and the row blocks that share a shared expert's
// weights) are in flight together.
template <int MODE>
__global__ __launch_bounds__(kT8Threads, 1) void ffn_tile_kernel(FfnArgs a, ExpertTable tab,
                                                                 GroupList groups) {
  extern __shared__ __attribute__((aligned(16))) unsigned char ring[];
  __shared__ TilePlan plan;
  tile_plan_build(plan, a, groups);
  const int slabs = a.N / (MODE == kGateUp ? 64 : 128);
  const int total = plan.first[groups.n] * slabs;
  const int xcd = blockIdx.x & 7, stride = gridDim.x >> 3;   // grid is a multiple of 8
  int local = blockIdx.x >> 3;
  // round-robin only if allowed and the experts' blocks differ in size class
  const TileOrder order = tile_order(total, xcd, a.interleave && (plan.sizes & (plan.sizes - 1)) != 0);
  if (local >= order.count) return;
  const int lane = threadIdx.x & (MOE_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);
  const int w_adv = a.tiled ? 1024 : kTileK;

  TileItem it = tile_item(groups, plan, order.item(local), slabs);
  const uint16_t* src[kT8Fetch];
  {
    int rows[kT8Tok];
    tile8_rows<MODE>(a, it, lane, wave, rows);
    tile8_sources<MODE>(a, tab, it, rows, lane, wave, src);
    tile8_fetch<kT8Tok>(src, 0, w_adv, wave, ring);
    if (a.K / kTileK > 1) tile8_fetch<kT8Tok>(src, 1, w_adv, wave, ring);
  }
  while (true) {
    const bool has_next = local + stride < order.count;
    TileItem nxt = it;
    if (has_next) nxt = tile_item(groups, plan, order.item(local + stride), slabs);
    const int tiles = (min(it.row_end - it.r0, kTileRows) + 15) / 16;
    if (tiles <= 4) ffn_tile_block<MODE, 1>(a, tab, it, has_next, nxt, src, ring);
    else if (tiles <= 8) ffn_tile_block<MODE, 2>(a, tab, it, has_next, nxt, src, ring);
    else if (tiles <= 12) ffn_tile_block<MODE, 3>(a, tab, it, has_next, nxt, src, ring);
    else ffn_tile_block<MODE, 4>(a, tab, it, has_next, nxt, src, ring);
    if (!has_next) break;
    it = nxt;
    local += stride;
  }
}


// ----------------------------------- tiled kernel, at most 64 tokens ----
constexpr int kSmallNJ = 2;   // token tiles per wave: blocks of at most 64 rows
constexpr int kSmallRows = 32 * kSmallNJ;

// Issue this wave's fetches of an item's stage st into ring buffer `slot`: the
// first NTOK of its eight token fetches (token blocks 0 .. 2 NTOK - 1 of the
// sixteen) and its four weight fetches.  A source pointer advances 64 elements
// along its row per stage, or two KiB tiles for tiled weights.
template <int NTOK>
__device__ __forceinline__ void tile_fetch_slot(const uint16_t* const (&src)[kFetchPerWave], int st,
                                           int slot, int w_adv, int wave, unsigned char* ring) {
  unsigned char* base = ring + slot * kTileStage;
#pragma unroll
  for (int q = 0; q < kFetchPerWave; ++q) {
    if (q >= NTOK && q < 8) continue;
    // weights are read once: marked non-temporal, so that they do not push the
    // token rows (re-read by every slab of a block) out of L2
    if (q >= 8)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(src[q] + (size_t)st * w_adv),
          (__attribute__((address_space(3))) void*)(base + (wave + 4 * q) * kFragBytes), 16, 0, 2);
    else
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(src[q] + (size_t)st * kTileK),
          (__attribute__((address_space(3))) void*)(base + (wave + 4 * q) * kFragBytes), 16, 0, 0);
  }
}

__device__ __forceinline__ int tile_slot_after(int slot, int n) { return (slot + n) % kTileStages; }

// Result stores a wave issues per item: every wave issues all of them, rows past
// the bucket's end are dropped by the buffer resource's range check, so the
// number is a constant of the variant and the hand-written waits can count them.
template <int MODE>
constexpr int small_stores() { return kSmallNJ * (MODE == kGateUp ? 2 : 4); }

// s_waitcnt vmcnt(n) for a wave-uniform run-time n (rounded down to an even
// number: waiting for more is always safe), then the bare barrier.
template <int C>
__device__ __forceinline__ void small_wait_even(int half) {
  if (half >= C) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * C) : "memory");
  else if constexpr (C > 0) small_wait_even<C - 1>(half);
}
__device__ __forceinline__ void small_wait_barrier(int n) { small_wait_even<24>(n >> 1); }

// One item.  On entry the fetches of its stages 0 and 1 are in flight (issued
// by the previous item, or by the kernel's preamble).  The ring does not drain
// between items: during its own last two stages an item issues the first two
// stages of the workgroup's next item into the buffers that fall free, exactly
// where a longer contraction would have put its stages ns and ns + 1; the next
// item starts at ring position `slot0` + ns.
// `older_stores` = result stores of the previous item that this wave issued
// behind the fetches of stages 0 and 1 (0 for a workgroup's first item).
template <int MODE>
__device__ __forceinline__ void ffn_small_block(const FfnArgs& a, const ExpertTable& tab,
                                               const TileItem& it, bool has_next,
                                               const TileItem& nxt,
                                               const uint16_t* (&src)[kFetchPerWave],
                                               unsigned char* ring, int older_stores, int slot0) {
  constexpr int NJ = kSmallNJ;
  const int r0 = it.r0, row_end = it.row_end;
  const int lane = threadIdx.x & (MOE_WAVE - 1), wave = threadIdx.x / MOE_WAVE;
  const int wm = wave & 1, wn = wave >> 1;
  const int n0 = it.slab * (MODE == kGateUp ? 64 : 128);
  const int w_adv = a.tiled ? 1024 : kTileK;
  // where lane (r, g) finds row r, chunk 4 s + g of a block, for k-step s = 0, 1
  int rd[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) rd[ks] = tile_read_offset(lane & 15, 4 * ks + (lane >> 4));
  // tiled weights arrive as whole MFMA tiles: k-step ks is the ks-th KiB of the block
  int rdw[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) rdw[ks] = a.tiled ? ks * kFragBytes + lane * 16 : rd[ks];

  f32x4 acc[4][NJ];   // this wave's token tiles are wm, wm + 2, ...
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  int next_ids[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) next_ids[q] = 0;

  // One stage's arithmetic on the ring buffer at byte offset `slot_bytes`.  The
  // operand reads are written as instructions, not as loads through a pointer:
  // seeing a read of the ring, the compiler protects it from the direct-to-LDS
  // fetches in flight with a wait for ALL of them wherever control flow has
  // merged (after the run-time wait selection, after the next item's set-up)
  // -- the ring's own discipline (wait, barrier, buffer freed a stage ago)
  // already orders them.  All reads are issued, one wait, then the MFMAs in the
  // same order as in the general kernel (same sums, same bits).
  const uint32_t ring_lds =
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)ring;
  uint32_t wofs[2], tofs[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    wofs[ks] = ring_lds + rdw[ks] + (16 + wn * (MODE == kGateUp ? 2 : 4)) * kDblFrag;
    tofs[ks] = ring_lds + rd[ks] + wm * kDblFrag;
  }
  auto multiply = [&](int slot_bytes) {
    bf16x8 wf[2][4], tf[2][NJ];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const uint32_t wa = wofs[ks] + slot_bytes, ta = tofs[ks] + slot_bytes;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        // gate/up: blocks 16 + (i >> 1) * 4 + wn * 2 + (i & 1); down: 16 + wn * 4 + i
        if (MODE == kGateUp)
          asm volatile("ds_read_b128 %0, %1 offset:%2"
                       : "=v"(wf[ks][i])
                       : "v"(wa), "n"(((i >> 1) * 4 + (i & 1)) * kDblFrag));
        else
          asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(wf[ks][i]) : "v"(wa), "n"(i * kDblFrag));
      }
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(tf[ks][j]) : "v"(ta), "n"(2 * j * kDblFrag));
    }
    static_assert(NJ == 2, "the wait below names every operand register");
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(wf[0][0]), "+v"(wf[0][1]), "+v"(wf[0][2]), "+v"(wf[0][3]), "+v"(wf[1][0]),
                   "+v"(wf[1][1]), "+v"(wf[1][2]), "+v"(wf[1][3]), "+v"(tf[0][0]), "+v"(tf[0][1]),
                   "+v"(tf[1][0]), "+v"(tf[1][1]));
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[ks][i], tf[ks][j], acc[i][j], 0, 0, 0);
  };

  // D layout: lane holds rows 4*g .. 4*g+3 of the 16-row weight tile, column r = token.
  // The stores go through a buffer resource that covers this block's rows of the
  // output and nothing else: a row past the bucket's end is out of its range and
  // the hardware drops the store, so every wave issues the same number of stores.
  const int block_rows = __builtin_amdgcn_readfirstlane(min(row_end - r0, kSmallRows));
  const size_t out_elt = MODE == kGateUp ? 2 : 4;
  const size_t block_base = (size_t)__builtin_amdgcn_readfirstlane(r0) * a.N * out_elt;
  const ActRsrc out_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      static_cast<unsigned char*>(a.out) + block_base, 0, (int)(block_rows * a.N * out_elt), 0x00020000);
  auto epilogue = [&]() {
    const int r = lane & 15, g = lane >> 4;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int row = (wm + 2 * j) * 16 + r;   // inside the block
      if (MODE == kGateUp) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          float hv[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) hv[q] = silu_f(acc[i][j][q]) * acc[2 + i][j][q];
          u32x2 pk;
          pk[0] = pack_bf16x2(hv[0], hv[1]);
          pk[1] = pack_bf16x2(hv[2], hv[3]);
          __builtin_amdgcn_raw_buffer_store_b64(
              pk, out_rsrc, (int)((row * a.N + n0 + (wn * 2 + i) * 16 + 4 * g) * out_elt), 0, 0);
        }
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          u32x4 v;
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] = __float_as_uint(acc[i][j][q]);
          __builtin_amdgcn_raw_buffer_store_b128(
              v, out_rsrc, (int)((row * a.N + n0 + (wn * 4 + i) * 16 + 4 * g) * out_elt), 0, 0);
        }
      }
    }
  };

  // Every stage starts with a wait and a barrier: this wave's fetches of stage
  // st have landed once at most the operations issued after them are still
  // outstanding (loads complete in order).  A bare barrier, not
  // __syncthreads(): the fence that comes with the latter makes the compiler
  // wait for EVERY outstanding fetch (the ones of the next stages too), which
  // would put the whole ring one stage deep.  What the barrier has to order is
  // covered by hand: the vmcnt wait above it (this wave's direct-to-LDS fetches
  // of stage st have been written), and program order (a wave's LDS reads of
  // stage st-1 fed MFMAs it has already issued).  What is younger than stage
  // st's fetches at its wait:
  //   stage 0:      stage 1 (NJ + 4 fetches per wave, like every stage here) and
  //                 the previous item's result stores -- loads and stores share the one
  //                 in-order counter, and a store is acknowledged long after a
  //                 load of the same age has landed, so they are counted, not
  //                 waited for;
  //   stage 1:      those stores and stage 2 (NJ + 4 fetches: only the token
  //                 blocks this item multiplies);
  //   last stage:   the next item's stage 0 (NJ + 4), if there is a next item;
  //   other stages: the following stage, NJ + 4 (the row look-ups or the stores
  //                 in between only make the wait conservative).
  const int ns = a.K / kTileK;
  const uint16_t* next_src[kFetchPerWave];
  const bool same_rows = has_next && nxt.e == it.e && nxt.r0 == it.r0;
  int slot = slot0;   // ring buffer of the stage at hand
  auto stage_base = [&]() {
    const int bytes = slot * kTileStage;
    slot = tile_slot_after(slot, 1);
    return bytes;
  };
  if (ns >= 4) {
    small_wait_barrier(NJ + 4 + older_stores);
    tile_fetch_slot<NJ>(src, 2, tile_slot_after(slot, 2), w_adv, wave, ring);
    multiply(stage_base());
    small_wait_barrier(NJ + 4 + older_stores);
    tile_fetch_slot<NJ>(src, 3, tile_slot_after(slot, 2), w_adv, wave, ring);
    multiply(stage_base());
    for (int st = 2; st < ns - 2; ++st) {
      asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(NJ + 4) : "memory");
      tile_fetch_slot<NJ>(src, st + 2, tile_slot_after(slot, 2), w_adv, wave, ring);   // into the buffer stage st-1 used
      multiply(stage_base());
    }
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(NJ + 4) : "memory");
    // (Both paths are written out to the end: behind the join of a conditional
    // the compiler would first wait for every outstanding fetch.)
    if (has_next) {
      // The next item's first two stages (every block of this kernel has the
      // same size class).  If it is another slab of the same row block, its pointers need
      // no look-up result: otherwise the first use of one makes the compiler
      // wait for everything outstanding (it cannot count past direct-to-LDS
      // fetches), stage ns - 1 included.
      // (Nor are the look-ups issued early for the other case: a load the
      // compiler has to assume pending on some path makes it wait for
      // everything outstanding at the first reuse of a register of theirs.)
      if (same_rows) {
        tile_sources<MODE, kFetchPerWave, true>(a, tab, nxt, next_ids, lane, wave, next_src, src);
      } else {
        tile_rows<MODE>(a, nxt, lane, wave, next_ids);
        tile_sources<MODE, kFetchPerWave>(a, tab, nxt, next_ids, lane, wave, next_src);
      }
      tile_fetch_slot<NJ>(next_src, 0, tile_slot_after(slot, 2), w_adv, wave, ring);
      multiply(stage_base());
      asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(NJ + 4) : "memory");
      tile_fetch_slot<NJ>(next_src, 1, tile_slot_after(slot, 2), w_adv, wave, ring);
      multiply(stage_base());
      epilogue();
#pragma unroll
      for (int q = 0; q < kFetchPerWave; ++q) src[q] = next_src[q];
    } else {
      multiply(stage_base());
      asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
      multiply(stage_base());
      epilogue();
    }
    return;
  }

  // Contractions of fewer than four stages: the simple hand-over (the next
  // item's first fetches are issued after the last stage).
  for (int st = 0; st < ns; ++st) {
    if (st + 1 >= ns) asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    else if (st == 0) small_wait_barrier(NJ + 4 + older_stores);
    else small_wait_barrier(NJ + 4 + older_stores);
    if (st + 2 < ns) tile_fetch_slot<NJ>(src, st + 2, tile_slot_after(slot, 2), w_adv, wave, ring);
    multiply(stage_base());
  }
  if (has_next) {
    tile_rows<MODE>(a, nxt, lane, wave, next_ids);
    tile_sources<MODE, kFetchPerWave>(a, tab, nxt, next_ids, lane, wave, next_src);
    asm volatile("s_barrier" ::: "memory");
    tile_fetch_slot<NJ>(next_src, 0, slot, w_adv, wave, ring);
    if (ns > 1) tile_fetch_slot<NJ>(next_src, 1, tile_slot_after(slot, 1), w_adv, wave, ring);
    epilogue();
#pragma unroll
    for (int q = 0; q < kFetchPerWave; ++q) src[q] = next_src[q];
  } else {
    epilogue();
  }
}

// Launches of at most 64 tokens: no bucket, a shared expert's included, holds
// more than 64 rows, so every block is the smallest variant (two token tiles
// per wave).  A kernel of its own, so that the longer live ranges of the
// continuous ring meet that variant's register budget and not the largest one's.
template <int MODE>
__global__ __launch_bounds__(kThreads, 1) void ffn_tile_small_kernel(FfnArgs a, ExpertTable tab,
                                                                     GroupList groups) {
  extern __shared__ __attribute__((aligned(16))) unsigned char ring[];
  __shared__ TilePlan plan;
  // blocks of at most 64 rows: a bucket that holds more (possible only when a
  // caller's top-k lists name an expert twice for one token) is split, never cut
  tile_plan_build<kSmallRows>(plan, a, groups);
  const int slabs = a.N / (MODE == kGateUp ? 64 : 128);
  const int total = plan.first[groups.n] * slabs;
  const int xcd = blockIdx.x & 7;   // grid is a multiple of 8
  int stride = gridDim.x >> 3;
  int local = blockIdx.x >> 3;
  const TileOrder order = tile_order(total, xcd, a.interleave && (plan.sizes & (plan.sizes - 1)) != 0);
  // The walk takes ceil(count / stride) rounds whatever the stride; with the
  // fewest workgroups that still finish in that many rounds every workgroup
  // gets the same number of items (one token, two active experts: 56 items per
  // XCD over 28 workgroups, two each, instead of 24 with two and 8 with one),
  // and none of them shares the memory system with workgroups that leave early.
  if (a.split_tail && order.count > 0) {
    const int rounds = (order.count + stride - 1) / stride;
    stride = (order.count + rounds - 1) / rounds;
  }
  if (local >= min(stride, order.count)) return;
  const int lane = threadIdx.x & (MOE_WAVE - 1), wave = threadIdx.x / MOE_WAVE;
  const int w_adv = a.tiled ? 1024 : kTileK;

  TileItem it = tile_item<kSmallRows>(groups, plan, order.item(local), slabs);
  const uint16_t* src[kFetchPerWave];
  {
    int rows[8];
    tile_rows<MODE>(a, it, lane, wave, rows);
    tile_sources<MODE, kFetchPerWave>(a, tab, it, rows, lane, wave, src);
    tile_fetch_slot<kSmallNJ>(src, 0, 0, w_adv, wave, ring);
    if (a.K / kTileK > 1) tile_fetch_slot<kSmallNJ>(src, 1, 1, w_adv, wave, ring);
  }
  int slot0 = 0;          // ring buffer of the current item's stage 0
  int older_stores = 0;   // result stores of the previous item, issued behind this item's first fetches
  while (true) {
    const bool has_next = local + stride < order.count;
    TileItem nxt = it;
    if (has_next) nxt = tile_item<kSmallRows>(groups, plan, order.item(local + stride), slabs);
    ffn_small_block<MODE>(a, tab, it, has_next, nxt, src, ring, older_stores, slot0);
    older_stores = small_stores<MODE>();
    if (!has_next) break;
    slot0 = tile_slot_after(slot0, a.K / kTileK);
    it = nxt;
    local += stride;
  }
}

// ------------------------------------- prefill: weights in registers ----
// A second form of the tiled kernel for well-filled blocks (many rows per
// expert).  Two measurements shape it.  A wavefront that is alone on its SIMD
// issues a 16x16x32 MFMA only every ~27 clocks; two wavefronts sharing a SIMD
// reach the pipe's 16.  And everything the form above multiplies goes through
// the direct-to-LDS path, 48 KiB per stage for 256 x 128 x 64 multiply-adds.
// Here a workgroup has EIGHT wavefronts, two per SIMD, and only the token rows
// go through LDS.  The waves split the WEIGHT rows of a slab twice as wide
// (gate/up: 16 gate + 16 up rows each, 128 columns of h per workgroup; down:
// 32 rows each, 256 columns of y) and fetch their own weight tiles straight
// into registers in MFMA operand layout, as the decode stream kernel does,
// kWideWeightSets - 1 stages ahead.  Every wave multiplies all token tiles of
// the 256-row block, read from a four-slot ring of 32 KiB stages: 64 KiB per
// stage for 256 x 256 x 64 multiply-adds.  Same group list and block list, same
// persistent loop with the next item's first token stages issued ahead of the
// epilogue, same order of accumulation along the contraction.
constexpr int kWideWaves = 8;
constexpr int kWideThreads = kWideWaves * MOE_WAVE;
constexpr int kWideTiles = 16;                     // token tiles of a block
constexpr int kWideRows = 16 * kWideTiles;
constexpr int kWideStage = kWideTiles * kDblFrag;  // 32 KiB
constexpr int kWideStages = 4;                     // token ring
constexpr int kWideWeightSets = 3;                 // weight stages in registers
constexpr int kWideLds = kWideStage * kWideStages;
constexpr int kWideFetch = 2 * kWideTiles / kWideWaves;   // token fetches per wave and stage
constexpr int kWideSlabGateUp = 16 * kWideWaves;   // columns of h per item
constexpr int kWideSlabDown = 32 * kWideWaves;     // columns of y per item
constexpr int kWideWLead = kWideWeightSets - 1, kWideTLead = kWideStages - 1;
constexpr int kWideTail = kWideWLead > kWideTLead ? kWideWLead : kWideTLead;   // stages that issue less
constexpr int kWideMinStages = 2 + kWideWeightSets + kWideTail;   // shorter contractions use the form above
static_assert(2 * kWideTiles % kWideWaves == 0, "token fetches must divide over the waves");

// Loads a stage issues when d stages remain (itself included), and the number
// of loads that are younger than the tokens of the stage with d remaining:
// those of the two stages before it.
constexpr int wide_issue_w(int d) { return d > kWideWLead ? 4 : 0; }
// (ntok = token fetches a stage of this item issues per wave: only the blocks it
// multiplies.  The stages an item inherits were fetched in full, which makes the
// first waits conservative, never short.)
constexpr int wide_issue_t(int d, int ntok) { return d > kWideTLead ? ntok : 0; }
constexpr int wide_wait(int d, int ntok) {
  return wide_issue_w(d + 2) + wide_issue_t(d + 2, ntok) + wide_issue_w(d + 1) + wide_issue_t(d + 1, ntok);
}

// The token fetches of this form go through a buffer resource (base = the
// activation matrix, one 32-bit byte offset per lane, the stage as a scalar
// offset) rather than through per-lane 64-bit addresses: the compiler counts a
// buffer instruction among the ordinary loads, so its own waits for the weight
// registers come out exact.  (Behind a direct-to-LDS load in the flat-address
// encoding it waits for every outstanding load instead.)
__device__ __forceinline__ ActRsrc wide_resource(const FfnArgs& a, long long act_rows) {
  // out-of-range reads return zero; the launcher keeps the matrix under 2 GiB
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.act), 0,
                                           (int)(act_rows * a.K * 2), 0x00020000);
}

// Wave w issues the fetches h = w + 8 q of a stage: rows 8 (h & 1) .. of token
// block h / 2.  First half of an item's set-up, as tile_rows above.
template <int MODE>
__device__ __forceinline__ void wide_rows(const FfnArgs& a, const TileItem& it, int lane, int wave,
                                          int (&ids)[kWideFetch]) {
#pragma unroll
  for (int q = 0; q < kWideFetch; ++q) {
    const int h = wave + kWideWaves * q, blk = h >> 1, u = h & 1;
    const int p = min(it.r0 + blk * 16 + tile_fetch_row(lane, u), it.row_end - 1);
    ids[q] = MODE == kGateUp ? a.perm[min(p, a.A - 1)] : 0;
  }
}

// Second half: byte offsets of this lane's token fetches of stage 0.
template <int MODE>
__device__ __forceinline__ void wide_offsets(const FfnArgs& a, const TileItem& it,
                                             const int (&ids)[kWideFetch], int lane, int wave,
                                             uint32_t (&off)[kWideFetch]) {
  const int e = it.e;
  const int chunk = tile_fetch_chunk(lane);
#pragma unroll
  for (int q = 0; q < kWideFetch; ++q) {
    const int h = wave + kWideWaves * q, blk = h >> 1, u = h & 1;
    const int p = min(it.r0 + blk * 16 + tile_fetch_row(lane, u), it.row_end - 1);
    int row = p;                                                 // down: h is in bucket order
    if (MODE == kGateUp) row = e >= a.E ? p - (a.A + (e - a.E) * a.T) : ids[q] / a.k;
    off[q] = ((uint32_t)row * a.K + chunk * 8) * 2;
  }
  // computed here, not between the fetches (see tile_sources)
#pragma unroll
  for (int q = 0; q < kWideFetch; ++q) asm volatile("" : "+v"(off[q]));
}

// Token fetches of stage st into ring slot st mod 4.
template <int NTOK = kWideFetch>
__device__ __forceinline__ void wide_fetch(ActRsrc rsrc, const uint32_t (&off)[kWideFetch], int st,
                                           int wave, unsigned char* ring) {
  unsigned char* base = ring + (st % kWideStages) * kWideStage;
#pragma unroll
  for (int q = 0; q < NTOK; ++q)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        rsrc,
        (__attribute__((address_space(3))) void*)(base + (wave + kWideWaves * q) * kFragBytes), 16,
        off[q], st * (kTileK * 2), 0, 0);
}

template <int V>
using Tag = std::integral_constant<int, V>;

// NT = token tiles multiplied (4, 8, 12 or 16): a compile-time bound.
// R = (K/64 - 2 - kWideTail) % kWideWeightSets.  ONCE: no other block reads these weight tiles.
// YB (down only): the rows of Y are rounded to bf16 on the way out (half the store bytes).
template <int MODE, int NT, int R, bool ONCE, bool YB>
__device__ __forceinline__ void ffn_wide_block(const FfnArgs& a, const ExpertTable& tab,
                                               const TileItem& it, bool has_next,
                                               const TileItem& nxt, ActRsrc rsrc,
                                               uint32_t (&src)[kWideFetch],
                                               unsigned char* ring) {
  const int r0 = it.r0, row_end = it.row_end;
  const int lane = threadIdx.x & (MOE_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);   // uniform: a scalar register
  const int n0 = it.slab * (MODE == kGateUp ? kWideSlabGateUp : kWideSlabDown);
  // this wave's two weight tiles: gate/up -> 16 rows of Wg and the same rows of
  // Wu; down -> 32 consecutive rows of Wd
  const uint16_t* w[2];
  int nrow[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const uint16_t* W;
    if (MODE == kGateUp) {
      W = static_cast<const uint16_t*>(i ? tab.Wu[it.e] : tab.Wg[it.e]);
      nrow[i] = n0 + wave * 16;
    } else {
      W = static_cast<const uint16_t*>(tab.Wd[it.e]);
      nrow[i] = n0 + wave * 32 + i * 16;
    }
    w[i] = W + weight_lane_offset(a.tiled, nrow[i] / 16, a.K, lane);
  }
  const int wstep = weight_kstep_stride(a.tiled);
  int rd[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) rd[ks] = tile_read_offset(lane & 15, 4 * ks + (lane >> 4));

  f32x4 acc[2][NT];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  int next_ids[kWideFetch];
#pragma unroll
  for (int q = 0; q < kWideFetch; ++q) next_ids[q] = 0;

  const int ns = a.K / kTileK;
  constexpr int WS = kWideWeightSets;
  bf16x8 wreg[WS][2][2];                           // [stage % WS][k-step][tile]
  auto load_w = [&](auto set_tag, int st) {
    constexpr int SET = decltype(set_tag)::value;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        // non-temporal when nobody reads the tile again (see Streamer::load_weight)
        const bf16x8* q = reinterpret_cast<const bf16x8*>(w[i] + (size_t)(2 * st + ks) * wstep);
        wreg[SET][ks][i] = ONCE ? __builtin_nontemporal_load(q) : *q;
      }
  };
  load_w(Tag<0>{}, 0);
  load_w(Tag<1>{}, 1);
  if constexpr (WS > 3) load_w(Tag<2 % WS>{}, 2);
  if constexpr (WS > 4) load_w(Tag<3 % WS>{}, 3);
  static_assert(WS >= 3 && WS <= 5, "the preamble loads above cover three to five register sets");

  // One stage.  Loads complete in order; a stage issues weights(st + WS - 1) and
  // tokens(st + 3).  tokens(st) were issued in stage st - 3 (or before the item
  // began, ahead of its first weight loads), and whatever the two stages since
  // then issued is younger: "at most that many outstanding" says tokens(st)
  // have landed.  The compiler adds its own exact waits for the weight
  // registers.  The last stages issue less (D = stages remaining decides), so
  // they wait for fewer.  All of this is fixed at compile time: a stage has no
  // branches, which keeps the compiler's load bookkeeping exact.
  auto stage = [&](int st, auto set_tag, auto remaining_tag, auto rows_tag) {
    constexpr int SET = decltype(set_tag)::value;
    constexpr int D = decltype(remaining_tag)::value;
    // token blocks this item multiplies: 2 NT fetches of the 32, NT / 4 per wave
    constexpr int NTOK = NT / 4;
    constexpr bool IW = wide_issue_w(D) > 0, IT = wide_issue_t(D, NTOK) > 0;
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(wide_wait(D, NTOK)) : "memory");
    if (decltype(rows_tag)::value && has_next) {
      // the lane index re-derived and made opaque here: the look-up addresses are
      // then worked out on the spot instead of ahead of the item (where they would
      // be spilled, and their reload would wait for every outstanding load)
      int lane_here;
      asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane_here));
      wide_rows<MODE>(a, nxt, lane_here, wave, next_ids);
    }
    if (IW) load_w(Tag<(SET + kWideWLead) % WS>{}, st + kWideWLead);
    if (IT) wide_fetch<NTOK>(rsrc, src, st + kWideTLead, wave, ring);
    const unsigned char* base = ring + (st % kWideStages) * kWideStage;
    bf16x8 tf[2][NT];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int j = 0; j < NT; ++j)
        tf[ks][j] = *reinterpret_cast<const bf16x8*>(base + j * kDblFrag + rd[ks]);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[SET][ks][i], tf[ks][j], acc[i][j], 0, 0, 0);
    // order for the scheduler: the loads, some LDS reads ahead, then one more
    // read per two MFMAs.  Four ahead measured best (prefill layer, us: 2 ahead
    // 421, 3: 411, 4: 409, 6: 414, 8: 420, 10: 427 -- each read in flight holds
    // four registers of a budget that is already full)
    constexpr int AHEAD = 4;
    if (IW || IT) __builtin_amdgcn_sched_group_barrier(0x020, (IW ? 4 : 0) + (IT ? NTOK : 0), 0);
    __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
#pragma unroll
    for (int q = 0; q < 2 * NT - AHEAD; ++q) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 2 * AHEAD, 0);
  };
  // ns = 2 + R + WS m + kWideTail stages (the launcher picks R): 0 and 1, R more
  // at full issue, m rounds of WS, then the kWideTail that issue less and less
  constexpr int FULL = kWideTail + 1;              // any "stages remaining" above the tail
  constexpr int S0 = (2 + R) % WS;                 // register set of the first looped stage
  stage(0, Tag<0>{}, Tag<FULL>{}, Tag<0>{});
  stage(1, Tag<1>{}, Tag<FULL>{}, Tag<1>{});
  if constexpr (R >= 1) stage(2, Tag<2 % WS>{}, Tag<FULL>{}, Tag<0>{});
  if constexpr (R >= 2) stage(3, Tag<3 % WS>{}, Tag<FULL>{}, Tag<0>{});
  if constexpr (R >= 3) stage(4, Tag<4 % WS>{}, Tag<FULL>{}, Tag<0>{});
  if constexpr (R >= 4) stage(5, Tag<5 % WS>{}, Tag<FULL>{}, Tag<0>{});
  int st = 2 + R;
  for (; st < ns - kWideTail; st += WS) {
    stage(st, Tag<S0>{}, Tag<FULL>{}, Tag<0>{});
    stage(st + 1, Tag<(S0 + 1) % WS>{}, Tag<FULL>{}, Tag<0>{});
    stage(st + 2, Tag<(S0 + 2) % WS>{}, Tag<FULL>{}, Tag<0>{});
    if constexpr (WS > 3) stage(st + 3, Tag<(S0 + 3) % WS>{}, Tag<FULL>{}, Tag<0>{});
    if constexpr (WS > 4) stage(st + 4, Tag<(S0 + 4) % WS>{}, Tag<FULL>{}, Tag<0>{});
  }
  if constexpr (kWideTail >= 4) stage(ns - 4, Tag<(S0 + kWideTail + WS - 4) % WS>{}, Tag<4>{}, Tag<0>{});
  stage(ns - 3, Tag<(S0 + kWideTail - 3) % WS>{}, Tag<3>{}, Tag<0>{});
  stage(ns - 2, Tag<(S0 + kWideTail - 2) % WS>{}, Tag<2>{}, Tag<0>{});
  stage(ns - 1, Tag<(S0 + kWideTail - 1) % WS>{}, Tag<1>{}, Tag<0>{});
  static_assert(kWideTail == 3 || kWideTail == 4, "tail stages are written out for three or four");

  // D layout: lane holds rows 4*g .. 4*g+3 of the 16-row weight tile, column r = token
  auto epilogue = [&]() {
    const int r = lane & 15, g = lane >> 4;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int p = r0 + j * 16 + r;
      if (p >= row_end) continue;
      if (MODE == kGateUp) {
        uint16_t* h = static_cast<uint16_t*>(a.out);
        float hv[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) hv[q] = silu_f(acc[0][j][q]) * acc[1][j][q];
        uint2 pk;
        pk.x = pack_bf16x2(hv[0], hv[1]);
        pk.y = pack_bf16x2(hv[2], hv[3]);
        *reinterpret_cast<uint2*>(h + (size_t)p * a.N + nrow[0] + 4 * g) = pk;
      } else if (YB) {
        uint16_t* y = static_cast<uint16_t*>(a.out);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          uint2 pk;
          pk.x = pack_bf16x2(acc[i][j][0], acc[i][j][1]);
          pk.y = pack_bf16x2(acc[i][j][2], acc[i][j][3]);
          *reinterpret_cast<uint2*>(y + (size_t)p * a.N + nrow[i] + 4 * g) = pk;
        }
      } else {
        float* y = static_cast<float*>(a.out);
#pragma unroll
        for (int i = 0; i < 2; ++i)
          *reinterpret_cast<float4*>(y + (size_t)p * a.N + nrow[i] + 4 * g) =
              make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
      }
    }
  };

  // The ring is free once every wave has read the last stage: start the next
  // item, then write this one's results while those fetches fly.
  if (has_next) {
    uint32_t next_src[kWideFetch];
    wide_offsets<MODE>(a, nxt, next_ids, lane, wave, next_src);
    asm volatile("s_barrier" ::: "memory");
#pragma unroll
    for (int q = 0; q < kWideTLead; ++q) wide_fetch(rsrc, next_src, q, wave, ring);
    epilogue();
#pragma unroll
    for (int q = 0; q < kWideFetch; ++q) src[q] = next_src[q];
  } else {
    epilogue();
  }
}

template <int MODE, int R, bool YB>
__global__ __launch_bounds__(kWideThreads, 1) void ffn_wide_kernel(FfnArgs a, ExpertTable tab,
                                                                   GroupList groups,
                                                                   long long act_rows) {
  extern __shared__ __attribute__((aligned(16))) unsigned char ring[];
  __shared__ TilePlan plan;
  tile_plan_build<kWideRows>(plan, a, groups);
  const int slabs = a.N / (MODE == kGateUp ? kWideSlabGateUp : kWideSlabDown);
  const int total = plan.first[groups.n] * slabs;
  const int xcd = blockIdx.x & 7, stride = gridDim.x >> 3;   // grid is a multiple of 8
  int local = blockIdx.x >> 3;
  const TileOrder order = tile_order(total, xcd, a.interleave && (plan.sizes & (plan.sizes - 1)) != 0);
  const TileSplit split = tile_split(order.count, stride, a.split_tail != 0);
  if (local >= split.count) return;
  const int lane = threadIdx.x & (MOE_WAVE - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / MOE_WAVE);   // uniform: a scalar register
  auto item_at = [&](int n) {
    TileItem t = tile_item<kWideRows>(groups, plan, order.item(split.item(n)), slabs);
    const int part = split.part(n);
    return part < 0 ? t : tile_item_part(t, kWideRows, part, split.parts);
  };

  TileItem it = item_at(local);
  const ActRsrc rsrc = wide_resource(a, act_rows);
  uint32_t src[kWideFetch];
  {
    int ids[kWideFetch];
    wide_rows<MODE>(a, it, lane, wave, ids);
    wide_offsets<MODE>(a, it, ids, lane, wave, src);
#pragma unroll
    for (int q = 0; q < kWideTLead; ++q) wide_fetch(rsrc, src, q, wave, ring);
  }
  while (true) {
    const bool has_next = local + stride < split.count;
    TileItem nxt = it;
    if (has_next) nxt = item_at(local + stride);
    const int tiles = (min(it.row_end - it.r0, kWideRows) + 15) / 16;
    // gate/up weights of an expert with a single block: non-temporal.  (For the
    // down projection the hint measured slower in this kernel.)
    bool done = false;
    if constexpr (MODE == kGateUp) {
      if (it.single) {
        if (tiles <= 4) ffn_wide_block<MODE, 4, R, true, YB>(a, tab, it, has_next, nxt, rsrc, src, ring);
        else if (tiles <= 8) ffn_wide_block<MODE, 8, R, true, YB>(a, tab, it, has_next, nxt, rsrc, src, ring);
        else if (tiles <= 12) ffn_wide_block<MODE, 12, R, true, YB>(a, tab, it, has_next, nxt, rsrc, src, ring);
        else ffn_wide_block<MODE, 16, R, true, YB>(a, tab, it, has_next, nxt, rsrc, src, ring);
        done = true;
      }
    }
    if (!done) {
      if (tiles <= 4) ffn_wide_block<MODE, 4, R, false, YB>(a, tab, it, has_next, nxt, rsrc, src, ring);
      else if (tiles <= 8) ffn_wide_block<MODE, 8, R, false, YB>(a, tab, it, has_next, nxt, rsrc, src, ring);
      else if (tiles <= 12) ffn_wide_block<MODE, 12, R, false, YB>(a, tab, it, has_next, nxt, rsrc, src, ring);
      else ffn_wide_block<MODE, 16, R, false, YB>(a, tab, it, has_next, nxt, rsrc, src, ring);
    }
    if (!has_next) break;
    it = nxt;
    local += stride;
  }
}

template <int MODE, bool YB, int R = 0>
struct WideKernels {
  static const void* get(int r) {
    if (r == R) return reinterpret_cast<const void*>(&ffn_wide_kernel<MODE, R, YB>);
    if constexpr (R + 1 < kWideWeightSets) return WideKernels<MODE, YB, R + 1>::get(r);
    return nullptr;
  }
};

// Upper bound on the number of row blocks a launch can need.
int max_row_blocks(const moe_shape& s, int block_rows) {
  return (s.T * s.k + s.S * s.T) / block_rows + s.E + s.S + 1;
}

// Round-robin dealing of the gate/up work items (see tile_order) is allowed when
// the token matrix is small enough to sit in every XCD's 4 MB L2 next to the
// weight stream; the kernel then uses it if the buckets are uneven.  (For the
// down projection, whose activations are the much larger h, it measured slower
// at every size.)  MOE_TUNE_INTERLEAVE=0|1 overrides (tuning builds only).
// MOE_TUNE_SPLIT=0 switches the cutting of last-round items off (tuning builds only).
int split_allowed() {
  static const char* env = tune_env("MOE_TUNE_SPLIT");
  return !(env && env[0] == '0');
}

int interleave_allowed(long long act_bytes) {
  static const char* env = tune_env("MOE_TUNE_INTERLEAVE");
  if (env && (env[0] == '0' || env[0] == '1')) return env[0] == '1';
  return act_bytes <= (4ll << 20);
}

// Within the tiled family: the weights-in-registers form once the blocks are
// well filled, if the output width is a multiple of its slab, the contraction
// is long enough for its fixed pipeline and the activation matrix fits a
// 32-bit buffer offset.  MOE_TUNE_WIDE=0|1 overrides the first
// condition (tuning builds only).
bool wide_form(const moe_shape& s, int phase) {
  const long long K = phase == 0 ? s.H : s.F;
  const long long act_rows = phase == 0 ? (long long)s.T : (long long)s.T * s.k + (long long)s.S * s.T;
  const int N = phase == 0 ? s.F : s.H;
  if (N % (phase == 0 ? kWideSlabGateUp : kWideSlabDown) != 0) return false;
  if (K / kTileK < kWideMinStages || act_rows * K * 2 >= (1ll << 31)) return false;
  static const char* env = tune_env("MOE_TUNE_WIDE");
  if (env && (env[0] == '0' || env[0] == '1')) return (env[1] ? env[phase] : env[0]) == '1';   // "10": gate/up only
  const double rows = (double)s.T * s.k / s.E;
  return rows >= 96.0 || (s.S > 0 && s.T > 256);
}

// Per-device launch state of the tiled kernels: the dynamic-LDS attribute has to
// be set once per kernel and device, and the persistent grids are sized by the
// device's compute units.
constexpr int kMaxDevices = 64;
struct TileDeviceState {
  std::once_flag once[2];      // per phase (the kernels are templates over it)
  hipError_t err[2] = {hipSuccess, hipSuccess};
  int n_cu = 0;
};
TileDeviceState g_tile_state[kMaxDevices];

template <int MODE>
hipError_t tile_attributes() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_tile_kernel<MODE>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kTileLds);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_tile_small_kernel<MODE>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kTileLds);
  if (e != hipSuccess) return e;
  for (int r = 0; r < kWideWeightSets; ++r) {
    e = hipFuncSetAttribute(WideKernels<MODE, false>::get(r), hipFuncAttributeMaxDynamicSharedMemorySize,
                            kWideLds);
    if (e != hipSuccess) return e;
    if (MODE != kDown) continue;
    e = hipFuncSetAttribute(WideKernels<kDown, true>::get(r), hipFuncAttributeMaxDynamicSharedMemorySize,
                            kWideLds);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

template <int MODE>
moe_status launch_tile(const moe_shape& s, const FfnArgs& args, const ExpertTable& tab,
                       const GroupList& groups, hipStream_t stream, bool wide, bool y_bf16 = false) {
  if (y_bf16 && !(wide && MODE == kDown))
    return fail(MOE_ERR_UNSUPPORTED, "bf16 rows of Y exist for the prefill form of the down projection only");
  int dev = 0;
  MOE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(MOE_ERR_UNSUPPORTED, "device index %d out of range", dev);
  TileDeviceState& ds = g_tile_state[dev];
  constexpr int ph = MODE == kGateUp ? 0 : 1;
  std::call_once(ds.once[ph], [&]() {
    ds.err[ph] = tile_attributes<MODE>();
    if (ds.err[ph] == hipSuccess && !ds.n_cu) {
      int n = 0;
      ds.err[ph] = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
      ds.n_cu = n;
    }
  });
  if (ds.err[ph] != hipSuccess)
    return fail(MOE_ERR_HIP, "tiled FFN kernel set-up: %s", hipGetErrorString(ds.err[ph]));
  int n_cu = ds.n_cu;
  if (!n_cu) MOE_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  const int slabs = wide ? (MODE == kGateUp ? s.F / kWideSlabGateUp : s.H / kWideSlabDown)
                         : (MODE == kGateUp ? s.F / 64 : s.H / 128);
  // one persistent workgroup per compute unit, never more than there can be items
  static const char* small_env = tune_env("MOE_TUNE_SMALL");   // 0: the general kernel for small launches too
  const bool small = s.T <= kSmallRows && !(small_env && small_env[0] == '0');
  const int block_rows = wide ? kWideRows : (small ? kSmallRows : kTileRows);
  const int grid = (std::min(slabs * max_row_blocks(s, block_rows), n_cu) + 7) / 8 * 8;
  if (wide) {
    // rows of the activation matrix: tokens for gate/up, bucket rows for down
    long long act_rows = MODE == kGateUp ? (long long)s.T : (long long)args.A + (long long)s.S * s.T;
    FfnArgs wargs = args;
    void* params[] = {&wargs, const_cast<ExpertTable*>(&tab), const_cast<GroupList*>(&groups), &act_rows};
    const int r = (args.K / kTileK - 2 - kWideTail) % kWideWeightSets;
    const void* kernel = y_bf16 ? WideKernels<kDown, true>::get(r) : WideKernels<MODE, false>::get(r);
    MOE_HIP(hipLaunchKernel(kernel, dim3(grid), dim3(kWideThreads), params, kWideLds, stream));
  } else {
    if (small)   // every bucket, a shared expert's too, has at most T rows
      hipLaunchKernelGGL((ffn_tile_small_kernel<MODE>), dim3(grid), dim3(kThreads), kTileLds, stream,
                         args, tab, groups);
    else
      hipLaunchKernelGGL((ffn_tile_kernel<MODE>), dim3(grid), dim3(kT8Threads), kTileLds, stream, args,
                         tab, groups);
  }
  MOE_HIP(hipGetLastError());
  return MOE_OK;
}

// ------------------------------------------------------- down, split-K ----
// Down projection for few rows per expert (decode): the four wavefronts of a
// workgroup share the same 32 weight rows and each walks a quarter of the
// contraction, so a Mixtral-shaped layer has 128 x E workgroups instead of
// 32 x E and the chip stays full even with two active experts.  No wave needs
// another wave's activations, so the B fragments go from global memory (h is a
// few MB and lives in L2) straight to registers: no LDS and no barrier in the
// loop.  The four partial accumulators meet in LDS once, summed in wave order.
template <int NT, bool ONCE, int NW>
struct SplitKStreamer {
  const uint16_t* w0;
  const uint16_t* w1;
  const uint16_t* b[NT];  // this lane's activation row (at its k-group) per tile
  int wstep;
  bf16x8 wreg[2][kStepsPerChunk][2];
  bf16x8 breg[2][NT][kStepsPerChunk];
  f32x4 acc0[NT], acc1[NT];

  __device__ __forceinline__ bf16x8 load_weight(const uint16_t* p) const {
    const bf16x8* q = reinterpret_cast<const bf16x8*>(p);
    return ONCE ? __builtin_nontemporal_load(q) : *q;   // see Streamer::load_weight
  }

  template <int SET>
  __device__ __forceinline__ void load(int c) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int s = 0; s < kStepsPerChunk; ++s)
        breg[SET][t][s] = *reinterpret_cast<const bf16x8*>(b[t] + (size_t)c * kChunk + s * kKStep);
#pragma unroll
    for (int s = 0; s < kStepsPerChunk; ++s) {
      wreg[SET][s][0] = load_weight(w0 + (size_t)(c * kStepsPerChunk + s) * wstep);
      if (NW == 2) wreg[SET][s][1] = load_weight(w1 + (size_t)(c * kStepsPerChunk + s) * wstep);
    }
  }

  template <int SET>
  __device__ __forceinline__ void multiply() {
#pragma unroll
    for (int s = 0; s < kStepsPerChunk; ++s)
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        acc0[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[SET][s][0], breg[SET][t][s], acc0[t], 0, 0, 0);
        if (NW == 2)
          acc1[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[SET][s][1], breg[SET][t][s], acc1[t], 0, 0, 0);
      }
  }

  __device__ __forceinline__ void run(int cb, int ce) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      acc0[t] = f32x4{0.f, 0.f, 0.f, 0.f};
      acc1[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    if (cb >= ce) return;
    load<0>(cb);
    int c = cb;
    for (; c + 1 < ce; c += 2) {
      load<1>(c + 1);
      multiply<0>();
      if (c + 2 < ce) load<0>(c + 2);
      multiply<1>();
    }
    if (c < ce) multiply<0>();
  }
};

constexpr int kSplitRows = 32;   // weight rows per workgroup (16 in the one-tile form)
constexpr int kSplitTok = 32;    // bucket rows per pass (NT <= 2)
constexpr int kSplitOneTileIds = 16;  // up to this many (token, slot) pairs: the one-tile form

template <int NT, bool ONCE, int NW, int NWV>
__device__ __forceinline__ void down_splitk_block(const FfnArgs& a, const uint16_t* Wd, int n0,
                                                  int r0, int row_end, float* red) {
  const int lane = threadIdx.x & (MOE_WAVE - 1), wave = threadIdx.x / MOE_WAVE;
  const int r = lane & 15, g = lane >> 4;
  SplitKStreamer<NT, ONCE, NW> st;
  st.wstep = weight_kstep_stride(a.tiled);
  st.w0 = Wd + weight_lane_offset(a.tiled, n0 / 16, a.K, lane);
  st.w1 = Wd + weight_lane_offset(a.tiled, n0 / 16 + (NW - 1), a.K, lane);
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int p = min(r0 + t * 16 + r, row_end - 1);
    st.b[t] = a.act + (size_t)p * a.K + g * 8;
  }
  const int nchunks = a.K / kChunk;
  const int per = (nchunks + NWV - 1) / NWV;
  st.run(min(wave * per, nchunks), min((wave + 1) * per, nchunks));

  // partial sums -> LDS [wave][t][tile][lane] (float4), then a fixed-order sum
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    reinterpret_cast<f32x4*>(red)[((wave * NT + t) * 2 + 0) * MOE_WAVE + lane] = st.acc0[t];
    if (NW == 2) reinterpret_cast<f32x4*>(red)[((wave * NT + t) * 2 + 1) * MOE_WAVE + lane] = st.acc1[t];
  }
  __syncthreads();
  float* y = static_cast<float*>(a.out);
  for (int q = wave; q < NT * 2; q += NWV) {  // q = t * 2 + tile
    const int t = q >> 1, tile = q & 1;
    if (tile >= NW) continue;
    f32x4 sum = reinterpret_cast<const f32x4*>(red)[((0 * NT + t) * 2 + tile) * MOE_WAVE + lane];
#pragma unroll
    for (int w = 1; w < NWV; ++w) {
      const f32x4 v = reinterpret_cast<const f32x4*>(red)[((w * NT + t) * 2 + tile) * MOE_WAVE + lane];
      sum[0] += v[0]; sum[1] += v[1]; sum[2] += v[2]; sum[3] += v[3];
    }
    const int p = r0 + t * 16 + r;
    if (p < row_end)
      *reinterpret_cast<float4*>(y + (size_t)p * a.N + n0 + tile * 16 + 4 * g) =
          make_float4(sum[0], sum[1], sum[2], sum[3]);
  }
}

// NW = weight tiles per wave: 2 (32 rows per workgroup), or 1 (16 rows) for the
// very smallest batches, where at most a handful of experts is active and twice
// the workgroups put twice the loads in flight.  A row's sum is the same four
// quarter sums in the same order either way.
// NWV = wavefronts per workgroup = parts of the contraction (4; with NW = 1 also
// 8 or 16).  What this kernel needs is loads in flight, and a launch has at most
// (active experts) x H / 16 workgroups: with one token two experts are active,
// 512 workgroups of four waves are eight waves per compute unit, each with two
// 4 KiB chunks of weights on the way, well short of what the memory system
// takes.  So the fewer (token, slot) pairs a launch has, the more parts the
// contraction is cut into (the launcher decides from T x k alone); the partial
// sums still meet in LDS in wave order.
template <int NW, int NWV>
__global__ __launch_bounds__(NWV * MOE_WAVE) void ffn_down_splitk_kernel(FfnArgs a, ExpertTable tab,
                                                                         GroupList groups) {
  static_assert(NWV == kWaves || NW == 1, "more than four parts only in the one-tile form");
  constexpr int kMaxNT = NWV == kWaves ? 2 : 1;   // pairs <= 4 with more parts: one token tile
  __shared__ __attribute__((aligned(16))) float red[NWV * kMaxNT * 2 * MOE_WAVE * 4];
  const int e = groups.id[blockIdx.y];
  int row_begin, row_end;
  if (e < a.E) {
    row_begin = a.offset[e];
    row_end = a.offset[e + 1];
  } else {
    row_begin = a.A + (e - a.E) * a.T;
    row_end = row_begin + a.T;
  }
  const int r0 = row_begin + blockIdx.z * kSplitTok;
  if (r0 >= row_end) return;
  const uint16_t* Wd = static_cast<const uint16_t*>(tab.Wd[e]);
  const int n0 = blockIdx.x * (16 * NW);
  const bool once = blockIdx.z == 0 && row_end - r0 <= kSplitTok;   // the bucket's only pass
  if (kMaxNT == 1 || row_end - r0 <= 16) {
    if (once) down_splitk_block<1, true, NW, NWV>(a, Wd, n0, r0, row_end, red);
    else down_splitk_block<1, false, NW, NWV>(a, Wd, n0, r0, row_end, red);
  } else {
    if (once) down_splitk_block<kMaxNT, true, NW, NWV>(a, Wd, n0, r0, row_end, red);
    else down_splitk_block<kMaxNT, false, NW, NWV>(a, Wd, n0, r0, row_end, red);
  }
}

// ---------------------------------------------------------------- float32 --
// One wavefront per (bucket row, output column): lanes stride over the
// contraction with float4 loads, float32 FMA, butterfly sum.
__device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, MOE_WAVE);
  return v;
}

struct F32Args {
  const float* act;
  const int32_t* perm;
  const int32_t* offset;
  float* out;
  int T, k, E, A, K, N;
};

template <int MODE>
__global__ __launch_bounds__(kThreads) void ffn_f32_kernel(F32Args a, ExpertTable tab,
                                                           GroupList groups) {
  const int e = groups.id[blockIdx.y];
  int row_begin, row_end, shared_base = -1;
  if (e < a.E) {
    row_begin = a.offset[e];
    row_end = a.offset[e + 1];
  } else {
    row_begin = a.A + (e - a.E) * a.T;
    row_end = row_begin + a.T;
    shared_base = row_begin;
  }
  const int lane = threadIdx.x & (MOE_WAVE - 1);
  const int wave = threadIdx.x / MOE_WAVE;
  const int n = blockIdx.x * kWaves + wave;  // output column
  if (n >= a.N) return;
  const float* W0 = static_cast<const float*>(MODE == kGateUp ? tab.Wg[e] : tab.Wd[e]) + (size_t)n * a.K;
  const float* W1 = MODE == kGateUp ? static_cast<const float*>(tab.Wu[e]) + (size_t)n * a.K : nullptr;
  for (int p = row_begin + blockIdx.z; p < row_end; p += gridDim.z) {
    int src;
    if (MODE == kGateUp) src = shared_base >= 0 ? p - shared_base : a.perm[p] / a.k;
    else src = p;
    const float* x = a.act + (size_t)src * a.K;
    float s0 = 0.f, s1 = 0.f;
    for (int kk = lane * 4; kk < a.K; kk += MOE_WAVE * 4) {
      const float4 xv = *reinterpret_cast<const float4*>(x + kk);
      const float4 wv = *reinterpret_cast<const float4*>(W0 + kk);
      s0 = fmaf(xv.x, wv.x, s0); s0 = fmaf(xv.y, wv.y, s0);
      s0 = fmaf(xv.z, wv.z, s0); s0 = fmaf(xv.w, wv.w, s0);
      if (MODE == kGateUp) {
        const float4 uv = *reinterpret_cast<const float4*>(W1 + kk);
        s1 = fmaf(xv.x, uv.x, s1); s1 = fmaf(xv.y, uv.y, s1);
        s1 = fmaf(xv.z, uv.z, s1); s1 = fmaf(xv.w, uv.w, s1);
      }
    }
    s0 = wave_sum_f(s0);
    if (MODE == kGateUp) {
      s1 = wave_sum_f(s1);
      if (lane == 0) a.out[(size_t)p * a.N + n] = s0 / (1.0f + expf(-s0)) * s1;
    } else {
      if (lane == 0) a.out[(size_t)p * a.N + n] = s0;
    }
  }
}

}  // namespace

// Which kernel serves a phase.  Gate/up and down choose separately:
//   kStream64   the stream kernel, 64-row passes, one weight tile per wave and matrix
//               (down: one tile per wave, 64 weight rows per workgroup -- with
//               128-row workgroups a fine-grained layer of some thirty active
//               experts has barely more workgroups than the chip has slots)
//   kTile       the tiled kernel (persistent, both operands through LDS)
//   kSplitK     down only: four waves split the contraction (32 rows per
//               workgroup, activations straight from L2): keeps the chip full
//               when very few experts are active
//   kHalves     down only: the stream kernel with the contraction halved
//               inside each wave (64 rows per workgroup)
// The tiled kernel is not only the many-rows form: its deep direct-to-LDS
// fetch ring streams long weight rows faster than the register-staged stream
// kernel does (5.6 against 5.3 TB/s on a Mixtral-shaped gate/up at 64 tokens),
// so it also takes the gate/up phase of wide experts at decode sizes (their
// many slabs balance over the persistent workgroups), and both phases from
// about 24 rows per expert on.
// MOE_TUNE_BLOCK=0|3 forces stream / tile for both phases,
// MOE_TUNE_GU=0|3 for gate/up only, MOE_TUNE_DOWN=lds|splitk|halves|tile
// for down only (tuning builds only, see tune_env).
enum Variant { kStream64 = 0, kTile = 3, kSplitK = 4, kHalves = 5 };

// The tiled kernel walks the contraction in steps of 64 and owns 64 / 128 rows.
bool tile_kernel_fits(const moe_shape& s) { return s.H % 128 == 0 && s.F % 64 == 0; }

static int forced_block() {
  static const char* env = tune_env("MOE_TUNE_BLOCK");
  return (env && (env[0] == '0' || env[0] == '3')) ? env[0] - '0' : -1;
}

static Variant rows_rule(const moe_shape& s) {
  const double rows = (double)s.T * s.k / s.E;   // expected rows per routed expert
  if (tile_kernel_fits(s) && (rows >= 24.0 || (s.S > 0 && s.T > 256))) return kTile;
  return kStream64;
}

Variant gate_up_variant(const moe_shape& s, int n_groups) {
  static const char* env = tune_env("MOE_TUNE_GU");
  if (env && (env[0] == '0' || env[0] == '3')) return (Variant)(env[0] - '0');
  if (forced_block() >= 0) return (Variant)forced_block();
  const Variant v = rows_rule(s);
  // shared experts see every token: from about a hundred tokens their buckets
  // (and the hot experts') would take the stream kernel two and more 64-row passes,
  // each streaming the expert's weights again, while a block of the tiled kernel
  // holds 256 rows (fine-grained layer with four shared experts, tiled against
  // stream, us: 96 tokens 74.4 / 72.2, 128: 76.3 / 78.5, 160: 85 / 103, 256: 100 / 130)
  if (v != kTile && tile_kernel_fits(s) && s.S > 0 && s.T > 96) return kTile;
  // wide experts: many slabs per expert, so the persistent workgroups get even
  // shares whatever number of experts turns out to be active.  Decided by the
  // layer's shape, not by how many experts this call lists: the streamed path
  // runs one expert per call and must land on the same kernel (same order of
  // every sum, same bits) as the all-resident call.
  (void)n_groups;
  if (v != kTile && tile_kernel_fits(s) && s.F / 64 >= 64 && (long)(s.E + s.S) * (s.F / 64) >= 2 * 256)
    return kTile;
  return v;
}

Variant down_variant(const moe_shape& s) {
  static const char* env = tune_env("MOE_TUNE_DOWN");
  const bool halves_ok = (s.F / kChunk) % 2 == 0;
  if (env && env[0] == 'l') return kStream64;
  if (env && env[0] == 's') return kSplitK;
  if (env && env[0] == 'h' && halves_ok) return kHalves;
  if (env && env[0] == 't' && tile_kernel_fits(s)) return kTile;
  if (forced_block() >= 0) return (Variant)forced_block();
  const Variant v = rows_rule(s);
  if (v != kStream64) return v;
  const double rows = (double)s.T * s.k / s.E;
  // wide outputs: the tiled kernel's ring streams the down projection faster
  // than the halved stream kernel and split-K as soon as its items -- (active
  // expert, 128 output columns) -- about fill the chip.  The experts a batch
  // activates are not known here; their expected number under uniform routing
  // stands in.  Mixtral shape, down phase in us, tiled against the rest: 10
  // tokens 125.8 / 126.0, 12: 128.6 / 132.6, 24: 138.5 / 144.1, 32: 138.9 /
  // 144.9, 48: 139.5 / 146.5, 65: 141.2 / 157.6, 80: 143.4 / 163.3; below (8
  // tokens, seven active experts) split-K wins, 122.2 against 125.5.
  const double active = s.E * (1.0 - pow(1.0 - 1.0 / s.E, (double)s.T * s.k)) + s.S;
  if (tile_kernel_fits(s) && s.H / 128 >= 32 && active * (s.H / 128) >= 240.0) return kTile;
  // split-K exists to fill the chip when few experts are active; with many
  // experts the halved stream kernel already has thousands of workgroups and
  // measured 9 % faster (128 experts of 2048 x 768, four rows each)
  const bool few_groups = (long)s.E * (s.H / 64) <= 1024;
  if (s.S == 0 || s.T <= 32) return ((rows <= 4.0 && few_groups) || !halves_ok) ? kSplitK : kHalves;
  return kStream64;
}

// Whether moe_layer_forward keeps the rows of Y in bf16 between the down
// projection and the combine: at the shapes whose down projection runs the
// prefill form.  There Y is the largest tensor the block writes and reads back
// (rows x H x 4 bytes: more than the activations and h together), an expert's
// output rounded to the storage dtype is what a module-by-module bf16 model
// produces anyway, and the stores are what the down kernel's items wait for.
// Decided by the shape alone, like the kernel choice.
bool layer_y_bf16(const moe_shape& s) {
  return s.dtype == MOE_BF16 && tile_kernel_fits(s) && down_variant(s) == kTile && wide_form(s, 1);
}

// Phase 1 (gate and up projections, SiLU gate) for the experts in `groups`.
moe_status launch_ffn_gate_up(const moe_shape& s, const void* X, const int32_t* perm,
                              const int32_t* offset, const ExpertTable& tab,
                              const GroupList& groups, const FfnScratch& scratch,
                              hipStream_t stream) {
  if (groups.n == 0 || s.T == 0) return MOE_OK;
  const int A = s.T * s.k;
  void* h = scratch.h;
  if (s.dtype == MOE_BF16) {
    FfnArgs gu{static_cast<const uint16_t*>(X), perm, offset, h, s.T, s.k, s.E, A, s.H, s.F,
               s.weight_layout == MOE_TILED, interleave_allowed((long long)s.T * s.H * 2), 0, split_allowed()};
    const Variant v = gate_up_variant(s, groups.n);
    if (v == kTile && tile_kernel_fits(s)) {
      return launch_tile<kGateUp>(s, gu, tab, groups, stream, wide_form(s, 0));
    } else {
      gu.heavy_first = s.S > 0 || s.T > 64;
      hipLaunchKernelGGL((ffn_stream_kernel<kGateUp, 4, 1>), dim3(s.F / (kWaves * 16), groups.n, (s.T + 63) / 64),
                         dim3(kThreads), 0, stream, gu, tab, groups);
    }
  } else {
    const int zb = s.T < 64 ? s.T : 64;
    F32Args gu{static_cast<const float*>(X), perm, offset, static_cast<float*>(h),
               s.T, s.k, s.E, A, s.H, s.F};
    hipLaunchKernelGGL((ffn_f32_kernel<kGateUp>), dim3((s.F + kWaves - 1) / kWaves, groups.n, zb),
                       dim3(kThreads), 0, stream, gu, tab, groups);
  }
  MOE_HIP(hipGetLastError());
  return MOE_OK;
}

// Phase 2 (down projection) for the experts in `groups`.
moe_status launch_ffn_down(const moe_shape& s, const FfnScratch& scratch, const int32_t* perm,
                           const int32_t* offset, const ExpertTable& tab, const GroupList& groups,
                           void* Y, hipStream_t stream, bool y_bf16) {
  if (groups.n == 0 || s.T == 0) return MOE_OK;
  if (y_bf16 && !layer_y_bf16(s))
    return fail(MOE_ERR_UNSUPPORTED, "bf16 rows of Y are not available for this shape");
  const int A = s.T * s.k;
  const void* h = scratch.h;
  if (s.dtype == MOE_BF16) {
    FfnArgs dn{static_cast<const uint16_t*>(h), perm, offset, Y, s.T, s.k, s.E, A, s.F, s.H,
               s.weight_layout == MOE_TILED, 0,    // h is too large to share between the XCDs' L2s
               s.S > 0 || s.T > 64, split_allowed()};
    const Variant v = down_variant(s);
    if (v == kTile && tile_kernel_fits(s)) {
      return launch_tile<kDown>(s, dn, tab, groups, stream, wide_form(s, 1), y_bf16);
    } else if (v == kHalves) {
      hipLaunchKernelGGL((ffn_stream_kernel<kDownHalves, 4, 1>), dim3(s.H / (kWaves * 16), groups.n, (s.T + 63) / 64),
                         dim3(kThreads), 0, stream, dn, tab, groups);
    } else if (v == kSplitK) {
      const int tok_blocks = (s.T + kSplitTok - 1) / kSplitTok;
      static const char* nw_env = tune_env("MOE_TUNE_SPLITNW");
      const long pairs = (long)s.T * s.k;
      const bool one_tile = nw_env ? nw_env[0] == '1' : pairs <= kSplitOneTileIds;
      // parts of the contraction (see the kernel): 16 up to two pairs, 8 up to four, else 4.
      // (Shared experts have T rows each, so they count as well.)
      static const char* wv_env = tune_env("MOE_TUNE_SPLITWAVES");
      int parts = (pairs <= 2 && s.T <= 2) ? 16 : (pairs <= 4 && s.T <= 4) ? 8 : 4;
      if (wv_env) parts = atoi(wv_env);
      if (one_tile && parts == 16 && pairs <= 16 && s.T <= 16)
        hipLaunchKernelGGL((ffn_down_splitk_kernel<1, 16>), dim3(s.H / 16, groups.n, tok_blocks),
                           dim3(16 * MOE_WAVE), 0, stream, dn, tab, groups);
      else if (one_tile && parts == 8 && pairs <= 16 && s.T <= 16)
        hipLaunchKernelGGL((ffn_down_splitk_kernel<1, 8>), dim3(s.H / 16, groups.n, tok_blocks),
                           dim3(8 * MOE_WAVE), 0, stream, dn, tab, groups);
      else if (one_tile)
        hipLaunchKernelGGL((ffn_down_splitk_kernel<1, kWaves>), dim3(s.H / 16, groups.n, tok_blocks),
                           dim3(kThreads), 0, stream, dn, tab, groups);
      else
        hipLaunchKernelGGL((ffn_down_splitk_kernel<2, kWaves>), dim3(s.H / kSplitRows, groups.n, tok_blocks),
                           dim3(kThreads), 0, stream, dn, tab, groups);
    } else {
      hipLaunchKernelGGL((ffn_stream_kernel<kDownNarrow, 4, 1>), dim3(s.H / (kWaves * 16), groups.n, (s.T + 63) / 64),
                         dim3(kThreads), 0, stream, dn, tab, groups);
    }
  } else {
    const int zb = s.T < 64 ? s.T : 64;
    F32Args dn{static_cast<const float*>(h), perm, offset, static_cast<float*>(Y), s.T, s.k, s.E, A, s.F, s.H};
    hipLaunchKernelGGL((ffn_f32_kernel<kDown>), dim3((s.H + kWaves - 1) / kWaves, groups.n, zb),
                       dim3(kThreads), 0, stream, dn, tab, groups);
  }
  MOE_HIP(hipGetLastError());
  return MOE_OK;
}

// Both phases.  `wait_gu` / `wait_d` (may be NULL) are events the stream waits
// on before the first and before the second phase: a streamed expert's first
// phase can start as soon as its gate and up projections have landed.  `mid`
// (may be NULL) is recorded between the phases.
moe_status launch_ffn_gated(const moe_shape& s, const void* X, const int32_t* perm,
                            const int32_t* offset, const ExpertTable& tab, const GroupList& groups,
                            void* Y, const FfnScratch& scratch, hipStream_t stream,
                            hipEvent_t wait_gu, hipEvent_t wait_d, hipEvent_t mid, bool y_bf16) {
  if (wait_gu) MOE_HIP(hipStreamWaitEvent(stream, wait_gu, 0));
  moe_status st = launch_ffn_gate_up(s, X, perm, offset, tab, groups, scratch, stream);
  if (st != MOE_OK) return st;
  if (mid) MOE_HIP(hipEventRecord(mid, stream));
  if (wait_d) MOE_HIP(hipStreamWaitEvent(stream, wait_d, 0));
  return launch_ffn_down(s, scratch, perm, offset, tab, groups, Y, stream, y_bf16);
}

moe_status launch_grouped_ffn(const moe_shape& s, const void* X, const int32_t* perm,
                              const int32_t* offset, const ExpertTable& tab,
                              const GroupList& groups, float* Y, const FfnScratch& scratch,
                              hipStream_t stream) {
  return launch_ffn_gated(s, X, perm, offset, tab, groups, Y, scratch, stream, nullptr, nullptr,
                          nullptr, false);
}

const char* ffn_kernel_name(const moe_shape& s, int phase, int n_groups) {
  if (s.dtype != MOE_BF16) return phase == 0 ? "ffn_f32_kernel<gate/up>" : "ffn_f32_kernel<down>";
  const Variant v = phase == 0 ? gate_up_variant(s, n_groups) : down_variant(s);
  switch (v) {
    case kTile:
      if (wide_form(s, phase)) return phase == 0 ? "ffn_wide_kernel<gate/up>" : "ffn_wide_kernel<down>";
      if (s.T <= 64) return phase == 0 ? "ffn_tile_small_kernel<gate/up>" : "ffn_tile_small_kernel<down>";
      return phase == 0 ? "ffn_tile_kernel<gate/up>" : "ffn_tile_kernel<down>";
    case kSplitK: return "ffn_down_splitk_kernel";
    case kHalves: return "ffn_stream_kernel<down, halved contraction>";
    default: return phase == 0 ? "ffn_stream_kernel<gate/up, 64 rows>" : "ffn_stream_kernel<down, 64 rows>";
  }
}

}  // namespace moe

extern "C" moe_status moe_grouped_ffn(const moe_shape* shape, const void* X, const int32_t* perm,
                                      const int32_t* offset, const moe_expert_ptrs* host_experts,
                                      const uint64_t* host_expert_mask, float* Y, void* workspace,
                                      void* stream) {
  moe_status st = moe::check_shape(shape, "moe_grouped_ffn");
  if (st != MOE_OK) return st;
  if (shape->T == 0) return MOE_OK;
  MOE_REQUIRE(X && perm && offset && host_experts && Y, "moe_grouped_ffn: NULL pointer argument");
  if (!workspace) return moe::fail(MOE_ERR_WORKSPACE, "moe_grouped_ffn: NULL workspace");
  moe::ExpertTable tab;
  moe::GroupList groups;
  groups.n = 0;
  const int n = shape->E + shape->S;
  for (int e = 0; e < n; ++e) {
    const bool on = !host_expert_mask || ((host_expert_mask[e >> 6] >> (e & 63)) & 1ull);
    tab.Wg[e] = host_experts[e].Wg;
    tab.Wu[e] = host_experts[e].Wu;
    tab.Wd[e] = host_experts[e].Wd;
    if (on) {
      MOE_REQUIRE(tab.Wg[e] && tab.Wu[e] && tab.Wd[e],
                  "moe_grouped_ffn: expert %d is in the mask but has a NULL matrix", e);
      groups.id[groups.n++] = (uint8_t)e;
    }
  }
  const moe::WorkspaceLayout L = moe::workspace_layout(*shape);
  const moe::FfnScratch scratch{static_cast<char*>(workspace) + L.h};
  return moe::launch_grouped_ffn(*shape, X, perm, offset, tab, groups, Y, scratch,
                                 static_cast<hipStream_t>(stream));
}

extern "C" int32_t moe_layer_y_dtype(const moe_shape* shape) {
  if (moe::check_shape(shape, "moe_layer_y_dtype") != MOE_OK) return -1;
  return moe::layer_y_bf16(*shape) ? MOE_BF16 : MOE_F32;
}

extern "C" const char* moe_ffn_kernel_name(const moe_shape* shape, int32_t phase, int32_t n_groups) {
  if (moe::check_shape(shape, "moe_ffn_kernel_name") != MOE_OK || phase < 0 || phase > 1) return "";
  return moe::ffn_kernel_name(*shape, phase, n_groups);
}
