// Internal helpers shared by the library's translation units (not part of the
// public boundary).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <stdarg.h>
#include <stdio.h>

#include "../../include/moe_hotpath.h"

#define MOE_MAX_E 128
#define MOE_MAX_K 16
#define MOE_MAX_S 8
#define MOE_MAX_GROUPS (MOE_MAX_E + MOE_MAX_S)
#define MOE_WAVE 64

namespace moe {

moe_status fail(moe_status st, const char* fmt, ...);
moe_status check_shape(const moe_shape* s, const char* who);

#define MOE_HIP(expr)                                                          \
  do {                                                                         \
    hipError_t _e = (expr);                                                    \
    if (_e != hipSuccess)                                                      \
      return moe::fail(MOE_ERR_HIP, "%s: %s (%s:%d)", #expr,                  \
                       hipGetErrorString(_e), __FILE__, __LINE__);             \
  } while (0)

#define MOE_REQUIRE(cond, ...)                                                 \
  do {                                                                         \
    if (!(cond)) return moe::fail(MOE_ERR_INVALID_ARG, __VA_ARGS__);           \
  } while (0)

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Kernel-selection overrides for measurement sweeps (environment variables
// MOE_TUNE_*).  They exist only in a library compiled with -DMOE_TUNING
// (build.py: MOE_BUILD_TUNING=1); the product build ignores the environment,
// so a stray variable can never change which kernels run or the order of a sum.
#ifdef MOE_TUNING
const char* tune_env(const char* name);
#else
static inline const char* tune_env(const char*) { return nullptr; }
#endif

// Workspace carve-up (all offsets 256-byte aligned).
struct WorkspaceLayout {
  size_t topk_idx, topk_w, count, offset, perm, inv_perm, logits, h, y, total;
};
WorkspaceLayout workspace_layout(const moe_shape& s);

static inline int rows_total(const moe_shape& s) { return s.T * s.k + s.S * s.T; }
static inline size_t elem_size(const moe_shape& s) { return s.dtype == MOE_F32 ? 4 : 2; }

// Expert pointer table handed to kernels by value (kernel argument segment).
struct ExpertTable {
  const void* Wg[MOE_MAX_GROUPS];
  const void* Wu[MOE_MAX_GROUPS];
  const void* Wd[MOE_MAX_GROUPS];
};

// Per-launch list of experts to run (indices into ExpertTable), by value.
struct GroupList {
  int32_t n;
  uint8_t id[MOE_MAX_GROUPS];
};

// Scratch of the grouped FFN inside a workspace: the intermediate h.
struct FfnScratch {
  void* h;
};

// internal launchers (each enqueues on `stream`, returns a status)
moe_status launch_route(const moe_shape& s, const void* X, const void* Wr, const float* bias,
                        int32_t* topk_idx, float* topk_w, double* logits_out, hipStream_t stream);
moe_status launch_route_bucket(const moe_shape& s, const void* X, const void* Wr, const float* bias,
                               int32_t* topk_idx, float* topk_w, double* logits, int32_t* count,
                               int32_t* offset, int32_t* perm, int32_t* inv_perm, hipStream_t stream,
                               bool* bucketed);
moe_status launch_permute(const moe_shape& s, const int32_t* topk_idx, int32_t* count,
                          int32_t* offset, int32_t* perm, int32_t* inv_perm, hipStream_t stream);
moe_status launch_grouped_ffn(const moe_shape& s, const void* X, const int32_t* perm,
                              const int32_t* offset, const ExpertTable& tab, const GroupList& groups,
                              float* Y, const FfnScratch& scratch, hipStream_t stream);
moe_status launch_ffn_gate_up(const moe_shape& s, const void* X, const int32_t* perm,
                              const int32_t* offset, const ExpertTable& tab,
                              const GroupList& groups, const FfnScratch& scratch, hipStream_t stream);
// y_bf16: the rows of Y are bf16 instead of float32 (only where layer_y_bf16()
// says so; the separate entry points always exchange float32 rows).
bool layer_y_bf16(const moe_shape& s);
moe_status launch_ffn_down(const moe_shape& s, const FfnScratch& scratch, const int32_t* perm,
                           const int32_t* offset, const ExpertTable& tab, const GroupList& groups,
                           void* Y, hipStream_t stream, bool y_bf16);
moe_status launch_ffn_gated(const moe_shape& s, const void* X, const int32_t* perm,
                            const int32_t* offset, const ExpertTable& tab, const GroupList& groups,
                            void* Y, const FfnScratch& scratch, hipStream_t stream,
                            hipEvent_t wait_gu, hipEvent_t wait_d, hipEvent_t mid, bool y_bf16);
moe_status launch_combine(const moe_shape& s, const void* Y, const float* topk_w,
                          const int32_t* inv_perm, const void* residual, void* out,
                          hipStream_t stream, bool y_bf16);

// ---- device helpers -------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}

// round to nearest even; inputs are finite in this library's use
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Two float32 values to packed bfloat16 (lo in bits 0..15), round to nearest
// even: one v_cvt_pk_bf16_f32.  Bit-identical to f32_to_bf16_bits for every
// finite input (checked exhaustively over the high halves with the tie and
// near-tie low halves).
typedef __bf16 bf16x2_hw __attribute__((ext_vector_type(2)));
typedef float f32x2_hw __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_hw v = {lo, hi};
  const bf16x2_hw b = __builtin_convertvector(v, bf16x2_hw);
  return __builtin_bit_cast(uint32_t, b);
}

}  // namespace moe
