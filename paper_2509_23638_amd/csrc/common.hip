// Shape validation, error strings, workspace carve-up.
#include "common.h"

#include <stdlib.h>
#include <string.h>

namespace moe {

static thread_local char g_err[512] = "";

moe_status fail(moe_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

#ifdef MOE_TUNING
const char* tune_env(const char* name) { return getenv(name); }
#endif

moe_status check_shape(const moe_shape* s, const char* who) {
  if (!s) return fail(MOE_ERR_INVALID_ARG, "%s: NULL shape", who);
  if (s->dtype != MOE_F32 && s->dtype != MOE_BF16)
    return fail(MOE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, s->dtype);
  if (s->weight_layout != MOE_ROW_MAJOR && s->weight_layout != MOE_TILED)
    return fail(MOE_ERR_INVALID_ARG, "%s: unknown weight layout %d", who, s->weight_layout);
  if (s->weight_layout == MOE_TILED && s->dtype != MOE_BF16)
    return fail(MOE_ERR_INVALID_ARG, "%s: the tiled weight layout exists for bf16 storage only", who);
  if (s->T < 0 || s->H <= 0 || s->F <= 0 || s->E <= 0 || s->k <= 0 || s->S < 0)
    return fail(MOE_ERR_INVALID_ARG, "%s: non-positive dimension (T=%d H=%d E=%d k=%d F=%d S=%d)",
                who, s->T, s->H, s->E, s->k, s->F, s->S);
  if (s->E > MOE_MAX_E || s->k > s->E || s->k > MOE_MAX_K || s->S > MOE_MAX_S)
    return fail(MOE_ERR_INVALID_ARG, "%s: need k <= E <= %d, k <= %d, S <= %d (E=%d k=%d S=%d)",
                who, MOE_MAX_E, MOE_MAX_K, MOE_MAX_S, s->E, s->k, s->S);
  const int mult = s->dtype == MOE_BF16 ? 128 : 8;
  if (s->H % mult || s->F % mult)
    return fail(MOE_ERR_INVALID_ARG, "%s: H and F must be multiples of %d for this dtype (H=%d F=%d)",
                who, mult, s->H, s->F);
  if ((int64_t)s->T * (s->k + s->S) >= (1 << 24))
    return fail(MOE_ERR_INVALID_ARG, "%s: T*(k+S) must stay below 2^24", who);
  return MOE_OK;
}

WorkspaceLayout workspace_layout(const moe_shape& s) {
  WorkspaceLayout L;
  const size_t A = (size_t)s.T * s.k, rows = A + (size_t)s.S * s.T;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
  L.topk_idx = take(A * 4);
  L.topk_w = take(A * 4);
  L.count = take((size_t)s.E * 4);
  L.offset = take((size_t)(s.E + 1) * 4);
  L.perm = take(A * 4);
  L.inv_perm = take(A * 4);
  L.logits = take((size_t)s.T * s.E * sizeof(double));
  L.h = take(rows * s.F * elem_size(s));
  L.y = take(rows * s.H * 4);
  L.total = o;
  return L;
}

}  // namespace moe

extern "C" const char* moe_version(void) {
#ifdef MOE_TUNING
  return "moe_hotpath 0.3 (gfx950, tuning build: MOE_TUNE_* overrides compiled in)";
#else
  return "moe_hotpath 0.3 (gfx950)";
#endif
}

extern "C" const char* moe_last_error(void) { return moe::g_err; }

extern "C" size_t moe_workspace_bytes(const moe_shape* shape) {
  if (moe::check_shape(shape, "moe_workspace_bytes") != MOE_OK) return 0;
  return moe::workspace_layout(*shape).total + 256;
}

extern "C" moe_status moe_workspace_views(const moe_shape* shape, void* workspace,
                                          int32_t** topk_idx, float** topk_w, int32_t** count,
                                          int32_t** offset, int32_t** perm, int32_t** inv_perm,
                                          void** Y) {
  moe_status st = moe::check_shape(shape, "moe_workspace_views");
  if (st != MOE_OK) return st;
  if (!workspace) return moe::fail(MOE_ERR_WORKSPACE, "moe_workspace_views: NULL workspace");
  const moe::WorkspaceLayout L = moe::workspace_layout(*shape);
  char* w = static_cast<char*>(workspace);
  if (topk_idx) *topk_idx = reinterpret_cast<int32_t*>(w + L.topk_idx);
  if (topk_w) *topk_w = reinterpret_cast<float*>(w + L.topk_w);
  if (count) *count = reinterpret_cast<int32_t*>(w + L.count);
  if (offset) *offset = reinterpret_cast<int32_t*>(w + L.offset);
  if (perm) *perm = reinterpret_cast<int32_t*>(w + L.perm);
  if (inv_perm) *inv_perm = reinterpret_cast<int32_t*>(w + L.inv_perm);
  if (Y) *Y = w + L.y;
  return MOE_OK;
}
