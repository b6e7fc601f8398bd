// Scheduling side of the hot path: the token counter and hot-expert table of
// Section 4.1, a gate-based predictor (Section 3.2), and the PreSched decision
// of Section 4.3 (Eq. 2-6).  The decisions are host arithmetic over at most a
// few hundred entries; only the counter and the predictor's routing touch the
// GPU.
#include "common.h"
#include "../../include/moe_sched.h"

#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

namespace moe {
namespace {

__global__ void counter_add_kernel(const int32_t* __restrict__ count, int64_t* __restrict__ total,
                                   int E) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e < E) total[e] += count[e];
}

__global__ void zero_counts_kernel(int32_t* __restrict__ count, int E) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e < E) count[e] = 0;
}

// prefix[i] = sum of t_c over the first i entries (Eq. 2 per entry)
std::vector<double> cpu_cost_prefix(const std::vector<int32_t>& tokens, double beta, double C) {
  std::vector<double> pre(tokens.size() + 1, 0.0);
  for (size_t i = 0; i < tokens.size(); ++i) pre[i + 1] = pre[i] + (beta * tokens[i] + C);
  return pre;
}

struct Entry {
  int32_t layer, expert, tokens;
};

}  // namespace
}  // namespace moe

extern "C" moe_status moe_counter_add(const moe_shape* shape, const int32_t* count, int64_t* total,
                                      void* stream) {
  moe_status st = moe::check_shape(shape, "moe_counter_add");
  if (st != MOE_OK) return st;
  MOE_REQUIRE(count && total, "moe_counter_add: NULL pointer argument");
  hipLaunchKernelGGL(moe::counter_add_kernel, dim3(1), dim3(MOE_MAX_E), 0,
                     static_cast<hipStream_t>(stream), count, total, shape->E);
  MOE_HIP(hipGetLastError());
  return MOE_OK;
}

extern "C" moe_status moe_hot_table(const int64_t* host_tokens, int32_t L, int32_t E,
                                    int64_t budget_experts, uint8_t* host_resident) {
  MOE_REQUIRE(host_tokens && host_resident, "moe_hot_table: NULL pointer argument");
  MOE_REQUIRE(L >= 1 && E >= 1, "moe_hot_table: L=%d, E=%d must be positive", L, E);
  const int64_t n = (int64_t)L * E;
  std::vector<int64_t> order(n);
  std::iota(order.begin(), order.end(), (int64_t)0);
  // flat index = layer * E + expert, so index order is (layer, expert) order
  std::stable_sort(order.begin(), order.end(),
                   [&](int64_t a, int64_t b) { return host_tokens[a] > host_tokens[b]; });
  std::fill(host_resident, host_resident + n, (uint8_t)0);
  const int64_t take = std::min<int64_t>(std::max<int64_t>(budget_experts, 0), n);
  for (int64_t r = 0; r < take; ++r) host_resident[order[r]] = 1;
  return MOE_OK;
}

extern "C" moe_status moe_predict_counts(const moe_shape* shape, const void* X, const void* Wr_next,
                                         const float* bias_next, int32_t* pred_count,
                                         void* workspace, void* stream) {
  moe_status st = moe::check_shape(shape, "moe_predict_counts");
  if (st != MOE_OK) return st;
  MOE_REQUIRE(pred_count, "moe_predict_counts: NULL pred_count");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (shape->T == 0) {
    hipLaunchKernelGGL(moe::zero_counts_kernel, dim3(1), dim3(MOE_MAX_E), 0, s, pred_count, shape->E);
    MOE_HIP(hipGetLastError());
    return MOE_OK;
  }
  MOE_REQUIRE(X && Wr_next, "moe_predict_counts: NULL pointer argument");
  if (!workspace) return moe::fail(MOE_ERR_WORKSPACE, "moe_predict_counts: NULL workspace");
  const moe::WorkspaceLayout w = moe::workspace_layout(*shape);
  char* base = static_cast<char*>(workspace);
  int32_t* idx = reinterpret_cast<int32_t*>(base + w.topk_idx);
  float* wts = reinterpret_cast<float*>(base + w.topk_w);
  int32_t* count = reinterpret_cast<int32_t*>(base + w.count);
  bool bucketed = false;
  st = moe::launch_route_bucket(*shape, X, Wr_next, bias_next, idx, wts,
                                reinterpret_cast<double*>(base + w.logits), count,
                                reinterpret_cast<int32_t*>(base + w.offset),
                                reinterpret_cast<int32_t*>(base + w.perm),
                                reinterpret_cast<int32_t*>(base + w.inv_perm), s, &bucketed);
  if (st != MOE_OK) return st;
  if (!bucketed)
    st = moe::launch_permute(*shape, idx, count, reinterpret_cast<int32_t*>(base + w.offset),
                             reinterpret_cast<int32_t*>(base + w.perm),
                             reinterpret_cast<int32_t*>(base + w.inv_perm), s);
  if (st != MOE_OK) return st;
  MOE_HIP(hipMemcpyAsync(pred_count, count, shape->E * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
  return MOE_OK;
}

extern "C" moe_status moe_pending_experts(const int32_t* host_count, int32_t E,
                                          const uint64_t* host_resident_mask,
                                          const uint64_t* host_in_flight_mask,
                                          moe_pending* host_pending, int32_t* n_pending) {
  MOE_REQUIRE(host_count && host_pending && n_pending, "moe_pending_experts: NULL pointer argument");
  MOE_REQUIRE(E >= 1 && E <= MOE_SCHED_MAX_EXPERTS, "moe_pending_experts: E=%d outside [1, %d]", E,
              MOE_SCHED_MAX_EXPERTS);
  int n = 0;
  for (int e = 0; e < E; ++e) {
    MOE_REQUIRE(host_count[e] >= 0, "moe_pending_experts: negative count for expert %d", e);
    const bool resident = host_resident_mask && ((host_resident_mask[e >> 6] >> (e & 63)) & 1ull);
    const bool in_flight = host_in_flight_mask && ((host_in_flight_mask[e >> 6] >> (e & 63)) & 1ull);
    if (host_count[e] > 0 && !resident && !in_flight) host_pending[n++] = {e, host_count[e]};
  }
  *n_pending = n;
  return MOE_OK;
}

extern "C" moe_status moe_prefetch_hottest(const moe_pending* host_pending, int32_t n_pending,
                                           int32_t n_prefetch, int32_t* host_chosen,
                                           int32_t* n_chosen) {
  MOE_REQUIRE(n_chosen, "moe_prefetch_hottest: NULL n_chosen");
  MOE_REQUIRE(n_pending >= 0 && n_pending <= MOE_SCHED_MAX_EXPERTS,
              "moe_prefetch_hottest: n_pending=%d outside [0, %d]", n_pending, MOE_SCHED_MAX_EXPERTS);
  *n_chosen = 0;
  const int take = std::min(std::max(n_prefetch, 0), n_pending);
  if (take == 0) return MOE_OK;
  MOE_REQUIRE(host_pending && host_chosen, "moe_prefetch_hottest: NULL list with a positive length");
  std::vector<moe_pending> order(host_pending, host_pending + n_pending);
  std::sort(order.begin(), order.end(), [](const moe_pending& a, const moe_pending& b) {
    return a.tokens != b.tokens ? a.tokens > b.tokens : a.expert < b.expert;
  });
  for (int i = 0; i < take; ++i) host_chosen[i] = order[i].expert;
  *n_chosen = take;
  return MOE_OK;
}

extern "C" moe_status moe_presched(const moe_presched_costs* c, const moe_pending* host_cur,
                                   int32_t n_cur, const moe_pending* host_next, int32_t n_next,
                                   moe_presched_plan* out) {
  using moe::Entry;
  MOE_REQUIRE(c && out, "moe_presched: NULL pointer argument");
  MOE_REQUIRE(n_cur >= 0 && n_cur <= MOE_SCHED_MAX_EXPERTS && n_next >= 0 &&
                  n_next <= MOE_SCHED_MAX_EXPERTS,
              "moe_presched: n_cur=%d, n_next=%d outside [0, %d]", n_cur, n_next,
              MOE_SCHED_MAX_EXPERTS);
  MOE_REQUIRE((n_cur == 0 || host_cur) && (n_next == 0 || host_next),
              "moe_presched: NULL list with a positive length");
  MOE_REQUIRE(c->t_io > 0.0, "moe_presched: t_io=%g must be positive", c->t_io);
  MOE_REQUIRE(c->r_hit >= 0.0 && c->r_hit <= 1.0, "moe_presched: r_hit=%g outside [0,1]", c->r_hit);
  for (int i = 0; i < n_cur; ++i)
    MOE_REQUIRE(host_cur[i].tokens >= 0, "moe_presched: negative token count in the current list");
  for (int i = 0; i < n_next; ++i)
    MOE_REQUIRE(host_next[i].tokens >= 0, "moe_presched: negative token count in the next list");

  // Premise 1: each layer's pending experts by ascending tokens (equal: by id),
  // then one merged list; a next-layer entry goes below an equal current one
  std::vector<Entry> cur(n_cur), nxt(n_next), all;
  for (int i = 0; i < n_cur; ++i) cur[i] = {0, host_cur[i].expert, host_cur[i].tokens};
  for (int i = 0; i < n_next; ++i) nxt[i] = {1, host_next[i].expert, host_next[i].tokens};
  auto colder = [](const Entry& a, const Entry& b) {
    if (a.tokens != b.tokens) return a.tokens < b.tokens;
    if (a.layer != b.layer) return a.layer > b.layer;
    return a.expert < b.expert;
  };
  std::sort(cur.begin(), cur.end(), colder);
  std::sort(nxt.begin(), nxt.end(), colder);
  all.resize(n_cur + n_next);
  std::merge(cur.begin(), cur.end(), nxt.begin(), nxt.end(), all.begin(), colder);

  *out = moe_presched_plan{};
  out->n_cur = n_cur;
  out->n_next = n_next;
  out->n_all = n_cur + n_next;
  for (int i = 0; i < n_cur; ++i) out->cur_sorted[i] = cur[i].expert;
  for (int i = 0; i < n_next; ++i) out->next_sorted[i] = nxt[i].expert;

  std::vector<int32_t> tok_all(all.size()), tok_cur(cur.size());
  for (size_t i = 0; i < all.size(); ++i) tok_all[i] = all[i].tokens;
  for (size_t i = 0; i < cur.size(); ++i) tok_cur[i] = cur[i].tokens;
  const std::vector<double> cpu_all = moe::cpu_cost_prefix(tok_all, c->beta, c->C);
  const std::vector<double> cpu_cur = moe::cpu_cost_prefix(tok_cur, c->beta, c->C);

  // Q1 (Eq. 3): loading E_all[i..] and computing once on the GPU against
  // computing E_all[0..i] on the CPU behind the attention
  const int total = out->n_all;
  bool next_wanted = false;
  std::vector<char> cur_in_queue(n_cur, 0);
  int seen_cur = 0;
  for (int i = 0; i < total; ++i) {
    bool q = true;
    if (c->cpu_executor) {
      const double gpu = c->alpha + (double)(total - i) * c->t_io + c->t_g;
      const double cpu = cpu_all[i + 1] + c->t_attn;
      q = gpu < cpu;
    }
    out->all_layer[i] = all[i].layer;
    out->all_expert[i] = all[i].expert;
    out->all_in_queue[i] = q ? 1 : 0;
    if (all[i].layer == 1) next_wanted |= q;
    else cur_in_queue[seen_cur++] = q;   // the merge keeps each layer's own order
  }

  // Eq. 4: first queued index of E_cur whose load chain ends before the CPU is
  // through with the colder experts
  int ip = n_cur;
  if (!c->cpu_executor) {
    ip = 0;
  } else {
    for (int i = 0; i < n_cur; ++i) {
      if (!cur_in_queue[i]) continue;
      const double gpu = c->alpha + (double)(n_cur - i) * c->t_io + c->t_g;
      if (gpu < cpu_cur[i]) { ip = i; break; }
    }
  }
  out->i_prime = ip;
  for (int i = ip; i < n_cur; ++i) out->ondemand[out->n_ondemand++] = cur[i].expert;

  // Q2 (Eq. 5) and Q3 (Eq. 6)
  out->T_gap = cpu_cur[ip] - c->alpha - (double)(n_cur - ip) * c->t_io;
  out->f = (out->T_gap + c->t_attn) / c->t_io;
  const double rounded = std::floor(out->f + 0.5);
  out->f_abs = (int32_t)std::min<double>(std::max<double>(rounded, 0.0), (double)n_next);
  const double gain = c->r_hit * (out->f - out->f_abs + 1.0);
  const double loss = (1.0 - c->r_hit) * (out->f_abs - out->f);
  out->xi = gain * c->t_io - loss * c->t_io;

  // Q4, then the critical-prefetch rule
  if (next_wanted) {
    const int n_pf = std::max(gain > loss ? out->f_abs : out->f_abs - 1, 0);
    for (int j = 0; j < n_pf; ++j) out->prefetch[out->n_prefetch++] = nxt[n_next - 1 - j].expert;
  }
  return MOE_OK;
}
