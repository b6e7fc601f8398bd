// The whole MoE block (paper Section 2.1) with experts taken from wherever they
// live, and the streaming of non-resident experts (Section 4.4).
//
// What is kept from Section 4.4: fixed device slots registered once (an
// on-demand double buffer plus a prefetch buffer in two groups that rotate
// every layer, so a prefetch for layer l+1 can never overwrite an expert layer
// l still needs), pinned host memory with asynchronous copies, on-demand loads
// queued ahead of prefetches, and sub-tensor granularity (gate and up
// projections land first and the first FFN phase starts on them while the
// down projection is still in flight).  Expert traffic is one ordered queue
// (Section 2.3 observes concurrent expert transfers are no faster than serial
// ones), here a single side stream at default priority.
//
// Slot hand-over is ordered with events only: `copied_*` (side stream, after
// the bytes land) gates the compute stream; `released` (compute stream, after
// the last kernel that reads the slot) gates the side stream's next overwrite.
#include "common.h"

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

namespace moe {
namespace {

struct Slot {
  char* mem = nullptr;
  uint64_t layer_id = 0;
  int expert = -1;
  bool valid = false;        // holds (or is receiving) `expert` of `layer_id`
  bool has_release = false;  // `released` has been recorded at least once
  hipEvent_t copied = nullptr;     // borrowed from the copy record; NULL = bytes have landed
  bool gu_pending = false;         // `copied_gu` was recorded for the copy in flight
  hipEvent_t copied_gu = nullptr;  // owned: gate and up projections have landed
  hipEvent_t released = nullptr;   // owned: last reader on the compute stream is done
};

// One expert copy on the side stream.  `done` is recorded right after the
// bytes and doubles as the gate for the compute stream and as the end of the
// timed interval.  Back-to-back copies do not record a start marker of their
// own (every marker is a bubble on the link): their interval starts at the
// previous copy's `done`.
struct CopyRec {
  hipEvent_t start = nullptr;  // owned, or NULL when the interval starts at the previous `done`
  hipEvent_t done = nullptr;   // owned
  int64_t bytes = 0;
};

}  // namespace
}  // namespace moe

struct moe_ctx {
  moe_shape max_shape;
  size_t matrix_bytes = 0;  // one of the three matrices at max_shape
  int device = 0;
  std::vector<moe::Slot> ondemand;
  std::vector<moe::Slot> prefetch[2];
  int cur_group = 0;        // prefetch[cur_group] serves the layer being computed
  int od_next = 0;
  hipStream_t copy_stream = nullptr;
  hipEvent_t ev_counts = nullptr;
  int32_t* host_counts = nullptr;  // pinned, MOE_MAX_E ints
  // MOE_OPT_EXPORT_COUNTS: every layer call also leaves its per-expert token counts here
  bool export_counts = false;
  int32_t* export_host = nullptr;  // pinned, MOE_MAX_E ints
  hipEvent_t ev_export = nullptr;
  int export_n = 0;                // experts of the last exported layer (0: none yet)
  std::vector<moe::CopyRec> pending;   // queued copies in stream order, oldest first
  hipEvent_t held_done = nullptr;      // `done` of the newest harvested copy (the next
                                       // record may start its interval there)
  std::vector<hipEvent_t> free_events; // timing-enabled, reusable
  int64_t tot_bytes = 0, tot_copies = 0;
  double tot_ms = 0.0;
  bool sync_copies = false;  // control run: no copy/compute overlap at all
  int copy_split = 1;        // 1: one copy per expert when its matrices are contiguous on the
                             // host; 3: one copy per matrix, first phase gated on gate+up only
  // optional per-phase timing of all-resident layers (6 boundary events each)
  int phase_timing = 0;      // 0 off, 1 all five phases, 2 only the gate/up phase, 3 = 2 on every fourth call
  int phase_calls = 0;       // calls since the mode was set (mode 3 samples by it)
  std::vector<hipEvent_t> phase_events;  // 6 (or 2) per timed layer, in call order
  std::vector<int> phase_kinds;          // per timed layer: 1 or 2
  std::vector<hipEvent_t> phase_free;
  double phase_ms[5] = {0, 0, 0, 0, 0};
  int64_t phase_layers = 0;
  double gate_up_only_ms = 0.0;
  int64_t gate_up_only_layers = 0;
};

namespace moe {
namespace {

moe_status make_slot(Slot& s, size_t bytes) {
  MOE_HIP(hipMalloc(reinterpret_cast<void**>(&s.mem), bytes));
  // touch the slot now: the first write into fresh device memory pays for its
  // page mappings (measured: 78 ms for four 336 MiB slots inside the first
  // decode step that used them), and creation is the place for that
  MOE_HIP(hipMemset(s.mem, 0, bytes));
  MOE_HIP(hipEventCreateWithFlags(&s.copied_gu, hipEventDisableTiming));
  MOE_HIP(hipEventCreateWithFlags(&s.released, hipEventDisableTiming));
  return MOE_OK;
}

void drop_slot(Slot& s) {
  if (s.mem) (void)hipFree(s.mem);
  if (s.copied_gu) (void)hipEventDestroy(s.copied_gu);
  if (s.released) (void)hipEventDestroy(s.released);
  s = Slot();
}

// A completed `done` event goes back to the pool: no slot may keep gating on it.
void recycle_done(moe_ctx* c, hipEvent_t ev) {
  if (!ev) return;
  auto clear = [&](std::vector<Slot>& v) {
    for (Slot& sl : v)
      if (sl.copied == ev) {
        sl.copied = nullptr;
        sl.gu_pending = false;
      }
  };
  clear(c->ondemand);
  clear(c->prefetch[0]);
  clear(c->prefetch[1]);
  c->free_events.push_back(ev);
}

// Account for finished copies, oldest first (one stream: they finish in order).
moe_status harvest(moe_ctx* c, bool wait) {
  size_t n = 0;
  for (; n < c->pending.size(); ++n) {
    CopyRec& r = c->pending[n];
    hipError_t q = wait ? hipEventSynchronize(r.done) : hipEventQuery(r.done);
    if (q == hipErrorNotReady) break;
    if (q != hipSuccess) return fail(MOE_ERR_HIP, "event query: %s", hipGetErrorString(q));
    float ms = 0.f;
    hipEvent_t from = r.start ? r.start : c->held_done;
    if (from) MOE_HIP(hipEventElapsedTime(&ms, from, r.done));
    c->tot_ms += ms;
    c->tot_bytes += r.bytes;
    c->tot_copies += 1;
    if (r.start) c->free_events.push_back(r.start);
    recycle_done(c, c->held_done);
    c->held_done = r.done;
  }
  c->pending.erase(c->pending.begin(), c->pending.begin() + n);
  return MOE_OK;
}

moe_status timing_event(moe_ctx* c, hipEvent_t* out) {
  if (c->free_events.empty() && c->pending.size() >= 32) {
    moe_status st = harvest(c, false);
    if (st != MOE_OK) return st;
  }
  if (!c->free_events.empty()) {
    *out = c->free_events.back();
    c->free_events.pop_back();
    return MOE_OK;
  }
  MOE_HIP(hipEventCreate(out));
  return MOE_OK;
}

// Queue the copy of one expert into `slot` on the side stream.
moe_status queue_copy(moe_ctx* c, const moe_shape& s, Slot& slot, const moe_expert_ptrs& src,
                      uint64_t layer_id, int expert, hipStream_t compute) {
  const size_t mb = (size_t)s.H * s.F * elem_size(s);
  if (c->sync_copies) MOE_HIP(hipStreamSynchronize(compute));
  bool waited = false;
  if (slot.has_release) {
    // only put a wait on the link's queue if the last reader is really still running
    const hipError_t q = hipEventQuery(slot.released);
    if (q == hipErrorNotReady) {
      MOE_HIP(hipStreamWaitEvent(c->copy_stream, slot.released, 0));
      waited = true;
    } else if (q != hipSuccess) {
      return fail(MOE_ERR_HIP, "event query: %s", hipGetErrorString(q));
    }
  }
  CopyRec rec;
  rec.bytes = (int64_t)(3 * mb);
  moe_status st = timing_event(c, &rec.done);
  if (st != MOE_OK) return st;
  // back to back with a copy that is still in flight: the interval starts at its `done`
  bool chained = !waited && !c->sync_copies && !c->pending.empty();
  if (chained) {
    const hipError_t q = hipEventQuery(c->pending.back().done);
    chained = q == hipErrorNotReady;
  }
  if (!chained) {
    // the link was (or may be) idle: drain the bookkeeping so that no later
    // record borrows a stale `done`, then mark the start explicitly
    st = harvest(c, false);
    if (st != MOE_OK) return st;
    st = timing_event(c, &rec.start);
    if (st != MOE_OK) return st;
    MOE_HIP(hipEventRecord(rec.start, c->copy_stream));
  }
  const char* g = static_cast<const char*>(src.Wg);
  const bool contiguous = static_cast<const char*>(src.Wu) == g + mb &&
                          static_cast<const char*>(src.Wd) == g + 2 * mb;
  slot.gu_pending = false;
  if (c->copy_split == 1 && contiguous) {
    MOE_HIP(hipMemcpyAsync(slot.mem, src.Wg, 3 * mb, hipMemcpyHostToDevice, c->copy_stream));
  } else {
    // need order: the first FFN phase reads gate and up, the second reads down
    MOE_HIP(hipMemcpyAsync(slot.mem, src.Wg, mb, hipMemcpyHostToDevice, c->copy_stream));
    MOE_HIP(hipMemcpyAsync(slot.mem + mb, src.Wu, mb, hipMemcpyHostToDevice, c->copy_stream));
    if (c->copy_split == 3) {
      MOE_HIP(hipEventRecord(slot.copied_gu, c->copy_stream));
      slot.gu_pending = true;
    }
    MOE_HIP(hipMemcpyAsync(slot.mem + 2 * mb, src.Wd, mb, hipMemcpyHostToDevice, c->copy_stream));
  }
  MOE_HIP(hipEventRecord(rec.done, c->copy_stream));
  c->pending.push_back(rec);
  if (c->sync_copies) MOE_HIP(hipStreamSynchronize(c->copy_stream));
  slot.copied = rec.done;
  slot.layer_id = layer_id;
  slot.expert = expert;
  slot.valid = true;
  return MOE_OK;
}

moe_status phase_event(moe_ctx* c, hipStream_t stream) {
  hipEvent_t ev;
  if (!c->phase_free.empty()) {
    ev = c->phase_free.back();
    c->phase_free.pop_back();
  } else {
    MOE_HIP(hipEventCreate(&ev));
  }
  MOE_HIP(hipEventRecord(ev, stream));
  c->phase_events.push_back(ev);
  return MOE_OK;
}

inline bool bit(const uint64_t* m, int e) { return (m[e >> 6] >> (e & 63)) & 1ull; }

// Queue the copies of `layer`'s experts named in `mask` into the slots of one
// prefetch group (as many as it has), in ascending expert order.  Whatever the
// group held before is dropped.
moe_status issue_prefetch(moe_ctx* c, const moe_shape& s, std::vector<Slot>& group,
                          const moe_layer_desc* layer, const uint64_t* mask, hipStream_t stream,
                          int* n_issued) {
  MOE_REQUIRE(layer->host_pinned, "prefetch requested but the layer has no pinned copies");
  size_t used = 0;
  for (Slot& sl : group) sl.valid = false;
  for (int e = 0; e < s.E && used < group.size(); ++e) {
    if (!bit(mask, e)) continue;
    const moe_expert_ptrs& src = layer->host_pinned[e];
    MOE_REQUIRE(src.Wg && src.Wu && src.Wd, "prefetch of expert %d without a pinned copy", e);
    moe_status st = queue_copy(c, s, group[used], src, layer->layer_id, e, stream);
    if (st != MOE_OK) return st;
    ++used;
  }
  *n_issued = (int)used;
  return MOE_OK;
}

}  // namespace

}  // namespace moe

extern "C" moe_status moe_create(const moe_shape* max_shape, int32_t n_ondemand_slots,
                                 int32_t n_prefetch_slots_per_group, moe_ctx** out_ctx) {
  moe_status st = moe::check_shape(max_shape, "moe_create");
  if (st != MOE_OK) return st;
  MOE_REQUIRE(out_ctx, "moe_create: NULL out_ctx");
  MOE_REQUIRE(n_ondemand_slots >= 0 && n_prefetch_slots_per_group >= 0 &&
                  n_ondemand_slots != 1 && n_ondemand_slots <= 64 &&
                  n_prefetch_slots_per_group <= MOE_MAX_E,
              "moe_create: on-demand slots must be 0 or >= 2 (double buffer), got %d / %d",
              n_ondemand_slots, n_prefetch_slots_per_group);
  moe_ctx* c = new (std::nothrow) moe_ctx();
  if (!c) return moe::fail(MOE_ERR_HIP, "moe_create: out of host memory");
  c->max_shape = *max_shape;
  c->matrix_bytes = (size_t)max_shape->H * max_shape->F * moe::elem_size(*max_shape);
  st = MOE_OK;
  auto body = [&]() -> moe_status {
    MOE_HIP(hipGetDevice(&c->device));
    MOE_HIP(hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking));
    MOE_HIP(hipEventCreateWithFlags(&c->ev_counts, hipEventDisableTiming));
    MOE_HIP(hipHostMalloc(reinterpret_cast<void**>(&c->host_counts), MOE_MAX_E * sizeof(int32_t),
                          hipHostMallocDefault));
    MOE_HIP(hipHostMalloc(reinterpret_cast<void**>(&c->export_host), MOE_MAX_E * sizeof(int32_t),
                          hipHostMallocDefault));
    MOE_HIP(hipEventCreateWithFlags(&c->ev_export, hipEventDisableTiming));
    c->ondemand.resize(n_ondemand_slots);
    for (auto& s : c->ondemand) {
      moe_status r = moe::make_slot(s, 3 * c->matrix_bytes);
      if (r != MOE_OK) return r;
    }
    for (int g = 0; g < 2; ++g) {
      c->prefetch[g].resize(n_prefetch_slots_per_group);
      for (auto& s : c->prefetch[g]) {
        moe_status r = moe::make_slot(s, 3 * c->matrix_bytes);
        if (r != MOE_OK) return r;
      }
    }
    return MOE_OK;
  };
  st = body();
  if (st != MOE_OK) {
    moe_destroy(c);
    return st;
  }
  *out_ctx = c;
  return MOE_OK;
}

extern "C" moe_status moe_destroy(moe_ctx* c) {
  if (!c) return MOE_OK;
  if (c->copy_stream) (void)hipStreamSynchronize(c->copy_stream);
  (void)hipDeviceSynchronize();
  for (auto& s : c->ondemand) moe::drop_slot(s);
  for (int g = 0; g < 2; ++g)
    for (auto& s : c->prefetch[g]) moe::drop_slot(s);
  for (auto& r : c->pending) {
    if (r.start) (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.done);
  }
  if (c->held_done) (void)hipEventDestroy(c->held_done);
  for (auto& e : c->free_events) (void)hipEventDestroy(e);
  for (auto& e : c->phase_events) (void)hipEventDestroy(e);
  for (auto& e : c->phase_free) (void)hipEventDestroy(e);
  if (c->ev_counts) (void)hipEventDestroy(c->ev_counts);
  if (c->host_counts) (void)hipHostFree(c->host_counts);
  if (c->export_host) (void)hipHostFree(c->export_host);
  if (c->ev_export) (void)hipEventDestroy(c->ev_export);
  if (c->copy_stream) (void)hipStreamDestroy(c->copy_stream);
  delete c;
  return MOE_OK;
}

extern "C" moe_status moe_stream_totals_get(moe_ctx* c, moe_stream_totals* out, int32_t reset) {
  MOE_REQUIRE(c && out, "moe_stream_totals_get: NULL argument");
  MOE_HIP(hipStreamSynchronize(c->copy_stream));
  moe_status st = moe::harvest(c, true);
  if (st != MOE_OK) return st;
  out->bytes = c->tot_bytes;
  out->n_copies = c->tot_copies;
  out->copy_ms = c->tot_ms;
  if (reset) {
    c->tot_bytes = 0;
    c->tot_copies = 0;
    c->tot_ms = 0.0;
  }
  return MOE_OK;
}

extern "C" moe_status moe_layer_forward(moe_ctx* c, const moe_shape* shape,
                                        const moe_layer_desc* layer,
                                        const uint64_t* host_resident_mask,
                                        const moe_layer_desc* next_layer,
                                        const uint64_t* host_prefetch_next_mask, const void* X,
                                        const void* residual, void* out, void* workspace,
                                        void* stream_, moe_layer_stats* stats) {
  using namespace moe;
  moe_status st = check_shape(shape, "moe_layer_forward");
  if (st != MOE_OK) return st;
  const moe_shape& s = *shape;
  MOE_REQUIRE(c && layer, "moe_layer_forward: NULL context or layer");
  MOE_REQUIRE(layer->Wr && layer->host_dev, "moe_layer_forward: layer without router or expert table");
  if (!workspace) return fail(MOE_ERR_WORKSPACE, "moe_layer_forward: NULL workspace");
  if (stats) {
    *stats = moe_layer_stats();
    stats->n_active = -1;
  }
  if (s.T == 0) return MOE_OK;
  MOE_REQUIRE(X && out, "moe_layer_forward: NULL X or out");
  MOE_REQUIRE((size_t)s.H * s.F * elem_size(s) <= c->matrix_bytes || (c->ondemand.empty() && c->prefetch[0].empty()),
              "moe_layer_forward: expert larger than the context's slots");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const WorkspaceLayout L = workspace_layout(s);
  char* w = static_cast<char*>(workspace);
  int32_t* topk_idx = reinterpret_cast<int32_t*>(w + L.topk_idx);
  float* topk_w = reinterpret_cast<float*>(w + L.topk_w);
  int32_t* count = reinterpret_cast<int32_t*>(w + L.count);
  int32_t* offset = reinterpret_cast<int32_t*>(w + L.offset);
  int32_t* perm = reinterpret_cast<int32_t*>(w + L.perm);
  int32_t* inv_perm = reinterpret_cast<int32_t*>(w + L.inv_perm);
  const FfnScratch h{w + L.h};
  void* Y = w + L.y;
  const bool y_bf16 = layer_y_bf16(s);   // rows of Y in bf16 at prefill sizes (see launch_ffn_down)
  const size_t mb = (size_t)s.H * s.F * elem_size(s);

  bool all_resident = true;
  if (host_resident_mask)
    for (int e = 0; e < s.E; ++e) all_resident = all_resident && bit(host_resident_mask, e);
  for (int e = 0; e < s.E + s.S; ++e) {
    const bool res = e >= s.E || !host_resident_mask || bit(host_resident_mask, e);
    if (res)
      MOE_REQUIRE(layer->host_dev[e].Wg && layer->host_dev[e].Wu && layer->host_dev[e].Wd,
                  "moe_layer_forward: resident expert %d has a NULL device matrix", e);
    else
      MOE_REQUIRE(layer->host_pinned && layer->host_pinned[e].Wg && layer->host_pinned[e].Wu &&
                      layer->host_pinned[e].Wd,
                  "moe_layer_forward: non-resident expert %d has no pinned host copy", e);
  }

  int timed = all_resident ? c->phase_timing : 0;
  if (timed == 3) timed = (c->phase_calls++ & 3) == 0 ? 2 : 0;
  // mark i of the six phase boundaries; mode 2 records only the two around gate/up
#define PHASE_MARK(i)                                            \
  do {                                                           \
    if (timed == 1 || (timed == 2 && ((i) == 2 || (i) == 3))) {  \
      moe_status _p = phase_event(c, stream);                    \
      if (_p != MOE_OK) return _p;                               \
    }                                                            \
  } while (0)
  if (timed) c->phase_kinds.push_back(timed);
  PHASE_MARK(0);
  bool bucketed = false;   // a batch of one token: the selecting launch buckets as well
  st = launch_route_bucket(s, X, layer->Wr, layer->bias, topk_idx, topk_w,
                           reinterpret_cast<double*>(w + L.logits), count, offset, perm, inv_perm, stream,
                           &bucketed);
  if (st != MOE_OK) return st;
  PHASE_MARK(1);
  if (!bucketed) st = launch_permute(s, topk_idx, count, offset, perm, inv_perm, stream);
  if (st != MOE_OK) return st;
  if (c->export_counts) {
    // for a scheduler on the host: the counts travel while the FFN runs, and
    // nobody waits for them here (moe_layer_counts does)
    MOE_HIP(hipMemcpyAsync(c->export_host, count, s.E * sizeof(int32_t), hipMemcpyDeviceToHost, stream));
    MOE_HIP(hipEventRecord(c->ev_export, stream));
    c->export_n = s.E;
  }
  PHASE_MARK(2);

  ExpertTable tab;
  for (int e = 0; e < s.E + s.S; ++e) {
    tab.Wg[e] = layer->host_dev[e].Wg;
    tab.Wu[e] = layer->host_dev[e].Wu;
    tab.Wd[e] = layer->host_dev[e].Wd;
  }
  GroupList res_groups;
  res_groups.n = 0;
  std::vector<Slot>& cur = c->prefetch[c->cur_group];
  std::vector<Slot>& nxt = c->prefetch[c->cur_group ^ 1];

  if (all_resident) {
    // nothing to decide on the host: kernels skip empty buckets by themselves
    for (int e = 0; e < s.E + s.S; ++e) res_groups.id[res_groups.n++] = (uint8_t)e;
    st = launch_ffn_gate_up(s, X, perm, offset, tab, res_groups, h, stream);
    if (st != MOE_OK) return st;
    PHASE_MARK(3);
    st = launch_ffn_down(s, h, perm, offset, tab, res_groups, Y, stream, y_bf16);
    if (st != MOE_OK) return st;
    PHASE_MARK(4);
  } else {
    // The host must know which experts are active before it can queue copies --
    // unless there is nothing it could have to copy: every non-resident expert
    // already sits in a prefetch slot for this layer.  Then the call does not
    // wait for the router (the kernels skip empty buckets by themselves, so every
    // expert is simply listed), which keeps the compute stream fed across layers;
    // a caller that asks for stats still gets the exact counts and pays the wait.
    bool covered = stats == nullptr;
    if (covered) {
      bool in_slot[MOE_MAX_E] = {};
      for (const Slot& sl : cur)
        if (sl.valid && sl.layer_id == layer->layer_id && sl.expert >= 0 && sl.expert < s.E)
          in_slot[sl.expert] = true;
      for (int e = 0; e < s.E; ++e) covered = covered && (bit(host_resident_mask, e) || in_slot[e]);
    }
    if (covered) {
      for (int e = 0; e < s.E; ++e) c->host_counts[e] = 1;
    } else {
      MOE_HIP(hipMemcpyAsync(c->host_counts, count, s.E * sizeof(int32_t), hipMemcpyDeviceToHost, stream));
      MOE_HIP(hipEventRecord(c->ev_counts, stream));
      MOE_HIP(hipEventSynchronize(c->ev_counts));
    }
    int n_active = 0, n_res = 0, n_hit = 0, n_miss = 0, n_wasted = 0;
    int hit_slot[MOE_MAX_E];
    std::vector<int> hits, misses;
    for (int e = 0; e < s.E; ++e) {
      hit_slot[e] = -1;
      const bool active = c->host_counts[e] > 0;
      const bool res = bit(host_resident_mask, e);
      if (active) ++n_active;
      if (active && res) {
        ++n_res;
        res_groups.id[res_groups.n++] = (uint8_t)e;
      }
    }
    for (size_t i = 0; i < cur.size(); ++i) {
      Slot& sl = cur[i];
      if (!sl.valid || sl.layer_id != layer->layer_id || sl.expert < 0 || sl.expert >= s.E) continue;
      const int e = sl.expert;
      if (c->host_counts[e] > 0 && !bit(host_resident_mask, e) && hit_slot[e] < 0) {
        hit_slot[e] = (int)i;
        hits.push_back(e);
        ++n_hit;
      } else {
        ++n_wasted;
      }
    }
    for (int e = 0; e < s.E; ++e)
      if (c->host_counts[e] > 0 && !bit(host_resident_mask, e) && hit_slot[e] < 0) misses.push_back(e);
    n_miss = (int)misses.size();
    if (n_miss > 0 && c->ondemand.empty())
      return fail(MOE_ERR_SLOT_EXHAUSTED,
                  "moe_layer_forward: %d expert(s) need an on-demand load but the context has no on-demand slots",
                  n_miss);
    for (int sx = 0; sx < s.S; ++sx) res_groups.id[res_groups.n++] = (uint8_t)(s.E + sx);

    // Prefetched experts: their copies were queued during the previous layer, in
    // slot order on the one side stream, so the hit in the highest slot was copied
    // last and once its bytes have landed so have the others'.
    GroupList hit_groups;
    hit_groups.n = 0;
    Slot* newest = nullptr;
    int newest_at = -1;
    for (int e : hits) {
      Slot& sl = cur[hit_slot[e]];
      tab.Wg[e] = sl.mem;
      tab.Wu[e] = sl.mem + mb;
      tab.Wd[e] = sl.mem + 2 * mb;
      hit_groups.id[hit_groups.n++] = (uint8_t)e;
      if (hit_slot[e] > newest_at) {
        newest_at = hit_slot[e];
        newest = &sl;
      }
    }
    // They join the residents' launch when they have already landed (as good as
    // resident), and also when a launch of their own could not fill the chip
    // (small experts: a few tens of work items cost two under-filled launches,
    // more than waiting for a copy that was queued a whole layer ago); the joint
    // launch then waits for the newest of their copies.  Large experts keep the
    // order "residents first, streamed experts behind their copies".
    bool hits_joined = false;
    hipEvent_t join_gu = nullptr, join_d = nullptr;
    if (newest) {
      const bool landed = !newest->copied || hipEventQuery(newest->copied) == hipSuccess;
      const bool small = (size_t)hit_groups.n * 3 * mb < ((size_t)64 << 20);
      hits_joined = landed || small;
      if (hits_joined) {
        for (int i = 0; i < hit_groups.n; ++i) res_groups.id[res_groups.n++] = hit_groups.id[i];
        if (!landed) {
          join_gu = newest->gu_pending ? newest->copied_gu : newest->copied;
          join_d = newest->copied;
        }
      }
    }

    // resident experts first: they need nothing from the link
    st = launch_ffn_gated(s, X, perm, offset, tab, res_groups, Y, h, stream, join_gu, join_d, nullptr, y_bf16);
    if (st != MOE_OK) return st;
    // hits still in flight: ONE grouped launch behind the newest of their copies
    // (sub-tensor mode: its gate and up projections landing gates the first
    // phase); a launch per expert costs more in launch and fill overhead than it
    // could win back
    if (newest && !hits_joined) {
      st = launch_ffn_gated(s, X, perm, offset, tab, hit_groups, Y, h, stream,
                            newest->gu_pending ? newest->copied_gu : newest->copied,
                            newest->copied, nullptr, y_bf16);
      if (st != MOE_OK) return st;
    }
    for (int e : hits) {
      Slot& sl = cur[hit_slot[e]];
      MOE_HIP(hipEventRecord(sl.released, stream));
      sl.has_release = true;
    }
    // on-demand loads, through the double buffer, ahead of any new prefetch.
    // Large experts run one launch each, as soon as their own copy has landed
    // (the next copy flies meanwhile); small ones are copied a buffer-full at a
    // time and run as one launch behind the last of those copies.
    const size_t per_launch = (3 * mb < ((size_t)32 << 20)) ? c->ondemand.size() : 1;
    for (size_t m0 = 0; m0 < misses.size(); m0 += per_launch) {
      GroupList batch;
      batch.n = 0;
      Slot* last = nullptr;
      std::vector<Slot*> used;
      for (size_t m = m0; m < std::min(misses.size(), m0 + per_launch); ++m) {
        const int e = misses[m];
        Slot& sl = c->ondemand[c->od_next];
        c->od_next = (c->od_next + 1) % (int)c->ondemand.size();
        st = queue_copy(c, s, sl, layer->host_pinned[e], layer->layer_id, e, stream);
        if (st != MOE_OK) return st;
        tab.Wg[e] = sl.mem;
        tab.Wu[e] = sl.mem + mb;
        tab.Wd[e] = sl.mem + 2 * mb;
        batch.id[batch.n++] = (uint8_t)e;
        last = &sl;
        used.push_back(&sl);
        if (stats) stats->bytes_on_demand += (int64_t)(3 * mb);
      }
      st = launch_ffn_gated(s, X, perm, offset, tab, batch, Y, h, stream,
                            last->gu_pending ? last->copied_gu : last->copied, last->copied, nullptr,
                            y_bf16);
      if (st != MOE_OK) return st;
      for (Slot* sl : used) {
        MOE_HIP(hipEventRecord(sl->released, stream));
        sl->has_release = true;
      }
    }
    if (stats) {
      stats->n_active = n_active;
      stats->n_resident = n_res;
      stats->n_hit = n_hit;
      stats->n_miss = n_miss;
      stats->n_wasted = n_wasted;
    }
  }

  // the current group has served this layer (its readers are queued and have
  // recorded `released`); it becomes the target of the layer after next
  for (Slot& sl : cur) sl.valid = false;

  st = launch_combine(s, Y, topk_w, inv_perm, residual, out, stream, y_bf16);
  if (st != MOE_OK) return st;
  PHASE_MARK(5);
#undef PHASE_MARK

  // prefetch for the next layer, behind every on-demand copy queued above
  if (next_layer && host_prefetch_next_mask && !nxt.empty()) {
    int issued = 0;
    st = issue_prefetch(c, s, nxt, next_layer, host_prefetch_next_mask, stream, &issued);
    if (st != MOE_OK) return st;
    if (stats) {
      stats->n_prefetch_issued += issued;
      stats->bytes_prefetch += (int64_t)issued * (int64_t)(3 * mb);
    }
  }
  c->cur_group ^= 1;
  return MOE_OK;
}

extern "C" moe_status moe_prefetch(moe_ctx* c, const moe_shape* shape, const moe_layer_desc* next_layer,
                                   const uint64_t* host_prefetch_mask, void* stream_,
                                   int32_t* n_issued) {
  using namespace moe;
  moe_status st = check_shape(shape, "moe_prefetch");
  if (st != MOE_OK) return st;
  MOE_REQUIRE(c && next_layer && host_prefetch_mask, "moe_prefetch: NULL argument");
  MOE_REQUIRE((size_t)shape->H * shape->F * elem_size(*shape) <= c->matrix_bytes,
              "moe_prefetch: expert larger than the context's slots");
  if (n_issued) *n_issued = 0;
  // the group the NEXT moe_layer_forward call reads
  std::vector<Slot>& tgt = c->prefetch[c->cur_group];
  if (tgt.empty()) return MOE_OK;
  int issued = 0;
  st = issue_prefetch(c, *shape, tgt, next_layer, host_prefetch_mask, static_cast<hipStream_t>(stream_),
                      &issued);
  if (n_issued) *n_issued = issued;
  return st;
}

extern "C" moe_status moe_layer_counts(moe_ctx* c, int32_t* host_count, int32_t E) {
  MOE_REQUIRE(c && host_count, "moe_layer_counts: NULL argument");
  MOE_REQUIRE(c->export_n > 0, "moe_layer_counts: no layer has exported its counts (set MOE_OPT_EXPORT_COUNTS first)");
  MOE_REQUIRE(E == c->export_n, "moe_layer_counts: the last layer had %d experts, not %d", c->export_n, E);
  MOE_HIP(hipEventSynchronize(c->ev_export));
  for (int e = 0; e < E; ++e) host_count[e] = c->export_host[e];
  return MOE_OK;
}

// ---- the block for callers that cannot allocate ---------------------------
// The workspace of an all-resident layer lives in a fixed device array inside
// the library.  In host code the array's name is only a stand-in for the
// symbol: its device address is looked up once per device, with that device
// current, and that address is what every kernel and copy is handed.
static __device__ __align__(256) unsigned char scratch[MOE_STATIC_WORKSPACE_BYTES];

namespace moe {
namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of this device's copy of `scratch` (every GPU the library runs
// on holds its own copy at its own address).
moe_status static_workspace(void** out) {
  int dev = -1;
  MOE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices)
    return fail(MOE_ERR_UNSUPPORTED, "moe_layer_forward_static: device index %d out of range", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    MOE_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(MOE_ERR_HIP, "moe_layer_forward_static: the scratch symbol has no device address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MOE_OK;
}

}  // namespace
}  // namespace moe

extern "C" size_t moe_static_workspace_bytes(void) { return MOE_STATIC_WORKSPACE_BYTES; }

extern "C" moe_status moe_layer_forward_static(const moe_shape* shape, const moe_layer_desc* layer,
                                               const void* X, const void* residual, void* out,
                                               void* stream_) {
  using namespace moe;
  moe_status st = check_shape(shape, "moe_layer_forward_static");
  if (st != MOE_OK) return st;
  const moe_shape& s = *shape;
  MOE_REQUIRE(layer && layer->Wr && layer->host_dev,
              "moe_layer_forward_static: layer without router or expert table");
  const WorkspaceLayout L = workspace_layout(s);
  if (L.total > (size_t)MOE_STATIC_WORKSPACE_BYTES)
    return fail(MOE_ERR_WORKSPACE,
                "moe_layer_forward_static: this shape needs %zu bytes of workspace, the fixed array "
                "holds %zu; use moe_layer_forward with a caller-allocated workspace",
                L.total, (size_t)MOE_STATIC_WORKSPACE_BYTES);
  if (s.T == 0) return MOE_OK;
  MOE_REQUIRE(X && out, "moe_layer_forward_static: NULL X or out");
  ExpertTable tab;
  GroupList groups;
  groups.n = 0;
  for (int e = 0; e < s.E + s.S; ++e) {
    MOE_REQUIRE(layer->host_dev[e].Wg && layer->host_dev[e].Wu && layer->host_dev[e].Wd,
                "moe_layer_forward_static: expert %d has a NULL device matrix (every expert must be resident)", e);
    tab.Wg[e] = layer->host_dev[e].Wg;
    tab.Wu[e] = layer->host_dev[e].Wu;
    tab.Wd[e] = layer->host_dev[e].Wd;
    groups.id[groups.n++] = (uint8_t)e;
  }
  void* base = nullptr;
  st = static_workspace(&base);
  if (st != MOE_OK) return st;
  char* w = static_cast<char*>(base);
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  int32_t* topk_idx = reinterpret_cast<int32_t*>(w + L.topk_idx);
  float* topk_w = reinterpret_cast<float*>(w + L.topk_w);
  int32_t* count = reinterpret_cast<int32_t*>(w + L.count);
  int32_t* offset = reinterpret_cast<int32_t*>(w + L.offset);
  int32_t* perm = reinterpret_cast<int32_t*>(w + L.perm);
  int32_t* inv_perm = reinterpret_cast<int32_t*>(w + L.inv_perm);
  const FfnScratch h{w + L.h};
  void* Y = w + L.y;
  const bool y_bf16 = layer_y_bf16(s);   // as in moe_layer_forward: the two must agree bit for bit
  // nothing in the workspace has to start at zero: every kernel below writes
  // what the next one reads (the previous call's contents are simply overwritten)
  bool bucketed = false;
  st = launch_route_bucket(s, X, layer->Wr, layer->bias, topk_idx, topk_w,
                           reinterpret_cast<double*>(w + L.logits), count, offset, perm, inv_perm, stream,
                           &bucketed);
  if (st != MOE_OK) return st;
  if (!bucketed) st = launch_permute(s, topk_idx, count, offset, perm, inv_perm, stream);
  if (st != MOE_OK) return st;
  st = launch_ffn_gate_up(s, X, perm, offset, tab, groups, h, stream);
  if (st != MOE_OK) return st;
  st = launch_ffn_down(s, h, perm, offset, tab, groups, Y, stream, y_bf16);
  if (st != MOE_OK) return st;
  return launch_combine(s, Y, topk_w, inv_perm, residual, out, stream, y_bf16);
}

extern "C" moe_status moe_set_option(moe_ctx* c, int32_t option, int64_t value) {
  MOE_REQUIRE(c, "moe_set_option: NULL context");
  switch (option) {
    case MOE_OPT_SYNC_COPIES:
      c->sync_copies = value != 0;
      return MOE_OK;
    case MOE_OPT_EXPORT_COUNTS:
      c->export_counts = value != 0;
      return MOE_OK;
    case MOE_OPT_COPY_SPLIT:
      MOE_REQUIRE(value == 1 || value == 3, "moe_set_option: copy split must be 1 or 3");
      c->copy_split = (int)value;
      return MOE_OK;
    default:
      return moe::fail(MOE_ERR_INVALID_ARG, "moe_set_option: unknown option %d", option);
  }
}

extern "C" moe_status moe_phase_timing(moe_ctx* c, int32_t mode) {
  MOE_REQUIRE(c, "moe_phase_timing: NULL context");
  MOE_REQUIRE(mode >= 0 && mode <= 3, "moe_phase_timing: mode must be 0, 1, 2 or 3");
  c->phase_timing = mode;
  c->phase_calls = 0;
  return MOE_OK;
}

extern "C" moe_status moe_phase_times_get(moe_ctx* c, moe_phase_times* out, int32_t reset) {
  MOE_REQUIRE(c && out, "moe_phase_times_get: NULL argument");
  size_t at = 0;
  for (size_t l = 0; l < c->phase_kinds.size(); ++l) {
    const int kind = c->phase_kinds[l];
    const size_t n = kind == 1 ? 6 : 2;
    if (at + n > c->phase_events.size()) break;
    MOE_HIP(hipEventSynchronize(c->phase_events[at + n - 1]));
    if (kind == 1) {
      for (int p = 0; p < 5; ++p) {
        float ms = 0.f;
        MOE_HIP(hipEventElapsedTime(&ms, c->phase_events[at + p], c->phase_events[at + p + 1]));
        c->phase_ms[p] += ms;
      }
      c->phase_layers += 1;
    } else {
      float ms = 0.f;
      MOE_HIP(hipEventElapsedTime(&ms, c->phase_events[at], c->phase_events[at + 1]));
      c->gate_up_only_ms += ms;
      c->gate_up_only_layers += 1;
    }
    at += n;
  }
  for (hipEvent_t e : c->phase_events) c->phase_free.push_back(e);
  c->phase_events.clear();
  c->phase_kinds.clear();
  out->route_ms = c->phase_ms[0];
  out->permute_ms = c->phase_ms[1];
  out->gate_up_ms = c->phase_ms[2];
  out->down_ms = c->phase_ms[3];
  out->combine_ms = c->phase_ms[4];
  out->n_layers = c->phase_layers;
  out->gate_up_only_ms = c->gate_up_only_ms;
  out->gate_up_only_layers = c->gate_up_only_layers;
  if (reset) {
    for (double& v : c->phase_ms) v = 0.0;
    c->phase_layers = 0;
    c->gate_up_only_ms = 0.0;
    c->gate_up_only_layers = 0;
  }
  return MOE_OK;
}
