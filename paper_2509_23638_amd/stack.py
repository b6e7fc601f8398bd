"""Driver of a stack of MoE blocks with streamed experts (argument marshalling
and call sequencing only; the arithmetic is in the library's kernels).

x_{l+1} = x_l + Block_l(rmsnorm(x_l)).  Per layer a residency mask says which
routed experts live in device memory; the others live in pinned host memory and
reach the GPU through the context's slots, either prefetched one layer ahead
(mask supplied by the caller) or on demand.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def _to_torch(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16)
    return torch.from_numpy(a)


class StreamedStack:
    def __init__(self, shape: B.moe_shape, layers_host: Sequence[dict],
                 resident_masks: Sequence[Sequence[bool]], n_ondemand_slots=2,
                 n_prefetch_slots_per_group=2, n_layers: Optional[int] = None):
        """layers_host: dicts with numpy Wr, b, Wg, Wu, Wd ([E+S, ...]).  If
        ``n_layers`` exceeds len(layers_host) the weights repeat with that
        period (each layer still has its own id, mask and slot traffic)."""
        self.shape = shape
        self.n_layers = n_layers or len(layers_host)
        self.ctx = B.Context(shape, n_ondemand_slots, n_prefetch_slots_per_group)
        self.ws = B.alloc_workspace(shape)
        self.resident = [list(m) for m in resident_masks]
        E, S = shape.E, shape.S
        P = len(layers_host)
        # one device / pinned copy per (weight period, expert), chosen by the
        # union of what the layers sharing those weights need
        need_dev = [[False] * (E + S) for _ in range(P)]
        need_pin = [[False] * (E + S) for _ in range(P)]
        for l in range(self.n_layers):
            for e in range(E + S):
                res = e >= E or self.resident[l][e]
                (need_dev if res else need_pin)[l % P][e] = True
        self._dev, self._pin, self._router = [], [], []
        self._pin_blocks = []
        for p, L in enumerate(layers_host):
            dev = {n: [None] * (E + S) for n in ("Wg", "Wu", "Wd")}
            pin = {n: [None] * (E + S) for n in ("Wg", "Wu", "Wd")}
            tiled = shape.weight_layout == B.MOE_TILED
            for e in range(E + S):
                ts = [_to_torch(L[n][e]) for n in ("Wg", "Wu", "Wd")]
                if tiled:
                    # pack once at load time, on the device; host copies hold the packed bytes
                    packed = []
                    for t in ts:
                        d = t.cuda()
                        o = torch.empty_like(d)
                        B.moe_pack_weights(d, o, t.shape[0], t.shape[1])
                        packed.append(o)
                    torch.cuda.synchronize()
                    ts = packed
                if need_dev[p][e]:
                    for n, t in zip(("Wg", "Wu", "Wd"), ts):
                        dev[n][e] = t.cuda()
                if need_pin[p][e]:
                    # the three matrices back to back: one copy moves the expert
                    blk = torch.empty(3 * ts[0].numel(), dtype=ts[0].dtype, pin_memory=True)
                    self._pin_blocks.append(blk)
                    for i, (n, t) in enumerate(zip(("Wg", "Wu", "Wd"), ts)):
                        v = blk[i * t.numel():(i + 1) * t.numel()].view(t.shape)
                        v.copy_(t)
                        pin[n][e] = v
            self._dev.append(dev)
            self._pin.append(pin)
            self._router.append((_to_torch(L["Wr"]).cuda(), _to_torch(L["b"]).cuda()))
        self.layers: List[B.Layer] = []
        for l in range(self.n_layers):
            p = l % P
            d, h = self._dev[p], self._pin[p]
            self.layers.append(B.make_layer_desc(
                shape, self._router[p][0], self._router[p][1],
                dev=(d["Wg"], d["Wu"], d["Wd"]), pinned=(h["Wg"], h["Wu"], h["Wd"]), layer_id=l))
        self._norm = None
        self._pred = torch.zeros(E, dtype=torch.int32, device="cuda")
        self._pred_host = None
        self._pred_event = None
        self._cur = torch.zeros(E, dtype=torch.int32, device="cuda")
        self._in_slot = [set() for _ in range(self.n_layers)]   # experts prefetched for layer l
        self.sched_log = {"n_decisions": 0, "n_prefetch_planned": 0, "f_sum": 0.0}

    def close(self):
        self.ctx.close()

    def warm_host_copies(self):
        """One host-to-device copy of every pinned expert block into a scratch
        buffer, meant for load time (outside any timed region): the first
        transfer out of freshly pinned pages is slower than the later ones, and a
        serving process should not pay that inside its first decode steps."""
        if not self._pin_blocks:
            return
        scratch = torch.empty(max(b.numel() for b in self._pin_blocks),
                              dtype=self._pin_blocks[0].dtype, device="cuda")
        for b in self._pin_blocks:
            scratch[:b.numel()].copy_(b, non_blocking=True)
        torch.cuda.synchronize()

    def layer_forward(self, l: int, x_in: torch.Tensor, out: torch.Tensor, residual=None,
                      prefetch_next_mask=None, next_l: Optional[int] = None, want_stats=True):
        """One block on an already normalised input."""
        nl = self.layers[next_l] if next_l is not None else None
        return B.moe_layer_forward(self.ctx, self.shape, self.layers[l], x_in, out, self.ws,
                                   resident_mask=self.resident[l], next_layer=nl,
                                   prefetch_next_mask=prefetch_next_mask, residual=residual,
                                   want_stats=want_stats)

    def step(self, X: torch.Tensor, prefetch_masks: Optional[Sequence] = None,
             wrap_prefetch: bool = False, want_stats=True):
        """One pass of the residual stream through all layers.  prefetch_masks[l]
        (or None) names the experts of layer l+1 to start copying while layer l
        computes; with ``wrap_prefetch`` the last entry targets layer 0 of the
        next step.  Returns (x_final, list of per-layer stats)."""
        if self._norm is None or self._norm.shape != X.shape:
            self._norm = torch.empty_like(X)
            self._bufs = [torch.empty_like(X), torch.empty_like(X)]
        x = X
        stats = []
        for l in range(self.n_layers):
            B.moe_rmsnorm(self.shape, x, self._norm)
            out = self._bufs[l & 1]
            nxt = l + 1 if l + 1 < self.n_layers else (0 if wrap_prefetch else None)
            pm = prefetch_masks[l] if (prefetch_masks is not None and nxt is not None) else None
            stats.append(self.layer_forward(l, self._norm, out, residual=x, prefetch_next_mask=pm,
                                            next_l=nxt if pm is not None else None,
                                            want_stats=want_stats))
            x = out
        return x, stats


    # ---- online prefetch policies (Section 3.2 predictor + Section 4.3 scheduler) ----
    def predicted_counts(self, l_router: int, x_norm: torch.Tensor, into: torch.Tensor) -> np.ndarray:
        """Tokens per expert when ``x_norm`` is routed by layer ``l_router``'s
        gate (device work in the library; the E counts come back to the host)."""
        Wr, b = self.layers[l_router].keep[0], self.layers[l_router].keep[1]
        B.moe_predict_counts(self.shape, x_norm, Wr, b, into, self.ws)
        return into.cpu().numpy()

    def _predict_async(self, l_router: int, x_norm: torch.Tensor):
        """Queue the gate-based prediction and the copy of its E counts to pinned
        host memory; nobody waits here."""
        if self._pred_host is None:
            self._pred_host = torch.empty(self.shape.E, dtype=torch.int32, pin_memory=True)
            self._pred_event = torch.cuda.Event()
        Wr, b = self.layers[l_router].keep[0], self.layers[l_router].keep[1]
        B.moe_predict_counts(self.shape, x_norm, Wr, b, self._pred, self.ws)
        self._pred_host.copy_(self._pred, non_blocking=True)
        self._pred_event.record()

    def _predict_wait(self) -> np.ndarray:
        self._pred_event.synchronize()
        return self._pred_host.numpy().copy()

    def step_online(self, X: torch.Tensor, policy: str, costs: Optional[B.moe_presched_costs] = None,
                    n_prefetch: int = 2, wrap_prefetch: bool = False, want_stats: bool = True):
        """One pass with the prefetch set decided online, layer by layer:

        ``gate_topn``  -- the ``n_prefetch`` non-resident experts of the next
                          layer with the most predicted tokens (gate-based
                          prediction from this layer's input);
        ``presched``   -- the same prediction fed to PreSched together with this
                          layer's own pending experts (its actual token counts,
                          exported by the layer call); the plan's prefetch list
                          (cut to the slots available) is issued;
        ``none``       -- on-demand loads only.

        Order per layer: the prediction is queued ahead of the layer, the layer
        is queued, and only then does the host wait for the (long finished)
        prediction, decide, and queue the prefetch as a call of its own -- so the
        decision runs in the shadow of the layer's GPU work and the copies start
        while that layer computes.  Returns (x_final, list of per-layer stats;
        ``n_prefetch_issued`` / ``bytes_prefetch`` are filled in here)."""
        E = self.shape.E
        if self._norm is None or self._norm.shape != X.shape:
            self._norm = torch.empty_like(X)
            self._bufs = [torch.empty_like(X), torch.empty_like(X)]
        self.ctx.set_export_counts(policy == "presched")
        expert_bytes = 3 * self.shape.H * self.shape.F * (2 if self.shape.dtype == B.MOE_BF16 else 4)
        x = X
        stats = []
        for l in range(self.n_layers):
            B.moe_rmsnorm(self.shape, x, self._norm)
            out = self._bufs[l & 1]
            nxt = l + 1 if l + 1 < self.n_layers else (0 if wrap_prefetch else None)
            online = nxt is not None and policy != "none"
            if online:
                self._predict_async(nxt, self._norm)
            st = self.layer_forward(l, self._norm, out, residual=x, want_stats=want_stats)
            in_slot = [e in self._in_slot[l] for e in range(E)]   # prefetched for this layer: not pending
            self._in_slot[l] = set()
            if online:
                cand = B.moe_pending_experts(self._predict_wait(), self.resident[nxt])
                if policy == "gate_topn":
                    chosen = B.moe_prefetch_hottest(cand, n_prefetch)
                elif policy == "presched":
                    mine = self.ctx.layer_counts(E)
                    cur = B.moe_pending_experts(mine, self.resident[l], in_slot)
                    plan = B.moe_presched(costs, cur, cand)
                    chosen = list(plan.prefetch[:min(plan.n_prefetch, n_prefetch)])
                    self.sched_log["n_decisions"] += 1
                    self.sched_log["n_prefetch_planned"] += plan.n_prefetch
                    self.sched_log["f_sum"] += plan.f
                else:
                    raise ValueError(policy)
                pm = np.zeros(E, dtype=bool)
                pm[chosen] = True
                issued = B.moe_prefetch(self.ctx, self.shape, self.layers[nxt], pm)
                self._in_slot[nxt] = set(chosen)
                if st is not None:
                    st["n_prefetch_issued"] += issued
                    st["bytes_prefetch"] += issued * expert_bytes
            if st is not None:
                stats.append(st)
            x = out
        return x, stats


def noisy_topk_prefetch_mask(next_logits: np.ndarray, noise: np.ndarray, k: int, n_prefetch: int,
                             resident: Sequence[bool]) -> np.ndarray:
    """Harness-side stand-in for an expert predictor (not part of the block):
    rank the next layer's experts by how many tokens have them in the top-k of
    (true logits + noise) and pick the ``n_prefetch`` best non-resident ones
    that got any vote; ties go to the lower index."""
    noisy = np.asarray(next_logits, dtype=np.float64) + np.asarray(noise, dtype=np.float64)
    E = noisy.shape[1]
    order = np.argsort(-noisy, axis=1, kind="stable")[:, :k]
    votes = np.bincount(order.reshape(-1), minlength=E)
    ranked = sorted(range(E), key=lambda e: (-int(votes[e]), e))
    mask = np.zeros(E, dtype=bool)
    for e in ranked:
        if mask.sum() >= n_prefetch:
            break
        if not resident[e] and votes[e] > 0:
            mask[e] = True
    return mask
