"""Plain CPU oracle of the scheduling-side logic.  TEST INFRASTRUCTURE ONLY.

Three pieces, each written out from the paper's equations in its notation:

  * the hot-expert table (Section 4.1): a counter of tokens processed per
    (layer, expert) ranks the experts; the hottest are made resident, in
    descending order, until the memory budget is used up;
  * a gate-based expert predictor (the strategy Section 3.2 attributes to
    earlier work and Figure 6 compares): the NEXT layer's router applied to the
    CURRENT layer's input, its top-k counted per expert;
  * PreSched (Section 4.3): the cross-layer queue of Q1 (Eq. 3), the local
    recheck (Eq. 4), the prefetch count of Q2 (Eq. 5), the critical-prefetch
    benefit of Q3 (Eq. 6), the no-benefit exit of Q4, with the CPU cost model of Eq. 2.

Readings taken where the paper is silent or at odds with itself:
  * experts with equal token counts are ordered by ascending expert index; in
    the merged list a next-layer expert sorts below a current-layer expert
    with the same count (the current layer's need is certain);
  * the queue condition of Q1 is evaluated index by index as in Algorithm 1;
    both costs are monotone in the index, so the queue is a suffix of E_all;
  * the recheck returns the smallest index i' of E_cur that is in the queue and
    has T_G(i') < T_C(i'); when no index qualifies nothing is loaded on demand
    (i' = n + 1), although Algorithm 1 initialises its load cursor to n;
  * |f| is f rounded half up, clamped to [0, n'];
  * the selected prefetches E_next[n'-c .. n'-1] are issued hottest first, as
    the text of Q3 says (Algorithm 1's loop runs the other way);
  * without a CPU executor (the GPU-only form this repository runs) no expert
    may stay on the host: the queue is all of E_all and i' = 0.  Eq. 4's T_C
    is then an empty sum, so T_gap = -alpha - (n+1) t_io and only t_attn (the
    time per layer in which the link has no on-demand work) opens a window.

Pins (tests/test_sched_pins.py): pending lists and the fixed-count policy by hand
and against the block oracle's separately written prefetch-set routine; two
timelines worked by hand, the min-max
property of the recheck against a brute-force search, suffix/monotonicity
invariants, degenerate cost models with known answers, brute-force ranking for
the hot table, and the predictor against the block oracle's own routing.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

from . import moe_oracle as _block


# --------------------------------------------------------- hot-expert table
def hot_expert_table(tokens_processed: np.ndarray, budget_experts: int) -> np.ndarray:
    """tokens_processed [L, E] (the Counter's totals) -> resident mask [L, E].

    Section 4.1: rank all experts by tokens processed and load the hottest in
    descending order until the budget (here: a number of equally sized experts)
    is exhausted.  Equal counts: lower layer first, then lower expert index."""
    c = np.asarray(tokens_processed)
    L, E = c.shape
    ranked = sorted(((int(c[l, e]), l, e) for l in range(L) for e in range(E)),
                    key=lambda r: (-r[0], r[1], r[2]))
    mask = np.zeros((L, E), dtype=bool)
    for _, l, e in ranked[:max(0, int(budget_experts))]:
        mask[l, e] = True
    return mask


# ------------------------------------------------------ gate-based predictor
def gate_based_counts(X_cur, Wr_next, b_next, k: int) -> np.ndarray:
    """Predicted pending tokens per expert of the next layer: route the current
    layer's input with the next layer's router (Section 3.2, gate-based
    strategy) and count each expert's appearances in the top-k lists."""
    idx, _, _ = _block.route(X_cur, Wr_next, b_next, k)
    E = np.asarray(Wr_next).shape[0]
    return np.bincount(idx.reshape(-1), minlength=E).astype(np.int64)


# ------------------------------------------- pending experts, fixed-count policy
def pending_experts(counts: Sequence[int], resident: Sequence[bool],
                    in_flight: Sequence[bool] = None) -> List[Tuple[int, int]]:
    """Premise 1 of Section 4.3.2: the experts a scheduling decision ranges
    over are those that are activated (or predicted) and neither on the GPU
    nor being loaded.  Returns (expert, tokens) by ascending expert id."""
    out = []
    for e, m in enumerate(counts):
        if m > 0 and not resident[e] and not (in_flight is not None and in_flight[e]):
            out.append((e, int(m)))
    return out


def prefetch_hottest(pending: Sequence[Tuple[int, int]], n_prefetch: int) -> List[int]:
    """The fixed-count policy Section 5.3's ablation uses in place of PreSched:
    take the n_prefetch pending experts with the most tokens, hottest first.
    Reading: equal counts go to the lower expert id."""
    chosen = []
    left = list(pending)
    while left and len(chosen) < n_prefetch:
        best = left[0]
        for cand in left[1:]:
            if cand[1] > best[1] or (cand[1] == best[1] and cand[0] < best[0]):
                best = cand
        chosen.append(best[0])
        left.remove(best)
    return chosen


# ------------------------------------------------------------------ PreSched
@dataclass
class Costs:
    t_io: float          # load time of one expert (fixed, Section 4.3.2)
    t_g: float           # GPU compute time of one expert (token-invariant)
    t_attn: float        # attention time of a layer
    beta: float = 0.0    # CPU cost per token        (Eq. 2)
    C: float = 0.0       # CPU start-up cost         (Eq. 2)
    alpha: float = 0.0   # delay of the first on-demand load behind a prefetch
    r_hit: float = 1.0   # hit rate of the critical prefetch; r_miss = 1 - r_hit
    cpu_executor: bool = True


@dataclass
class Plan:
    E_cur: List[Tuple[int, int]] = field(default_factory=list)    # (expert, tokens) ascending
    E_next: List[Tuple[int, int]] = field(default_factory=list)
    E_all: List[Tuple[int, int, int]] = field(default_factory=list)  # (layer 0/1, expert, tokens)
    gpu_q: List[bool] = field(default_factory=list)               # per E_all index
    i_prime: int = 0
    ondemand: List[int] = field(default_factory=list)             # expert ids, load order
    T_gap: float = 0.0
    f: float = 0.0
    f_abs: int = 0
    xi: float = 0.0
    prefetch: List[int] = field(default_factory=list)             # expert ids, issue order


def t_c(tokens: Sequence[int], costs: Costs) -> float:
    """Eq. 2 summed over a list of experts: sum_j (beta * m_j + C)."""
    return float(sum(costs.beta * m + costs.C for m in tokens))


def presched(cur: Sequence[Tuple[int, int]], nxt: Sequence[Tuple[int, int]], costs: Costs) -> Plan:
    """One scheduling decision for a layer.

    cur / nxt: (expert id, pending tokens) of the current layer's activated and
    the next layer's predicted experts, those already on the GPU or being
    loaded excluded (Premise 1)."""
    p = Plan()
    # Premise 1: ascending pending tokens; merged list by cross-layer ordering
    p.E_cur = sorted(cur, key=lambda r: (r[1], r[0]))
    p.E_next = sorted(nxt, key=lambda r: (r[1], r[0]))
    merged = [(0, e, m) for e, m in p.E_cur] + [(1, e, m) for e, m in p.E_next]
    p.E_all = sorted(merged, key=lambda r: (r[2], -r[0], r[1]))
    n = len(p.E_cur) - 1
    n_ = len(p.E_next)
    a, t_io, t_g = costs.alpha, costs.t_io, costs.t_g

    # Q1 (Eq. 3): E_all[i] belongs on the GPU when loading E_all[i..n+n'] and one
    # GPU computation is cheaper than computing E_all[0..i] on the CPU
    for i in range(len(p.E_all)):
        if costs.cpu_executor:
            TG_all = a + (n + n_ - i + 1) * t_io + t_g
            TC_all = t_c([m for _, _, m in p.E_all[:i + 1]], costs) + costs.t_attn
            p.gpu_q.append(TG_all < TC_all)
        else:
            p.gpu_q.append(True)

    # local recheck (Eq. 4) over the queue's current-layer members, coldest first
    p.i_prime = n + 1
    in_q = {(lay, e) for (lay, e, _), q in zip(p.E_all, p.gpu_q) if q}
    if not costs.cpu_executor:
        p.i_prime = 0
    else:
        for i_ in range(n + 1):
            if (0, p.E_cur[i_][0]) not in in_q:
                continue
            T_G = a + (n - i_ + 1) * t_io + t_g
            T_C = t_c([m for _, m in p.E_cur[:i_]], costs)
            if T_G < T_C:
                p.i_prime = i_
                break
    p.ondemand = [e for e, _ in p.E_cur[p.i_prime:]]

    # Q2 (Eq. 5): the window the current layer leaves on the link, in units of one load
    p.T_gap = t_c([m for _, m in p.E_cur[:p.i_prime]], costs) - a - (n - p.i_prime + 1) * t_io
    p.f = (p.T_gap + costs.t_attn) / t_io
    p.f_abs = min(max(int(math.floor(p.f + 0.5)), 0), n_)

    # Q3 (Eq. 6): expected benefit of the critical (last) prefetch
    r_miss = 1.0 - costs.r_hit
    p.xi = costs.r_hit * (p.f - p.f_abs + 1) * t_io - r_miss * (p.f_abs - p.f) * t_io

    # Q4: nothing of the next layer is wanted on the GPU -> no prefetch
    if not any(q and lay == 1 for (lay, _, _), q in zip(p.E_all, p.gpu_q)):
        return p
    if costs.r_hit * (p.f - p.f_abs + 1) > r_miss * (p.f_abs - p.f):
        c = p.f_abs
    else:
        c = p.f_abs - 1
    c = max(c, 0)
    p.prefetch = [e for e, _ in reversed(p.E_next[n_ - c:])] if c > 0 else []
    return p
