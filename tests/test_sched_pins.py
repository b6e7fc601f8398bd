"""Pins of the scheduling oracle (hot-expert table, gate-based predictor,
PreSched) against hand-worked timelines, properties the equations imply, and
brute force.  Each check is a plain function so the mutation tests at the
bottom can re-run it with a mistake planted in the oracle (CPU only).
"""
import itertools

import numpy as np
import pytest

import oracle.sched_oracle as S
from oracle.sched_oracle import Costs


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ----------------------------------------------------------- PreSched -----
def check_timeline_a():
    """Worked by hand (Section 4.3.3, Q1-Q3).  t_io 10, t_g 1, t_attn 5,
    t_c(m) = m + 2, alpha 0.  Current layer: experts 7,3,5,1 with 1,2,8,20
    pending tokens (n = 3); predicted next layer: experts 4,9 with 3,15 (n' = 2).
      E_all tokens        1    2    3    8   15   20     (index 0..5)
      T^G_all = (6-i)10+1 61   51   41   31  21   11
      t_c                 3    4    5    10  17   22
      T^C_all = cum + 5   8    12   17   27  44   66
    so the queue is E_all[4..5] = {next:9, cur:1}.  Recheck of cur index 3:
    T_G = 1*10 + 1 = 11 < T_C = 3 + 4 + 10 = 17, so i' = 3 and expert 1 loads.
    T_gap = 17 - 0 - 10 = 7, f = (7 + 5)/10 = 1.2, |f| = 1 (rounded down, so the
    critical prefetch costs nothing): prefetch E_next[1] = expert 9.
    xi = 0.8 * 1.2 * 10 - 0.2 * (-0.2) * 10 = 10.0."""
    c = Costs(t_io=10, t_g=1, t_attn=5, beta=1, C=2, alpha=0, r_hit=0.8)
    p = S.presched([(7, 1), (3, 2), (5, 8), (1, 20)], [(4, 3), (9, 15)], c)
    assert [e for e, _ in p.E_cur] == [7, 3, 5, 1]
    assert [(l, e) for l, e, _ in p.E_all] == [(0, 7), (0, 3), (1, 4), (0, 5), (1, 9), (0, 1)]
    assert p.gpu_q == [False, False, False, False, True, True]
    assert p.i_prime == 3 and p.ondemand == [1]
    assert p.T_gap == 7 and abs(p.f - 1.2) < 1e-15 and p.f_abs == 1
    assert abs(p.xi - 10.0) < 1e-12
    assert p.prefetch == [9]


def check_timeline_b():
    """Same lists, t_attn 9 and alpha 0: T^C_all = 12 16 21 31 48 70, the queue
    is still E_all[4..5]; f = (7 + 9)/10 = 1.6, |f| = 2 (rounded up by 0.4).
    Critical prefetch: gain r_hit * 0.6, loss r_miss * 0.4.
      r_hit 0.3: 0.18 < 0.28 -> |f| - 1 = 1 prefetch  (expert 9), xi = 1.8 - 2.8 = -1.0
      r_hit 0.5: 0.30 > 0.20 -> 2 prefetches, hottest first (9 then 4), xi = 3 - 2 = 1.0
    With alpha = 4: T_gap = 3, f = 1.2, |f| = 1 -> one prefetch whatever r_hit is."""
    cur, nxt = [(7, 1), (3, 2), (5, 8), (1, 20)], [(4, 3), (9, 15)]
    p = S.presched(cur, nxt, Costs(10, 1, 9, 1, 2, 0, 0.3))
    assert p.gpu_q == [False, False, False, False, True, True]
    assert abs(p.f - 1.6) < 1e-15 and p.f_abs == 2 and abs(p.xi + 1.0) < 1e-12
    assert p.prefetch == [9]
    p = S.presched(cur, nxt, Costs(10, 1, 9, 1, 2, 0, 0.5))
    assert p.f_abs == 2 and abs(p.xi - 1.0) < 1e-12 and p.prefetch == [9, 4]
    p = S.presched(cur, nxt, Costs(10, 1, 9, 1, 2, 4, 0.01))
    # alpha also raises T_G of the recheck to 4 + 10 + 1 = 15 < 17: still i' = 3
    assert p.i_prime == 3 and abs(p.f - 1.2) < 1e-15 and p.prefetch == [9]


def _random_case(r, n_cur=None, n_next=None):
    n_cur = int(r.integers(0, 7)) if n_cur is None else n_cur
    n_next = int(r.integers(0, 6)) if n_next is None else n_next
    ids = r.permutation(32)
    cur = [(int(ids[i]), int(r.integers(1, 40))) for i in range(n_cur)]
    nxt = [(int(ids[16 + i]), int(r.integers(1, 40))) for i in range(n_next)]
    c = Costs(t_io=float(r.uniform(1, 20)), t_g=float(r.uniform(0.1, 3)),
              t_attn=float(r.uniform(0, 30)), beta=float(r.uniform(0.05, 2)),
              C=float(r.uniform(0, 3)), alpha=float(r.uniform(0, 5)),
              r_hit=float(r.uniform(0, 1)))
    return cur, nxt, c


def check_recheck_balances_cpu_and_gpu():
    """Eq. 4 against a timeline played out event by event: loads run one after
    another on the link from time alpha (Premise 4), only the last loaded
    expert's computation is not hidden behind I/O (Premise 5), the CPU works
    through the experts left to it one by one (Eq. 2).  i' is the first split
    at which the GPU side finishes strictly earlier; and since one side falls
    and the other rises with the split point, the brute-force minimiser of the
    layer latency max(GPU, CPU) is i' or i' - 1.  (t_attn huge puts every
    expert in the queue, so the queue does not restrict the search.)"""
    r = _rng(11)
    for _ in range(400):
        cur, nxt, c = _random_case(r, n_cur=int(r.integers(1, 8)))
        c.t_attn = 1e9
        p = S.presched(cur, nxt, c)
        assert all(p.gpu_q)
        m = [t for _, t in p.E_cur]
        n = len(m) - 1

        def finish(i):           # E_cur[i..n] loaded, E_cur[0..i-1] on the CPU
            clock = c.alpha
            for _ in m[i:]:
                clock += c.t_io
            gpu = clock + c.t_g if i <= n else 0.0
            cpu = 0.0
            for tokens in m[:i]:
                cpu += c.beta * tokens + c.C
            return gpu, cpu
        for i in range(n + 1):
            gpu, cpu = finish(i)
            assert (gpu < cpu) == (i >= p.i_prime), (i, p.i_prime, gpu, cpu)
        best = min(range(n + 2), key=lambda i: (max(finish(i)), i))
        assert best in (p.i_prime - 1, p.i_prime), (best, p.i_prime)


def check_structure_invariants():
    r = _rng(12)
    for _ in range(400):
        cur, nxt, c = _random_case(r)
        p = S.presched(cur, nxt, c)
        # sorted ascending by tokens; merged list is a permutation of both
        assert [t for _, t in p.E_cur] == sorted(t for _, t in cur)
        assert [t for _, _, t in p.E_all] == sorted([t for _, t in cur] + [t for _, t in nxt])
        # the queue is a suffix of E_all (both costs are monotone in the index)
        q = p.gpu_q
        assert q == sorted(q)
        # Premise 2: the on-demand set is a suffix of E_cur, inside the queue
        assert p.ondemand == [e for e, _ in p.E_cur[p.i_prime:]]
        in_q = {(l, e) for (l, e, _), f in zip(p.E_all, q) if f}
        assert all((0, e) in in_q for e in p.ondemand)
        # with a CPU executor the coldest expert never loads: T_C of an empty prefix is 0
        assert p.i_prime >= 1 or not cur
        # prefetches: the hottest of E_next, hottest first, |f| or |f| - 1 of them, or none (Q4)
        hot_first = [e for e, _ in reversed(p.E_next)]
        assert p.prefetch == hot_first[:len(p.prefetch)]
        if any(f and l == 1 for (l, _, _), f in zip(p.E_all, q)):
            assert len(p.prefetch) in (p.f_abs, max(p.f_abs - 1, 0))
            if p.f_abs - p.f <= 0 and p.f - p.f_abs + 1 > 0 and c.r_hit > 0:
                assert len(p.prefetch) == p.f_abs      # rounded down: no cost side
        else:
            assert p.prefetch == []
        assert 0 <= p.f_abs <= len(nxt) and abs(p.f_abs - p.f) <= 0.5 or p.f_abs in (0, len(nxt))


def check_units_and_shifts():
    """Decisions depend on ratios of times only; alpha moves f by -alpha/t_io;
    t_attn moves f by +t_attn/t_io (Eq. 5)."""
    r = _rng(13)
    for _ in range(200):
        cur, nxt, c = _random_case(r)
        p = S.presched(cur, nxt, c)
        s = 8.0          # a power of two keeps every product exact
        c2 = Costs(c.t_io * s, c.t_g * s, c.t_attn * s, c.beta * s, c.C * s, c.alpha * s, c.r_hit)
        p2 = S.presched(cur, nxt, c2)
        assert (p2.gpu_q, p2.i_prime, p2.ondemand, p2.f_abs, p2.prefetch) == \
               (p.gpu_q, p.i_prime, p.ondemand, p.f_abs, p.prefetch)
        assert p2.f == p.f and p2.xi == p.xi * s and p2.T_gap == p.T_gap * s
        # same split point => f moves linearly
        c3 = Costs(c.t_io, c.t_g, c.t_attn, c.beta, c.C, c.alpha, c.r_hit, cpu_executor=False)
        c4 = Costs(c.t_io, c.t_g, c.t_attn + 3 * c.t_io, c.beta, c.C, c.alpha + c.t_io, c.r_hit,
                   cpu_executor=False)
        assert abs(S.presched(cur, nxt, c4).f - (S.presched(cur, nxt, c3).f + 2.0)) < 1e-9


def check_degenerate_cost_models():
    cur, nxt = [(0, 5), (1, 9), (2, 30)], [(3, 4), (4, 50)]
    # a free CPU (beta = C = 0) and attention shorter than one load: nothing is
    # worth moving, nothing is prefetched (Q4)
    p = S.presched(cur, nxt, Costs(t_io=10, t_g=1, t_attn=5, beta=0, C=0))
    assert p.gpu_q == [False] * 5 and p.ondemand == [] and p.prefetch == [] and p.i_prime == 3
    # T_gap = 0 - 0 - 0: f = 5/10 rounds half up to 1 but Q4 has already returned
    assert p.f == 0.5 and p.f_abs == 1
    # a hopeless CPU: everything queues, everything but the coldest loads
    p = S.presched(cur, nxt, Costs(t_io=10, t_g=1, t_attn=5, beta=1e9, C=0))
    assert all(p.gpu_q) and p.i_prime == 1 and p.ondemand == [1, 2]
    # empty lists
    p = S.presched([], [], Costs(t_io=10, t_g=1, t_attn=25))
    assert p.ondemand == [] and p.prefetch == [] and p.f == 2.5 and p.f_abs == 0
    p = S.presched([], nxt, Costs(t_io=10, t_g=1, t_attn=25, beta=1, C=0))
    # n = -1: T^G_all(i) = (2 - i)10 + 1 = 21, 11;  T^C_all = 4 + 25, 54 + 25: both queue
    assert p.gpu_q == [True, True] and p.f == 2.5 and p.f_abs == 2 and p.prefetch == [4, 3]


def check_gpu_only_form():
    """No CPU executor: every pending expert of the current layer loads, in
    ascending order of pending tokens; T_gap = -alpha - (n+1) t_io."""
    cur, nxt = [(6, 9), (2, 1), (5, 4)], [(1, 7), (0, 7), (3, 2)]
    c = Costs(t_io=4, t_g=1, t_attn=3 * 4 + 2 + 2.4 * 4, alpha=2, r_hit=0.9, cpu_executor=False)
    p = S.presched(cur, nxt, c)
    assert all(p.gpu_q) and p.i_prime == 0 and p.ondemand == [2, 5, 6]
    assert p.T_gap == -2 - 3 * 4 and abs(p.f - 2.4) < 1e-12 and p.f_abs == 2
    # equal counts: ascending expert index, so expert 1 is the hotter of the tie
    assert [e for e, _ in p.E_next] == [3, 0, 1] and p.prefetch == [1, 0]
    # link-bound layer: the window is negative, nothing is prefetched
    p = S.presched(cur, nxt, Costs(t_io=4, t_g=1, t_attn=0.5, cpu_executor=False))
    assert p.f < 0 and p.f_abs == 0 and p.prefetch == []


def check_cross_layer_tie_order():
    # equal token counts across layers: the next-layer expert sorts lower
    p = S.presched([(3, 5)], [(3, 5)], Costs(t_io=1, t_g=0.1, t_attn=100, beta=1))
    assert [(l, e) for l, e, _ in p.E_all] == [(1, 3), (0, 3)]


# ------------------------------------------------------ hot-expert table ---
def check_hot_table_by_hand_and_bruteforce():
    c = np.array([[5, 9, 0, 9],
                  [9, 1, 7, 2]])
    # ranking: 9 (l0,e1) 9 (l0,e3) 9 (l1,e0) 7 (l1,e2) 5 (l0,e0) 2 1 0
    assert S.hot_expert_table(c, 0).sum() == 0
    assert S.hot_expert_table(c, 2).tolist() == [[False, True, False, True], [False] * 4]
    assert S.hot_expert_table(c, 4).tolist() == [[False, True, False, True], [True, False, True, False]]
    assert S.hot_expert_table(c, 99).all()
    r = _rng(14)
    for _ in range(50):
        L, E = int(r.integers(1, 4)), int(r.integers(1, 5))
        c = r.integers(0, 6, size=(L, E))
        B = int(r.integers(0, L * E + 1))
        m = S.hot_expert_table(c, B)
        assert m.sum() == B
        # no other choice of B experts covers more tokens
        flat = c.reshape(-1)
        best = max(sum(flat[list(s)]) for s in itertools.combinations(range(L * E), B))
        assert c[m].sum() == best
        # among equals the earlier (layer, expert) wins
        if B and B < L * E:
            cut = c[m].min()
            tied_in = [i for i in range(L * E) if flat[i] == cut and m.reshape(-1)[i]]
            tied_out = [i for i in range(L * E) if flat[i] == cut and not m.reshape(-1)[i]]
            assert not tied_in or not tied_out or max(tied_in) < min(tied_out)


# ------------------------------------------------------ gate-based counts ---
def check_gate_based_counts_by_inspection():
    """Unit-vector inputs read single columns of the next layer's router, so
    the top-2 lists can be read off the matrix."""
    Wr = np.array([[3, 0, 1],
                   [2, 5, 1],
                   [1, 4, 1],
                   [0, 9, 0]], dtype=np.float32)          # [E=4, H=3]
    b = np.array([0, 0, 0.5, 0], dtype=np.float32)
    X = np.eye(3, dtype=np.float32)[[0, 1, 2, 1]]          # tokens read columns 0,1,2,1
    # column 0: 3,2,1.5,0 -> {0,1}; column 1: 0,5,4.5,9 -> {3,1} (twice); column 2: 1,1,1.5,0 -> {2,0}
    assert S.gate_based_counts(X, Wr, b, 2).tolist() == [2, 3, 1, 2]
    assert S.gate_based_counts(X, Wr, b, 1).tolist() == [1, 0, 1, 2]
    assert S.gate_based_counts(X[:0], Wr, b, 2).tolist() == [0, 0, 0, 0]


# -------------------------------------- pending list and fixed-count policy ---
def check_pending_and_hottest_by_hand():
    counts = [5, 0, 7, 7, 2, 9, 1, 7]
    resident = [False, False, False, True, False, True, False, False]
    in_flight = [False, False, False, False, True, False, False, False]
    # expert 1 has no tokens, 3 and 5 are resident, 4 is being loaded
    assert S.pending_experts(counts, resident) == [(0, 5), (2, 7), (4, 2), (6, 1), (7, 7)]
    pend = S.pending_experts(counts, resident, in_flight)
    assert pend == [(0, 5), (2, 7), (6, 1), (7, 7)]
    # hottest first; 2 and 7 tie on 7 tokens: the lower id goes first
    assert S.prefetch_hottest(pend, 1) == [2]
    assert S.prefetch_hottest(pend, 2) == [2, 7]
    assert S.prefetch_hottest(pend, 3) == [2, 7, 0]
    assert S.prefetch_hottest(pend, 9) == [2, 7, 0, 6]
    assert S.prefetch_hottest(pend, 0) == [] and S.prefetch_hottest([], 2) == []
    # input order must not matter
    assert S.prefetch_hottest(list(reversed(pend)), 3) == [2, 7, 0]


def check_hottest_against_block_oracle_prefetch_set():
    """oracle/moe_oracle.py states the same policy in its own words for the
    benchmark's predictor stand-in (votes of the noisy top-k, best non-resident
    experts with any vote, ties to the lower index); with zero noise the two
    separately written routines must choose the same set."""
    import oracle.moe_oracle as O
    r = np.random.Generator(np.random.PCG64(50))
    for trial in range(60):
        E, T = int(r.integers(3, 24)), int(r.integers(1, 20))
        k = int(r.integers(1, min(E, 5) + 1))
        n = int(r.integers(0, 5))
        lg = r.integers(-3, 4, size=(T, E)).astype(np.float64)      # many ties
        res = r.random(E) < 0.4
        want = O.predicted_prefetch_set(lg, np.zeros_like(lg), k, n, res)
        votes = np.zeros(E, dtype=np.int64)
        for t in range(T):
            for e in O.select_topk(lg[t], k):
                votes[e] += 1
        got = np.zeros(E, dtype=bool)
        got[S.prefetch_hottest(S.pending_experts(votes, res), n)] = True
        assert np.array_equal(got, want)


CHECKS = [v for k, v in sorted(globals().items()) if k.startswith("check_")]


@pytest.mark.parametrize("check", CHECKS, ids=lambda c: c.__name__)
def test_pin(check):
    check()


# ------------------------------------------------------------ mutations ----
def _mutant_presched(edit):
    """The oracle's source with one textual edit, compiled into a fresh module."""
    import inspect, sys, types
    src = inspect.getsource(S)
    old, new = edit
    assert src.count(old) == 1, old
    mod = types.ModuleType("oracle.sched_mutant")
    mod.__package__ = "oracle"
    sys.modules[mod.__name__] = mod        # dataclasses look their module up by name
    try:
        exec(compile(src.replace(old, new), "sched_mutant", "exec"), mod.__dict__)
    finally:
        del sys.modules[mod.__name__]
    return mod


MUTANTS = [
    ("queue_counts_one_load_less", ("(n + n_ - i + 1) * t_io + t_g", "(n + n_ - i) * t_io + t_g"),
     [check_timeline_b, check_degenerate_cost_models]),
    ("queue_forgets_attention", ("costs) + costs.t_attn", "costs)"), [check_degenerate_cost_models]),
    ("recheck_includes_own_cost", ("p.E_cur[:i_]], costs)", "p.E_cur[:i_ + 1]], costs)"),
     [check_recheck_balances_cpu_and_gpu, check_degenerate_cost_models]),
    ("recheck_forgets_compute", ("T_G = a + (n - i_ + 1) * t_io + t_g", "T_G = a + (n - i_ + 1) * t_io"),
     [check_recheck_balances_cpu_and_gpu]),
    ("gap_forgets_alpha", ("costs) - a - (n - p.i_prime + 1) * t_io", "costs) - (n - p.i_prime + 1) * t_io"),
     [check_timeline_b, check_units_and_shifts, check_gpu_only_form]),
    ("gap_sign_of_loads", ("- a - (n - p.i_prime + 1) * t_io", "- a + (n - p.i_prime + 1) * t_io"),
     [check_timeline_a, check_gpu_only_form]),
    ("f_forgets_attention", ("p.f = (p.T_gap + costs.t_attn) / t_io", "p.f = p.T_gap / t_io"),
     [check_timeline_a, check_units_and_shifts]),
    ("f_truncates", ("math.floor(p.f + 0.5)", "math.floor(p.f)"), [check_timeline_b]),
    ("critical_rule_swapped", ("if costs.r_hit * (p.f - p.f_abs + 1) > r_miss * (p.f_abs - p.f):",
                               "if costs.r_hit * (p.f - p.f_abs + 1) < r_miss * (p.f_abs - p.f):"),
     [check_timeline_a, check_timeline_b]),
    ("xi_sign", ("* t_io - r_miss * (p.f_abs - p.f) * t_io", "* t_io + r_miss * (p.f_abs - p.f) * t_io"),
     [check_timeline_b]),
    ("prefetch_coldest", ("reversed(p.E_next[n_ - c:])", "reversed(p.E_next[:c])"),
     [check_timeline_a, check_structure_invariants]),
    ("prefetch_order_ascending", ("[e for e, _ in reversed(p.E_next[n_ - c:])]", "[e for e, _ in p.E_next[n_ - c:]]"),
     [check_timeline_b, check_gpu_only_form]),
    ("sort_descending", ("p.E_cur = sorted(cur, key=lambda r: (r[1], r[0]))",
                         "p.E_cur = sorted(cur, key=lambda r: (-r[1], r[0]))"),
     [check_timeline_a, check_structure_invariants]),
    ("cross_layer_tie", ("key=lambda r: (r[2], -r[0], r[1])", "key=lambda r: (r[2], r[0], r[1])"),
     [check_cross_layer_tie_order]),
    ("hot_table_coldest", ("key=lambda r: (-r[0], r[1], r[2])", "key=lambda r: (r[0], r[1], r[2])"),
     [check_hot_table_by_hand_and_bruteforce]),
    ("hot_table_tie_order", ("key=lambda r: (-r[0], r[1], r[2])", "key=lambda r: (-r[0], -r[1], r[2])"),
     [check_hot_table_by_hand_and_bruteforce]),
    ("pending_keeps_resident", ("if m > 0 and not resident[e] and not (", "if m > 0 and not ("),
     [check_pending_and_hottest_by_hand, check_hottest_against_block_oracle_prefetch_set]),
    ("pending_keeps_idle", ("if m > 0 and not resident[e]", "if m >= 0 and not resident[e]"),
     [check_pending_and_hottest_by_hand, check_hottest_against_block_oracle_prefetch_set]),
    ("pending_ignores_in_flight", ("and not (in_flight is not None and in_flight[e])", ""),
     [check_pending_and_hottest_by_hand]),
    ("hottest_takes_coldest", ("if cand[1] > best[1] or (cand[1] == best[1] and cand[0] < best[0]):",
                               "if cand[1] < best[1] or (cand[1] == best[1] and cand[0] < best[0]):"),
     [check_pending_and_hottest_by_hand, check_hottest_against_block_oracle_prefetch_set]),
    ("hottest_tie_to_higher_id", ("(cand[1] == best[1] and cand[0] < best[0])",
                                  "(cand[1] == best[1] and cand[0] > best[0])"),
     [check_pending_and_hottest_by_hand, check_hottest_against_block_oracle_prefetch_set]),
    ("counts_own_layer_k", ("_block.route(X_cur, Wr_next, b_next, k)", "_block.route(X_cur, Wr_next, None, k)"),
     [check_gate_based_counts_by_inspection]),
]


@pytest.mark.parametrize("name,edit,checks", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, name, edit, checks):
    """A mistake planted in the oracle (CPU only) must fail its pins."""
    mutant = _mutant_presched(edit)
    for fn in ("presched", "hot_expert_table", "gate_based_counts", "pending_experts", "prefetch_hottest"):
        monkeypatch.setattr(S, fn, getattr(mutant, fn))
    for check in checks:
        with pytest.raises(AssertionError):
            check()
