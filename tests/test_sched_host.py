"""Host-only scheduling calls of the C-ABI (no GPU needed) against the
scheduling oracle: every field of the PreSched plan equal, doubles included
(both sides evaluate Eq. 2-6 in float64 in the same order), and the hot-expert
table equal entry by entry."""
import numpy as np
import pytest

import oracle.sched_oracle as S


@pytest.fixture(scope="module")
def B():
    import paper_2509_23638_amd.binding as b
    return b


def _costs(B, c: S.Costs):
    return B.moe_presched_costs(c.t_io, c.t_g, c.t_attn, c.beta, c.C, c.alpha, c.r_hit,
                                1 if c.cpu_executor else 0)


def _compare(B, cur, nxt, c):
    ref = S.presched(cur, nxt, c)
    got = B.moe_presched(_costs(B, c), cur, nxt)
    assert (got.n_cur, got.n_next, got.n_all) == (len(cur), len(nxt), len(cur) + len(nxt))
    assert list(got.cur_sorted[:got.n_cur]) == [e for e, _ in ref.E_cur]
    assert list(got.next_sorted[:got.n_next]) == [e for e, _ in ref.E_next]
    assert list(zip(got.all_layer[:got.n_all], got.all_expert[:got.n_all])) == \
        [(l, e) for l, e, _ in ref.E_all]
    assert [bool(q) for q in got.all_in_queue[:got.n_all]] == ref.gpu_q
    assert got.i_prime == ref.i_prime
    assert list(got.ondemand[:got.n_ondemand]) == ref.ondemand
    assert (got.T_gap, got.f, got.f_abs, got.xi) == (ref.T_gap, ref.f, ref.f_abs, ref.xi)
    assert list(got.prefetch[:got.n_prefetch]) == ref.prefetch
    return got


def test_presched_worked_timeline(B):
    c = S.Costs(t_io=10, t_g=1, t_attn=5, beta=1, C=2, alpha=0, r_hit=0.8)
    got = _compare(B, [(7, 1), (3, 2), (5, 8), (1, 20)], [(4, 3), (9, 15)], c)
    assert list(got.ondemand[:got.n_ondemand]) == [1] and list(got.prefetch[:got.n_prefetch]) == [9]


@pytest.mark.parametrize("cpu_executor", [True, False])
def test_presched_random_cases(B, cpu_executor):
    r = np.random.Generator(np.random.PCG64(21 + cpu_executor))
    for trial in range(600):
        n_cur, n_next = int(r.integers(0, 9)), int(r.integers(0, 9))
        if trial % 50 == 0:
            n_cur, n_next = 128, 128                      # the documented maximum
        ids = r.permutation(128)
        few = trial % 3 == 0                              # many equal counts
        hi = 4 if few else 60
        cur = [(int(ids[i]), int(r.integers(0, hi))) for i in range(n_cur)]
        nxt = [(int(ids[-1 - i]), int(r.integers(0, hi))) for i in range(n_next)]
        c = S.Costs(t_io=float(r.uniform(0.5, 20)), t_g=float(r.uniform(0, 3)),
                    t_attn=float(r.uniform(0, 60)), beta=float(r.uniform(0, 2)),
                    C=float(r.uniform(0, 3)), alpha=float(r.uniform(0, 5)),
                    r_hit=float(r.uniform(0, 1)), cpu_executor=cpu_executor)
        if trial % 7 == 0:
            c.r_hit = float(r.integers(0, 2))
        _compare(B, cur, nxt, c)


def test_presched_rejects_bad_arguments(B):
    ok = S.Costs(t_io=1, t_g=1, t_attn=1)
    for bad in (S.Costs(t_io=0, t_g=1, t_attn=1), S.Costs(t_io=1, t_g=1, t_attn=1, r_hit=1.5)):
        with pytest.raises(B.MoEError):
            B.moe_presched(_costs(B, bad), [(0, 1)], [])
    with pytest.raises(B.MoEError):
        B.moe_presched(_costs(B, ok), [(0, -1)], [])
    with pytest.raises(B.MoEError):
        B.moe_presched(_costs(B, ok), [(i, 1) for i in range(129)], [])
    assert "moe_presched" in B.moe_last_error()


def test_hot_table_matches_oracle(B):
    r = np.random.Generator(np.random.PCG64(23))
    for trial in range(200):
        L, E = int(r.integers(1, 40)), int(r.integers(1, 130))
        hi = 3 if trial % 2 else 10 ** 6
        tok = r.integers(0, hi, size=(L, E))
        for budget in (0, 1, int(r.integers(0, L * E + 1)), L * E, L * E + 5, -3):
            assert np.array_equal(B.moe_hot_table(tok, budget), S.hot_expert_table(tok, budget))
    with pytest.raises(B.MoEError):
        B.moe_hot_table(np.zeros((0, 4), dtype=np.int64), 1)


def test_pending_list_and_fixed_count_policy_match_oracle(B):
    r = np.random.Generator(np.random.PCG64(29))
    for trial in range(400):
        E = int(r.integers(1, 129)) if trial % 20 else 128
        hi = 3 if trial % 2 else 500
        counts = r.integers(0, hi, size=E).tolist()
        res = (r.random(E) < 0.4).tolist()
        fly = (r.random(E) < 0.2).tolist() if trial % 3 else None
        pend = B.moe_pending_experts(counts, res, fly)
        assert pend == S.pending_experts(counts, res, fly)
        for n in (0, 1, 2, int(r.integers(0, E + 3))):
            assert B.moe_prefetch_hottest(pend, n) == S.prefetch_hottest(pend, n)
    assert B.moe_pending_experts([3, 0, 4], None, None) == [(0, 3), (2, 4)]
    with pytest.raises(B.MoEError):
        B.moe_pending_experts([1, -2], [False, False])
    with pytest.raises(B.MoEError):
        B.moe_prefetch_hottest([(i, 1) for i in range(129)], 2)
