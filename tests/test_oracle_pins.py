"""Pins of the CPU oracle against things other than itself.

Each check is a plain function so that the mutation tests at the bottom can
re-run it with a mistake planted in the oracle (on the CPU) and see it fail.
Nothing here touches the GPU library.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle.moe_oracle as O
from workloads import get_config, make_layer, bf16_bits_from_f32

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ---------------------------------------------------------------- storage --
def check_widen_known_bits():
    bits = np.array([0x3F80, 0x4049, 0xC000, 0x0000, 0x3F81, 0x7F7F], dtype=np.uint16)
    want = [1.0, 3.140625, -2.0, 0.0, 1.0078125, 3.3895313892515355e38]
    got = O.widen(bits)
    assert got.dtype == np.float64
    assert got.tolist() == want
    f = np.array([0.1, -7.25], dtype=np.float32)
    assert O.widen(f).tolist() == [float(f[0]), -7.25]


def check_bf16_rounding():
    import torch
    r = _rng(5)
    a = np.concatenate([r.standard_normal(4096) * 10.0 ** r.integers(-6, 6, 4096),
                        [1.00390625, 1.01171875, -1.00390625, 0.0, 1.0, 3.0e38]])
    got = O.round_to_bf16_bits(a)
    # library conversion as an independent reference: float64 values that are
    # exactly float32 convert to bf16 with round-to-nearest-even in torch
    a32 = a.astype(np.float32)
    exact = a32.astype(np.float64) == a
    ref = torch.from_numpy(a32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got[exact], ref[exact])
    # hand-checked ties: 1 + 2^-8 is halfway between 1.0 (even) and 1 + 2^-7
    assert got[-6] == 0x3F80 and got[-5] == 0x3F82 and got[-4] == 0xBF80
    # every result is the nearest representable value
    back = O.widen(got)
    up = O.widen((got + 1).astype(np.uint16))
    dn = O.widen((got - 1).astype(np.uint16))
    fin = np.isfinite(up) & np.isfinite(dn)
    assert np.all(np.abs(back - a)[fin] <= np.abs(up - a)[fin])
    assert np.all(np.abs(back - a)[fin] <= np.abs(dn - a)[fin])
    # the input generator's float32 -> bf16 rounding agrees on float32 inputs
    assert np.array_equal(bf16_bits_from_f32(a32), O.round_to_bf16_bits(a32.astype(np.float64)))


# ------------------------------------------------------------------- gate --
def check_softmax_closed_form():
    # logits = ln(1..6)  =>  softmax = (1..6)/21 ; top-3 = experts 5,4,3 with
    # renormalised weights 6/15, 5/15, 4/15
    logit = np.log(np.arange(1.0, 7.0))
    idx = O.select_topk(logit, 3)
    assert idx.tolist() == [5, 4, 3]
    w = O.gate_weights(logit, idx)
    assert np.allclose(w, [6 / 15, 5 / 15, 4 / 15], rtol=0, atol=1e-15)
    # shift invariance, and no overflow for huge logits
    w2 = O.gate_weights(logit + 1000.0, idx)
    assert np.allclose(w2, w, rtol=0, atol=1e-13)
    # k = E keeps the plain softmax
    full = O.gate_weights(logit, O.select_topk(logit, 6))
    assert np.allclose(full, np.arange(6.0, 0.0, -1.0) / 21.0, rtol=0, atol=1e-15)


def check_weights_sum_and_order():
    r = _rng(1)
    for E, k in [(8, 2), (60, 4), (64, 6), (5, 5), (3, 1)]:
        lg = r.standard_normal((50, E)) * 3
        for t in range(50):
            idx = O.select_topk(lg[t], k)
            w = O.gate_weights(lg[t], idx)
            assert abs(w.sum() - 1.0) < 1e-12
            assert np.all(w > 0)
            assert np.all(np.diff(w) <= 0)
            # same thing as a softmax over just the selected logits
            z = [math.exp(lg[t, e] - lg[t, idx[0]]) for e in idx]
            assert np.allclose(w, np.array(z) / math.fsum(z), rtol=0, atol=1e-14)


def _brute_topk(logit, k):
    """All k-subsets; best = largest sum, then lexicographically smallest
    sorted index tuple; output ordered by (-logit, index)."""
    E = len(logit)
    best = None
    for sub in itertools.combinations(range(E), k):
        key = (-math.fsum(logit[e] for e in sub), sub)
        if best is None or key < best[0]:
            best = (key, sub)
    return sorted(best[1], key=lambda e: (-logit[e], e))


def check_topk_bruteforce():
    r = _rng(2)
    for E in range(1, 9):
        for k in range(1, E + 1):
            for trial in range(6):
                # small integers => many exact ties, sums exact
                lg = r.integers(-2, 3, size=E).astype(np.float64)
                assert O.select_topk(lg, k).tolist() == _brute_topk(lg, k)
            lg = r.standard_normal(E)
            assert O.select_topk(lg, k).tolist() == _brute_topk(lg, k)
    # all equal: indices 0..k-1 in order
    assert O.select_topk(np.zeros(8), 3).tolist() == [0, 1, 2]
    # ties produced through the router itself: Wr = 0 => logits = bias
    X = _rng(3).standard_normal((4, 16)).astype(np.float32)
    Wr = np.zeros((6, 16), dtype=np.float32)
    b = np.array([0.5, 1.0, 1.0, -1.0, 0.5, 1.0], dtype=np.float32)
    idx, w, lg = O.route(X, Wr, b, 4)
    assert np.all(idx == np.array([1, 2, 5, 0]))
    assert np.all(lg == b.astype(np.float64))


def check_router_logits_exact():
    # integer-valued inputs: every product and sum is exact, compare with
    # Python integers.  E != H and asymmetric values catch a transposed Wr.
    r = _rng(4)
    X = r.integers(-8, 9, size=(5, 12)).astype(np.float32)
    Wr = r.integers(-8, 9, size=(7, 12)).astype(np.float32)
    b = r.integers(-8, 9, size=7).astype(np.float32)
    lg = O.router_logits(X, Wr, b)
    for t in range(5):
        for e in range(7):
            want = int(b[e]) + sum(int(X[t, h]) * int(Wr[e, h]) for h in range(12))
            assert lg[t, e] == want
    # bf16 storage takes the same path
    lg2 = O.router_logits(bf16_bits_from_f32(X), bf16_bits_from_f32(Wr), b)
    assert np.array_equal(lg, lg2)
    assert np.array_equal(O.router_logits(X, Wr, None), lg - b.astype(np.float64))


def check_routing_margins_hand_worked():
    """The margin is the smallest gap between neighbours among the k+1 LARGEST
    logits: gaps inside the top-k fix the output order, the gap between the
    k-th and the (k+1)-th fixes membership; anything further down is irrelevant."""
    rows = np.array([
        [3.0, 1.0, 2.5, 0.0],      # sorted 3, 2.5, 1, 0
        [5.0, 4.0, 3.9, 0.0],      # the k-th / (k+1)-th gap (0.1) is the small one at k = 2
        [0.99, 5.0, 1.0, 3.0],     # unsorted; the tiny gap 1 - 0.99 sits below the top-2
        [-1.0, -4.0, -1.5, -9.0],  # negative logits
        [2.0, 1.0, 2.0, 0.0],      # exact tie inside the top-2
    ])
    m1 = O.routing_margins(rows, 1)
    assert np.allclose(m1, [0.5, 1.0, 2.0, 0.5, 0.0], rtol=0, atol=1e-15)
    m2 = O.routing_margins(rows, 2)
    assert np.allclose(m2, [0.5, 0.1, 2.0, 0.5, 0.0], rtol=0, atol=1e-12)
    assert m2[4] == 0.0
    m3 = O.routing_margins(rows, 3)
    assert np.allclose(m3, [0.5, 0.1, 0.01, 0.5, 0.0], rtol=0, atol=1e-12)
    # k = E: only the gaps inside the list (there is no (k+1)-th logit)
    m4 = O.routing_margins(rows, 4)
    assert np.allclose(m4, [0.5, 0.1, 0.01, 0.5, 0.0], rtol=0, atol=1e-12)
    # one expert: nothing to confuse
    assert np.all(np.isinf(O.routing_margins(np.array([[0.3], [-2.0]]), 1)))
    # a tie between the k-th and the (k+1)-th logit is a zero margin
    assert O.routing_margins(np.array([[7.0, 1.0, 1.0, 0.0]]), 2)[0] == 0.0
    assert O.routing_margins(np.array([[7.0, 1.0, 1.0, 0.0]]), 1)[0] == 6.0
    # consistent with the selector: perturbing any logit by less than half the margin
    # changes neither the selected experts nor their order
    r = _rng(40)
    for _ in range(40):
        E = int(r.integers(2, 9))
        k = int(r.integers(1, E + 1))
        lg = r.standard_normal((1, E))
        m = O.routing_margins(lg, k)[0]
        assert m > 0
        base = O.select_topk(lg[0], k).tolist()
        for _ in range(8):
            pert = lg[0] + r.uniform(-0.49, 0.49, size=E) * m
            assert O.select_topk(pert, k).tolist() == base
        # and a swap of the two logits that realise the margin does change it
        s = np.argsort(-lg[0], kind="stable")
        top = s[: min(k + 1, E)]
        gaps = lg[0][top[:-1]] - lg[0][top[1:]]
        j = int(np.argmin(gaps))
        assert abs(gaps[j] - m) < 1e-15
        sw = lg[0].copy()
        sw[top[j]], sw[top[j + 1]] = sw[top[j + 1]], sw[top[j]]
        assert O.select_topk(sw, k).tolist() != base


# ----------------------------------------------------------------- expert --
def _py_ffn(x, Wg, Wu, Wd):
    """SiLU-gated FFN with exactly rounded dot products (math.fsum), pure
    Python, independent of numpy's matmul."""
    F, H = len(Wg), len(x)
    h = []
    for f in range(F):
        g = math.fsum(Wg[f][i] * x[i] for i in range(H))
        u = math.fsum(Wu[f][i] * x[i] for i in range(H))
        h.append(g / (1.0 + math.exp(-g)) * u)
    return [math.fsum(Wd[o][f] * h[f] for f in range(F)) for o in range(len(Wd))]


def check_ffn_closed_form():
    # constant matrices: g_f = c, u_f = d for every f, y_o = silu(c)*d
    H, F = 8, 5
    x = np.ones(H)
    c, d = 1.25, -0.75
    y = O.expert_ffn(x, np.full((F, H), c / H), np.full((F, H), d / H), np.full((H, F), 1.0 / F))
    want = c / (1 + math.exp(-c)) * d
    assert np.allclose(y, want, rtol=1e-14, atol=0)
    # negative pre-activation: silu(-2) = -2/(1+e^2), sign mistakes show here
    y = O.expert_ffn(x, np.full((F, H), -2.0 / H), np.full((F, H), 1.0 / H), np.full((H, F), 1.0 / F))
    assert np.allclose(y, -2.0 / (1.0 + math.exp(2.0)), rtol=1e-14, atol=0)
    # rank-one matrices: g = a_g (b_g.x) etc.
    r = _rng(6)
    H, F = 7, 11
    x = r.standard_normal(H)
    ag, au, bd = r.standard_normal(F), r.standard_normal(F), r.standard_normal(F)
    bg, bu, ad = r.standard_normal(H), r.standard_normal(H), r.standard_normal(H)
    y = O.expert_ffn(x, np.outer(ag, bg), np.outer(au, bu), np.outer(ad, bd))
    sg, su = float(bg @ x), float(bu @ x)
    hvec = [(ag[f] * sg) / (1 + math.exp(-ag[f] * sg)) * (au[f] * su) for f in range(F)]
    s = math.fsum(bd[f] * hvec[f] for f in range(F))
    assert np.allclose(y, ad * s, rtol=1e-12, atol=1e-15)


def check_ffn_vs_pure_python():
    r = _rng(7)
    H, F = 6, 9
    x = r.standard_normal(H)
    Wg, Wu, Wd = r.standard_normal((F, H)), r.standard_normal((F, H)), r.standard_normal((H, F))
    y = O.expert_ffn(x, Wg, Wu, Wd)
    want = _py_ffn(x.tolist(), Wg.tolist(), Wu.tolist(), Wd.tolist())
    assert np.allclose(y, want, rtol=1e-13, atol=1e-15)


def _tiny_layer(seed, T=5, H=6, E=4, F=7, S=0, dtype=np.float32):
    r = _rng(seed)
    return dict(
        X=r.standard_normal((T, H)).astype(dtype),
        Wr=r.standard_normal((E, H)).astype(dtype),
        b=r.standard_normal(E).astype(np.float32),
        Wg=(r.standard_normal((E + S, F, H)) * 0.5).astype(dtype),
        Wu=(r.standard_normal((E + S, F, H)) * 0.5).astype(dtype),
        Wd=(r.standard_normal((E + S, H, F)) * 0.5).astype(dtype),
    )


def check_single_expert_is_plain_ffn():
    L = _tiny_layer(8, E=1)
    res = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k=1)
    assert np.all(res["topk_w"] == 1.0) and np.all(res["topk_idx"] == 0)
    for t in range(L["X"].shape[0]):
        want = _py_ffn(L["X"][t].astype(float).tolist(), L["Wg"][0].astype(float).tolist(),
                       L["Wu"][0].astype(float).tolist(), L["Wd"][0].astype(float).tolist())
        assert np.allclose(res["out"][t], want, rtol=1e-12, atol=1e-15)


def check_dense_mixture_when_k_equals_E():
    L = _tiny_layer(9, E=4)
    E = 4
    res = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k=E)
    for t in range(L["X"].shape[0]):
        x = L["X"][t].astype(float).tolist()
        lg = [float(L["b"][e]) + math.fsum(float(L["Wr"][e, h]) * x[h] for h in range(len(x)))
              for e in range(E)]
        m = max(lg)
        z = [math.exp(v - m) for v in lg]
        p = [v / math.fsum(z) for v in z]
        ys = [_py_ffn(x, L["Wg"][e].astype(float).tolist(), L["Wu"][e].astype(float).tolist(),
                      L["Wd"][e].astype(float).tolist()) for e in range(E)]
        want = [math.fsum(p[e] * ys[e][o] for e in range(E)) for o in range(len(x))]
        assert np.allclose(res["out"][t], want, rtol=1e-12, atol=1e-15)


def check_topk_layer_vs_pure_python():
    # k < E with shared experts: the selected set and weights come from the
    # brute-force selector above, the FFNs from the pure-Python routine.
    L = _tiny_layer(10, E=5, S=2)
    E, k, S = 5, 2, 2
    res = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k=k, S=S)
    tolist = lambda a: a.astype(float).tolist()
    for t in range(L["X"].shape[0]):
        x = tolist(L["X"][t])
        lg = [float(L["b"][e]) + math.fsum(float(L["Wr"][e, h]) * x[h] for h in range(len(x)))
              for e in range(E)]
        sel = _brute_topk(lg, k)
        assert res["topk_idx"][t].tolist() == sel
        z = [math.exp(lg[e] - lg[sel[0]]) for e in sel]
        w = [v / math.fsum(z) for v in z]
        ys = [_py_ffn(x, tolist(L["Wg"][e]), tolist(L["Wu"][e]), tolist(L["Wd"][e]))
              for e in sel]
        sh = [_py_ffn(x, tolist(L["Wg"][E + s]), tolist(L["Wu"][E + s]), tolist(L["Wd"][E + s]))
              for s in range(S)]
        want = [math.fsum([w[j] * ys[j][o] for j in range(k)] + [sh[s][o] for s in range(S)])
                for o in range(len(x))]
        assert np.allclose(res["out"][t], want, rtol=1e-12, atol=1e-15)


# --------------------------------------------------------------- bucketing --
def check_bucket_invariants():
    r = _rng(11)
    for (T, E, k) in [(8, 8, 2), (1, 8, 2), (128, 60, 4), (3, 64, 6), (40, 5, 5)]:
        idx = np.stack([r.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
        count, offset, perm, inv = O.bucket_by_expert(idx, E)
        A = T * k
        assert count.sum() == A and offset[0] == 0 and offset[-1] == A
        assert np.array_equal(offset[1:], np.cumsum(count))
        assert sorted(perm.tolist()) == list(range(A))
        assert np.array_equal(perm[inv], np.arange(A))
        flat = idx.reshape(-1)
        for e in range(E):
            seg = perm[offset[e]:offset[e + 1]]
            assert np.all(flat[seg] == e)
            assert np.all(np.diff(seg) > 0)          # stable
        # a stable library sort by expert id is the same permutation
        assert np.array_equal(perm, np.argsort(flat, kind="stable"))
        assert np.array_equal(count, np.bincount(flat, minlength=E))


def check_identity_roundtrip():
    # if every expert returned its input, combine gives X back (weights sum to 1)
    r = _rng(12)
    T, E, k, H = 9, 6, 3, 10
    X = r.standard_normal((T, H))
    idx, w, _ = O.route(X.astype(np.float32), r.standard_normal((E, H)).astype(np.float32), None, k)
    count, offset, perm, inv = O.bucket_by_expert(idx, E)
    Y = X.astype(np.float32).astype(np.float64)[perm // k]
    out = O.combine_rows(Y, w, inv, T, k)
    assert np.allclose(out, X.astype(np.float32), rtol=0, atol=1e-14)


def check_decomposed_equals_definition():
    # route -> bucket -> grouped rows -> combine  ==  the token-major definition
    for S in (0, 2):
        L = _tiny_layer(13 + S, T=7, E=5, S=S)
        k = 2
        res = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k, S)
        count, offset, perm, inv = O.bucket_by_expert(res["topk_idx"], 5)
        Y = O.grouped_ffn_rows(L["X"], perm, offset, k, L["Wg"], L["Wu"], L["Wd"], S)
        out = O.combine_rows(Y, res["topk_w"], inv, 7, k, S)
        assert np.allclose(out, res["out"], rtol=1e-13, atol=1e-15)
        res2 = O.combine_rows(Y, res["topk_w"], inv, 7, k, S, residual=L["X"])
        assert np.allclose(res2, res["out"] + L["X"].astype(np.float64), rtol=1e-13, atol=1e-15)


# ------------------------------------------------------------- properties --
def check_batch_independence_and_equivariance():
    L = _tiny_layer(20, T=6, E=5)
    k = 2
    full = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k)
    p = np.array([3, 0, 5, 1, 4, 2])
    perm = O.moe_layer(L["X"][p], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k)
    assert np.array_equal(perm["out"], full["out"][p])
    assert np.array_equal(perm["topk_idx"], full["topk_idx"][p])
    one = O.moe_layer(L["X"][2:3], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k)
    assert np.array_equal(one["out"][0], full["out"][2])
    some = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k, tokens=[4, 1])
    assert np.array_equal(some["out"][[1, 4]], full["out"][[1, 4]])
    assert not some["out"][0].any()


def check_linearity_in_down_projection():
    L = _tiny_layer(21, T=4, E=3)
    k = 2
    base = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k)
    Wd2 = L["Wd"].copy()
    Wd2[1] *= 2.0
    dbl = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], Wd2, k)
    Wd0 = L["Wd"].copy()
    Wd0[1] = 0.0
    zero = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], Wd0, k)
    # out = rest + c1 ; doubled = rest + 2 c1 ; zeroed = rest
    assert np.allclose(dbl["out"] - zero["out"], 2.0 * (base["out"] - zero["out"]),
                       rtol=1e-12, atol=1e-15)
    uses = (base["topk_idx"] == 1).any(axis=1)
    assert np.all((base["out"] - zero["out"])[~uses] == 0.0)
    assert uses.any() and (np.abs(base["out"] - zero["out"])[uses] > 0).any()


def check_shared_experts_concat():
    # S shared experts of width F  ==  one SiLU-gated FFN of width S*F
    L = _tiny_layer(22, T=3, E=2, S=3)
    res = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k=1, S=3)
    nos = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"][:2], L["Wu"][:2], L["Wd"][:2], k=1, S=0)
    Wg = np.concatenate(list(L["Wg"][2:]), axis=0).astype(np.float64)
    Wu = np.concatenate(list(L["Wu"][2:]), axis=0).astype(np.float64)
    Wd = np.concatenate(list(L["Wd"][2:]), axis=1).astype(np.float64)
    for t in range(3):
        want = _py_ffn(L["X"][t].astype(float).tolist(), Wg.tolist(), Wu.tolist(), Wd.tolist())
        assert np.allclose(res["out"][t] - nos["out"][t], want, rtol=1e-11, atol=1e-14)


# ------------------------------------------------------------------ stack --
def check_rmsnorm_and_stack():
    n = O.rmsnorm(np.array([[3.0, 4.0]]))
    assert np.allclose(n, np.array([[3.0, 4.0]]) / math.sqrt(12.5 + 1e-6), rtol=1e-15, atol=0)
    L = [_tiny_layer(30 + i, T=3, E=3) for i in range(2)]
    X0 = L[0]["X"]
    xf, trace = O.moe_stack(X0, L, k=2, storage="f32")
    x = X0.astype(np.float64)
    for i in range(2):
        inp = (x / np.sqrt((x * x).mean(axis=1, keepdims=True) + 1e-6)).astype(np.float32)
        assert np.array_equal(trace[i]["inp"], inp)
        r = O.moe_layer(inp, L[i]["Wr"], L[i]["b"], L[i]["Wg"], L[i]["Wu"], L[i]["Wd"], 2)
        x = x + r["out"]
    assert np.array_equal(xf, x)


def check_stack_bf16_hand_worked():
    """bf16 storage of the stack, two layers, values worked by hand.

    Row 0 is +-1 everywhere: mean square 1, so the normalised row is
    +-1/sqrt(1 + 1e-6) = +-0.9999995, which rounds to bf16 +-1.0 (0x3F80 /
    0xBF80).  Row 1 alternates 3, 4: mean square 12.5; 3/sqrt(12.500001) =
    0.848528 lies in [0.5, 1) where bf16 steps are 2^-8, 0.848528 * 256 = 217.22
    -> 217/256 = 0.84765625 = 0x3F59; 4/sqrt(12.500001) = 1.131371 lies in
    [1, 2) with steps 2^-7, 1.131371 * 128 = 144.82 -> 145/128 = 1.1328125 =
    0x3F91.  The layer input must be exactly those bits; the residual stream
    adds the block output to the UN-normalised float64 row."""
    H, E, F, k = 4, 3, 5, 2
    X0 = bf16_bits_from_f32(np.array([[1, -1, 1, -1], [3, 4, 3, 4]], dtype=np.float32))
    want_bits = np.array([[0x3F80, 0xBF80, 0x3F80, 0xBF80], [0x3F59, 0x3F91, 0x3F59, 0x3F91]],
                         dtype=np.uint16)
    want_vals = [[1.0, -1.0, 1.0, -1.0], [217 / 256, 145 / 128, 217 / 256, 145 / 128]]
    r = _rng(41)
    bf = lambda a: bf16_bits_from_f32(a.astype(np.float32))
    layers = [dict(Wr=bf(r.standard_normal((E, H))), b=r.standard_normal(E).astype(np.float32),
                   Wg=bf(r.standard_normal((E, F, H)) * 0.5), Wu=bf(r.standard_normal((E, F, H)) * 0.5),
                   Wd=bf(r.standard_normal((E, H, F)) * 0.5)) for _ in range(2)]
    xf, trace = O.moe_stack(X0, layers, k=k, storage="bf16")
    assert trace[0]["inp"].dtype == np.uint16
    assert np.array_equal(trace[0]["inp"], want_bits)

    # layer 0 by the pure-Python routines on the hand-worked input values
    def py_layer(L, rows):
        tolist = lambda a: O.widen(a).tolist()
        outs = []
        for x in rows:
            lg = [float(L["b"][e]) + math.fsum(w * v for w, v in zip(tolist(L["Wr"][e]), x))
                  for e in range(E)]
            sel = _brute_topk(lg, k)
            z = [math.exp(lg[e] - lg[sel[0]]) for e in sel]
            w = [v / math.fsum(z) for v in z]
            ys = [_py_ffn(x, tolist(L["Wg"][e]), tolist(L["Wu"][e]), tolist(L["Wd"][e])) for e in sel]
            outs.append([math.fsum(w[j] * ys[j][o] for j in range(k)) for o in range(H)])
        return np.array(outs)

    out0 = py_layer(layers[0], want_vals)
    assert np.allclose(trace[0]["out"], out0, rtol=1e-12, atol=1e-15)
    x1 = np.array([[1.0, -1.0, 1.0, -1.0], [3.0, 4.0, 3.0, 4.0]]) + out0
    # layer 1 sees bf16(rmsnorm(x1)): nearest bf16 neighbours checked with exact fractions
    n1 = x1 / np.sqrt((x1 * x1).mean(axis=1, keepdims=True) + 1e-6)
    got1 = O.widen(trace[1]["inp"])
    for v, g in zip(n1.reshape(-1), got1.reshape(-1)):
        ulp = 2.0 ** (math.floor(math.log2(abs(g))) - 7)
        assert Fraction(g) % Fraction(ulp) == 0            # a bf16 value
        assert abs(Fraction(v) - Fraction(g)) <= Fraction(ulp) / 2
    out1 = py_layer(layers[1], got1.tolist())
    assert np.allclose(xf, x1 + out1, rtol=1e-12, atol=1e-14)


def check_prefetch_set():
    lg = np.array([[5.0, 4.0, 0.0, 0.0], [5.0, 0.0, 4.0, 0.0], [0.0, 0.0, 5.0, 4.0]])
    z = np.zeros_like(lg)
    res = np.array([True, False, False, False])
    # votes: e0=2, e1=1, e2=2, e3=1 ; non-resident ranking: e2, e1, e3
    assert O.predicted_prefetch_set(lg, z, 2, 2, res).tolist() == [False, True, True, False]
    assert O.predicted_prefetch_set(lg, z, 2, 1, res).tolist() == [False, False, True, False]
    noise = np.zeros_like(lg)
    noise[:, 3] = 10.0
    assert O.predicted_prefetch_set(lg, noise, 2, 1, res).tolist() == [False, False, False, True]


# ----------------------------------------------------------------- paper ---
def check_table2_sizes():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table2_expert_sizes.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for name, layers, experts, topk, mib, H, F in rows:
        assert 3 * int(H) * int(F) * 2 == Fraction(mib) * 2 ** 20
    c2, c4, c5 = get_config("c2_mixtral"), get_config("c4_dsv2lite_prefill"), get_config("c5_stack")
    assert c2.expert_bytes == 352321536 and c5.expert_bytes == 352321536
    assert c4.expert_bytes == 17301504
    assert (c2.E, c2.k, c5.layers) == (int(rows[0][2]), int(rows[0][3]), int(rows[0][1]))
    assert (c4.E, c4.k) == (int(rows[1][2]), int(rows[1][3]))
    c6 = get_config("c6_qwen3_a3b")
    assert c6.expert_bytes == 9 * 2 ** 20
    assert (c6.E, c6.k, c6.H, c6.F) == tuple(int(rows[3][i]) for i in (2, 3, 5, 6))


def check_table3_identity():
    size = {"deepseek": 17301504, "qwen": 3 * 2048 * 768 * 2, "mixtral": 352321536}
    peak = {"pcie3x16": 15.75e9, "pcie4x16": 31.5e9}
    for l in open(os.path.join(GOLDEN, "table3_transfer.txt")):
        if not l.strip() or l.startswith("#"):
            continue
        link, model, ms, util = l.split()
        t = size[model] / (float(util) * peak[link]) * 1e3
        assert abs(t - float(ms)) / float(ms) < 0.08, (link, model, t, ms)


ALL_CHECKS = [v for k, v in sorted(globals().items()) if k.startswith("check_")]


@pytest.mark.parametrize("check", ALL_CHECKS, ids=lambda f: f.__name__)
def test_pin(check):
    check()


# ------------------------------------------------------------ mutations ----
def _m_no_renorm(logit_row, idx):
    z = np.exp(logit_row - logit_row.max())
    return (z / z.sum())[idx]


def _m_silu_sign(z):
    return z / (1.0 + np.exp(z))


def _m_ffn_swapped(x, Wg, Wu, Wd):
    return Wd @ (O.silu(Wu @ x) * (Wg @ x))


def _m_ffn_no_gate(x, Wg, Wu, Wd):
    return Wd @ (O.silu(Wg @ x))


def _m_topk_highest_index(logit_row, k):
    order = sorted(range(len(logit_row)), key=lambda e: (-logit_row[e], -e))
    return np.array(order[:k], dtype=np.int32)


def _m_topk_ascending(logit_row, k):
    order = sorted(range(len(logit_row)), key=lambda e: (-logit_row[e], e))
    return np.array(order[:k][::-1], dtype=np.int32)


def _m_logits_no_bias(X, Wr, b=None):
    return O.widen(X) @ O.widen(Wr).T


def _m_softmax_selected_only_wrong(logit_row, idx):
    z = np.exp(logit_row[idx])            # no shift: overflows on huge logits
    return z / z.sum()


def _m_margins_topk_only(logits, k):
    out = np.empty(logits.shape[0])
    for t in range(logits.shape[0]):
        s = np.sort(logits[t])[::-1][:k]
        out[t] = np.min(s[:-1] - s[1:]) if s.shape[0] > 1 else np.inf
    return out


def _m_margins_all_gaps(logits, k):
    s = np.sort(logits, axis=1)[:, ::-1]
    return np.min(s[:, :-1] - s[:, 1:], axis=1) if logits.shape[1] > 1 else np.full(logits.shape[0], np.inf)


def _m_margins_boundary_only(logits, k):
    s = np.sort(logits, axis=1)[:, ::-1]
    E = logits.shape[1]
    return s[:, k - 1] - s[:, k] if k < E else np.full(logits.shape[0], np.inf)


def _m_rmsnorm_no_eps(x, eps=1e-6):
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True))


def _m_rmsnorm_sum_not_mean(x, eps=1e-6):
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.sum(x * x, axis=-1, keepdims=True) + eps)


def _m_bf16_truncate(a):
    f = np.asarray(a, dtype=np.float64).astype(np.float32)
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _m_stack_residual_is_normalised(X0, layers, k, S=0, storage="bf16"):
    x = O.widen(X0)
    trace = []
    for L in layers:
        inp = O.round_to_bf16_bits(O.rmsnorm(x))
        r = O.moe_layer(inp, L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k, S)
        r["inp"] = inp
        trace.append(r)
        x = O.widen(inp) + r["out"]
    return x, trace


def _m_stack_no_residual(X0, layers, k, S=0, storage="bf16"):
    x = O.widen(X0)
    trace = []
    for L in layers:
        inp = O.round_to_bf16_bits(O.rmsnorm(x))
        r = O.moe_layer(inp, L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k, S)
        r["inp"] = inp
        trace.append(r)
        x = r["out"]
    return x, trace


MUTATIONS = [
    ("routing_margins", _m_margins_topk_only, [check_routing_margins_hand_worked]),
    ("routing_margins", _m_margins_all_gaps, [check_routing_margins_hand_worked]),
    ("routing_margins", _m_margins_boundary_only, [check_routing_margins_hand_worked]),
    ("rmsnorm", _m_rmsnorm_sum_not_mean, [check_rmsnorm_and_stack, check_stack_bf16_hand_worked]),
    ("rmsnorm", _m_rmsnorm_no_eps, [check_rmsnorm_and_stack]),
    ("round_to_bf16_bits", _m_bf16_truncate, [check_bf16_rounding, check_stack_bf16_hand_worked]),
    ("moe_stack", _m_stack_residual_is_normalised, [check_stack_bf16_hand_worked]),
    ("moe_stack", _m_stack_no_residual, [check_stack_bf16_hand_worked]),
    ("gate_weights", _m_no_renorm, [check_softmax_closed_form, check_weights_sum_and_order]),
    ("gate_weights", _m_softmax_selected_only_wrong, [check_softmax_closed_form]),
    ("silu", _m_silu_sign, [check_ffn_closed_form, check_ffn_vs_pure_python]),
    ("expert_ffn", _m_ffn_swapped, [check_ffn_closed_form, check_ffn_vs_pure_python,
                                    check_single_expert_is_plain_ffn]),
    ("expert_ffn", _m_ffn_no_gate, [check_ffn_closed_form, check_dense_mixture_when_k_equals_E]),
    ("select_topk", _m_topk_highest_index, [check_topk_bruteforce]),
    ("select_topk", _m_topk_ascending, [check_topk_bruteforce, check_softmax_closed_form]),
    ("router_logits", _m_logits_no_bias, [check_router_logits_exact, check_topk_bruteforce]),
]


@pytest.mark.parametrize("name,mutant,checks", MUTATIONS,
                         ids=[f"{n}-{m.__name__}" for n, m, _ in MUTATIONS])
def test_planted_mistake_is_caught(monkeypatch, name, mutant, checks):
    """A mistake planted in the oracle (CPU only) must fail its pins."""
    monkeypatch.setattr(O, name, mutant)
    for chk in checks:
        with pytest.raises((AssertionError, FloatingPointError, RuntimeWarning)):
            with np.errstate(over="raise", invalid="raise"):
                chk()


def test_configs_have_safe_routing_margins():
    """Bit-exact routing is only well posed if no top-(k+1) gap of the fixed
    seeds is at rounding-noise level (float64 summation-order noise ~1e-15)."""
    for name in ("c1_tiny", "c3_finegrained"):
        cfg = get_config(name)
        L = make_layer(cfg, threads=4)
        lg = O.router_logits(L["X"], L["Wr"], L["b"])
        assert O.routing_margins(lg, cfg.k).min() > 1e-9
