"""Plain fp64 CPU oracle of one MoE block.  TEST INFRASTRUCTURE ONLY.

What it computes (paper Section 2.1, the block equation): for every token the
gate picks the top-k experts e_j with routing weights w_j from a softmax, and
the block output is  x' = sum_j w_j * Expert_{e_j}(a).  An expert is the three
linear maps gate_proj, up_proj, down_proj (Section 4.4); the evaluated models
use them as a SiLU-gated FFN.  Expert residency / prefetching (Section 4.4)
moves bytes only and never changes this result, so the oracle has no notion of
it.

Everything is evaluated token by token in float64 with no intermediate
rounding, no bucketing and no reordering; numpy's ``@`` (a matrix-vector
product) is the only library primitive used as a step.

Readings taken where the paper is silent:
  * selection is on the router logits, ties to the lowest expert index, output
    order = order of selection (descending logit);
  * the k selected weights are renormalised to sum to one;
  * an optional router bias is added to the logit before selection and softmax;
  * shared experts see every token with weight one, outside the softmax;
  * in a stack, x_{l+1} = x_l + MoE_l(rmsnorm(x_l)), weightless RMS norm with
    eps = 1e-6, the normalised input rounded to the storage dtype.

Pins (tests/test_oracle_pins.py): closed-form softmax weights, rank-one
closed-form FFN against pure-Python exact sums, brute-force subset top-k incl.
crafted ties, k = E dense mixture, E = 1 plain FFN, bucket invariants,
identity-expert round trip, linearity, shared-expert concatenation, the expert
sizes printed in Table 2, hand-worked routing margins (checked against the
selector under perturbation), and a two-layer bf16 stack whose normalised
inputs land on bf16 bit patterns worked by hand.  Planted mistakes in each of
these functions fail their pins.  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "widen", "router_logits", "select_topk", "gate_weights", "route",
    "routing_margins", "silu", "expert_ffn", "bucket_by_expert",
    "grouped_ffn_rows", "combine_rows", "moe_layer", "rmsnorm", "moe_stack",
    "round_to_bf16_bits", "predicted_prefetch_set",
]


# --------------------------------------------------------------------------
# storage -> float64 (exact)
# --------------------------------------------------------------------------
def widen(a: np.ndarray) -> np.ndarray:
    """Exact widening of stored values to float64.

    float32/float64 arrays widen directly; ``uint16`` arrays are bfloat16 bit
    patterns (sign, 8 exponent bits, 7 mantissa bits = the top half of a
    float32)."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if a.dtype in (np.float32, np.float64):
        return a.astype(np.float64)
    raise TypeError(f"unsupported storage dtype {a.dtype}")


def round_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float64 values to bfloat16, nearest even, via one exact float64 ->
    float32 -> bf16 path guarded against double rounding (used only to hand a
    stack layer's input to the next layer in the storage dtype)."""
    a = np.asarray(a, dtype=np.float64)
    f = a.astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lo = (u & np.uint64(0xFFFF0000)).astype(np.uint32).view(np.float32).astype(np.float64)
    # candidates: truncation toward zero (lo) and one bf16 ulp further out (hi)
    hi_bits = ((u & np.uint64(0xFFFF0000)) + np.uint64(0x10000)).astype(np.uint32)
    hi = hi_bits.view(np.float32).astype(np.float64)
    dl = np.abs(a - lo)
    dh = np.abs(hi - a)
    lo_even = ((u >> np.uint64(16)) & np.uint64(1)) == 0
    take_hi = (dh < dl) | ((dh == dl) & ~lo_even)
    bits = np.where(take_hi, hi_bits >> np.uint32(16), (u >> np.uint64(16)).astype(np.uint32))
    return bits.astype(np.uint16)


# --------------------------------------------------------------------------
# gate (Section 2.1: "e_i, w_i = Gate(a)")
# --------------------------------------------------------------------------
def router_logits(X, Wr, b=None) -> np.ndarray:
    """logit[t, e] = b[e] + sum_h X[t, h] * Wr[e, h], float64."""
    Xd, Wd = widen(X), widen(Wr)
    T, E = Xd.shape[0], Wd.shape[0]
    out = np.empty((T, E), dtype=np.float64)
    for t in range(T):
        out[t] = Wd @ Xd[t]
        if b is not None:
            out[t] += np.asarray(b, dtype=np.float64)
    return out


def select_topk(logit_row: np.ndarray, k: int) -> np.ndarray:
    """k rounds: take the largest logit not taken yet; among equal logits the
    lowest expert index wins.  Returns indices in order of selection."""
    E = logit_row.shape[0]
    if not 1 <= k <= E:
        raise ValueError("need 1 <= k <= E")
    taken = np.zeros(E, dtype=bool)
    out = np.empty(k, dtype=np.int32)
    for j in range(k):
        best = -1
        for e in range(E):
            if taken[e]:
                continue
            if best < 0 or logit_row[e] > logit_row[best]:
                best = e
        taken[best] = True
        out[j] = best
    return out


def gate_weights(logit_row: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Softmax over ALL experts (max subtracted), then the selected entries
    renormalised to sum to one."""
    z = logit_row - np.max(logit_row)
    p = np.exp(z)
    p = p / np.sum(p)
    sel = p[idx]
    return sel / np.sum(sel)


def route(X, Wr, b, k):
    """(topk_idx [T,k] int32, topk_w [T,k] float64, logits [T,E] float64)."""
    logits = router_logits(X, Wr, b)
    T = logits.shape[0]
    idx = np.empty((T, k), dtype=np.int32)
    w = np.empty((T, k), dtype=np.float64)
    for t in range(T):
        idx[t] = select_topk(logits[t], k)
        w[t] = gate_weights(logits[t], idx[t])
    return idx, w, logits


def routing_margins(logits: np.ndarray, k: int) -> np.ndarray:
    """Per token: the smallest gap between neighbouring logits among the k+1
    largest (gaps inside the top-k decide the output order, the k-th gap decides
    membership).  A tiny margin means the routing of that token is decided by
    rounding noise and cannot be compared bit-exactly."""
    T, E = logits.shape
    out = np.empty(T, dtype=np.float64)
    for t in range(T):
        s = np.sort(logits[t])[::-1]
        top = s[: min(k + 1, E)]
        out[t] = np.min(top[:-1] - top[1:]) if top.shape[0] > 1 else np.inf
    return out


# --------------------------------------------------------------------------
# expert (Section 4.4: gate_proj, up_proj, down_proj)
# --------------------------------------------------------------------------
def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def expert_ffn(x: np.ndarray, Wg: np.ndarray, Wu: np.ndarray, Wd: np.ndarray) -> np.ndarray:
    """y = Wd . ( silu(Wg . x) * (Wu . x) );  all operands already float64.
    Wg, Wu are [F, H]; Wd is [H, F]."""
    g = Wg @ x
    u = Wu @ x
    h = silu(g) * u
    return Wd @ h


class _Wide:
    """Memo of exactly-widened expert matrices (a conversion cache, not a
    change of arithmetic).  Keeps at most ``keep`` experts alive."""

    def __init__(self, Wg, Wu, Wd, keep=3):
        self.Wg, self.Wu, self.Wd, self.keep = Wg, Wu, Wd, keep
        self.memo = {}

    def get(self, e):
        if e not in self.memo:
            if len(self.memo) >= self.keep:
                self.memo.pop(next(iter(self.memo)))
            self.memo[e] = (widen(self.Wg[e]), widen(self.Wu[e]), widen(self.Wd[e]))
        return self.memo[e]


# --------------------------------------------------------------------------
# bucketing (per-expert pending-token counts, Section 4.3.2 Premise 1)
# --------------------------------------------------------------------------
def bucket_by_expert(topk_idx: np.ndarray, E: int):
    """Group the flat assignments i = t*k + j by expert, keeping ascending i
    inside a group.

    Returns count [E], offset [E+1] (exclusive scan), perm [A] (perm[p] = the
    assignment stored at bucket position p) and inv_perm [A] (inv_perm[i] = the
    bucket position of assignment i)."""
    flat = np.asarray(topk_idx).reshape(-1)
    A = flat.shape[0]
    count = np.zeros(E, dtype=np.int32)
    for i in range(A):
        count[flat[i]] += 1
    offset = np.zeros(E + 1, dtype=np.int32)
    for e in range(E):
        offset[e + 1] = offset[e] + count[e]
    cursor = offset[:-1].copy()
    perm = np.empty(A, dtype=np.int32)
    inv_perm = np.empty(A, dtype=np.int32)
    for i in range(A):
        p = cursor[flat[i]]
        cursor[flat[i]] += 1
        perm[p] = i
        inv_perm[i] = p
    return count, offset, perm, inv_perm


def grouped_ffn_rows(X, perm, offset, k, Wg, Wu, Wd, S=0):
    """Y [A + S*T, H] float64: row p (< A) is Expert_e(x_t) for the assignment
    perm[p] = t*k + j that lives in expert e's bucket; row A + s*T + t is shared
    expert s applied to token t."""
    Xd = widen(X)
    T, H = Xd.shape
    E = offset.shape[0] - 1
    A = perm.shape[0]
    wide = _Wide(Wg, Wu, Wd)
    Y = np.zeros((A + S * T, H), dtype=np.float64)
    for e in range(E):
        for p in range(offset[e], offset[e + 1]):
            t = perm[p] // k
            Y[p] = expert_ffn(Xd[t], *wide.get(e))
    for s in range(S):
        for t in range(T):
            Y[A + s * T + t] = expert_ffn(Xd[t], *wide.get(E + s))
    return Y


def combine_rows(Y, topk_w, inv_perm, T, k, S=0, residual=None):
    """out[t] = sum_j w[t,j] * Y[inv_perm[t*k+j]] + sum_s Y[A + s*T + t]
    (+ residual[t])."""
    Y = np.asarray(Y, dtype=np.float64)
    A = T * k
    out = np.zeros((T, Y.shape[1]), dtype=np.float64)
    for t in range(T):
        for j in range(k):
            out[t] += float(topk_w[t, j]) * Y[inv_perm[t * k + j]]
        for s in range(S):
            out[t] += Y[A + s * T + t]
        if residual is not None:
            out[t] += widen(residual)[t]
    return out


# --------------------------------------------------------------------------
# the block (Section 2.1 equation), token by token
# --------------------------------------------------------------------------
def moe_layer(X, Wr, b, Wg, Wu, Wd, k, S=0, tokens=None):
    """out[t] = sum_j w_j * Expert_{e_j}(x_t) + sum_s Shared_s(x_t).

    Wg/Wu/Wd hold the E routed experts followed by the S shared experts.
    ``tokens``: optional list of token indices to evaluate (others are left
    zero in ``out``); routing is always computed for every token.

    Returns dict(out [T,H] f64, topk_idx, topk_w, logits)."""
    Xd = widen(X)
    T, H = Xd.shape
    E = np.asarray(Wr).shape[0]
    idx, w, logits = route(X, Wr, b, k)
    wide = _Wide(Wg, Wu, Wd)
    out = np.zeros((T, H), dtype=np.float64)
    todo = range(T) if tokens is None else tokens
    # visiting tokens grouped by their first expert only keeps the widening
    # memo warm; each token's arithmetic is untouched
    for t in sorted(todo, key=lambda t: (int(idx[t, 0]), t)):
        acc = np.zeros(H, dtype=np.float64)
        for j in range(k):
            acc += w[t, j] * expert_ffn(Xd[t], *wide.get(int(idx[t, j])))
        for s in range(S):
            acc += expert_ffn(Xd[t], *wide.get(E + s))
        out[t] = acc
    return {"out": out, "topk_idx": idx, "topk_w": w, "logits": logits}


# --------------------------------------------------------------------------
# the stack used by the streamed configuration
# --------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, eps: float = 1e-6) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps), per row, float64, no learned scale."""
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


def moe_stack(X0, layers, k, S=0, storage="bf16"):
    """x_{l+1} = x_l + MoE_l(store(rmsnorm(x_l))) over ``layers`` (an iterable
    of dicts with Wr, b, Wg, Wu, Wd).  The residual stream stays float64; the
    normalised layer input is rounded to the storage dtype because that is what
    a layer is handed.  Returns (x_final, per_layer list of dict(inp, out,
    topk_idx, topk_w, logits))."""
    x = widen(X0)
    trace = []
    for L in layers:
        n = rmsnorm(x)
        inp = round_to_bf16_bits(n) if storage == "bf16" else n.astype(np.float32)
        r = moe_layer(inp, L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k, S)
        r["inp"] = inp
        trace.append(r)
        x = x + r["out"]
    return x, trace


def predicted_prefetch_set(next_logits, noise, k, n_prefetch, resident):
    """Stand-in for an expert predictor: perturb the next layer's true logits
    with the given noise, count for each expert the tokens whose noisy top-k
    contains it, and return the ``n_prefetch`` non-resident experts with the
    highest predicted token count (ties to the lowest index), as a bool [E]."""
    noisy = np.asarray(next_logits, dtype=np.float64) + np.asarray(noise, dtype=np.float64)
    T, E = noisy.shape
    votes = np.zeros(E, dtype=np.int64)
    for t in range(T):
        for e in select_topk(noisy[t], k):
            votes[e] += 1
    order = sorted(range(E), key=lambda e: (-votes[e], e))
    out = np.zeros(E, dtype=bool)
    n = 0
    for e in order:
        if n >= n_prefetch:
            break
        if not resident[e] and votes[e] > 0:
            out[e] = True
            n += 1
    return out
