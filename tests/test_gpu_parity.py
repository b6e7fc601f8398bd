"""GPU parity: every call goes through the C-ABI (ctypes binding) and is
compared element by element with the CPU oracle on the same seeded inputs.

Bars: routing indices, counts, offsets and permutations bit-exact; gate weights
within 1e-5 absolute; outputs within 2e-2 (bf16) / 1e-5 (f32) in the
row-normalised max-error metric  max_t ||d[t]||_inf / ||ref[t]||_inf.
"""
import numpy as np
import pytest
import torch

import oracle.moe_oracle as O
from workloads import MoEConfig, get_config, make_layer, make_hidden
from gpu_util import to_dev, to_host_bits, row_rel_err, TOL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import paper_2509_23638_amd.binding as b
    return b


def _shape(B, cfg, T=None, layout="row_major"):
    return B.make_shape(cfg.T if T is None else T, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, cfg.dtype,
                        layout if cfg.dtype == "bf16" else "row_major")


def _experts_dev(B, L, layout):
    """Expert matrices on the GPU in the requested layout (tiled = packed once
    by the library, the way a loader would)."""
    Wg, Wu, Wd = to_dev(L["Wg"]), to_dev(L["Wu"]), to_dev(L["Wd"])
    if layout == "tiled" and L["Wg"].dtype == np.uint16:
        Wg, Wu, Wd = B.pack_experts(Wg), B.pack_experts(Wu), B.pack_experts(Wd)
    return Wg, Wu, Wd


LAYOUTS = ["row_major", "tiled"]


def _small(name, **kw):
    base = dict(name=name, T=40, H=256, E=4, k=2, F=384, S=0, dtype="bf16", bias="normal",
                bias_scale=0.5, w_std=0.05, seed=3)
    base.update(kw)
    return MoEConfig(**base)


SMALL = [
    _small("s_bf16"),
    _small("s_bf16_shared", S=2, T=23),
    _small("s_bf16_ragged", T=150, E=2, k=1, H=384, F=256),       # > 64 rows per expert
    _small("s_bf16_many", T=33, E=60, k=4, H=128, F=128, S=1, bias="zipf", bias_scale=1.1),
    _small("s_bf16_e128", T=17, E=128, k=8, H=256, F=128),
    _small("s_bf16_limits", T=5, E=128, k=16, S=8, H=128, F=128),      # every documented maximum
    _small("s_bf16_big_blocks", T=300, E=4, k=2, H=256, F=384, S=1),   # > 128 rows per expert
    _small("s_bf16_odd_chunks", T=20, E=4, k=1, H=128, F=1408, bias="none"),  # 11 k-chunks of 128
    _small("s_bf16_one", T=1, E=8, k=2),
    _small("s_bf16_k_eq_e", T=9, E=3, k=3),
    _small("s_f32", dtype="f32", T=19, H=64, F=96, S=1),
    _small("s_f32_e1", dtype="f32", T=5, E=1, k=1, H=72, F=40),
    # many tokens x experts take the matrix-core router: ragged hidden size, ragged tiles, E = 128
    _small("s_f32_mfma_route", dtype="f32", T=530, E=60, k=2, H=72, F=40),
    _small("s_bf16_mfma_route_e128", T=260, E=128, k=8, H=256, F=128),
    _small("s_bf16_mfma_route_e20", T=1030, E=20, k=3, H=384, F=128, S=1),
    # few tokens, many experts: every tile of the vector router (1, 2, 4 tokens per lane)
    _small("s_bf16_route_t3_e60", T=3, E=60, k=4, H=384, F=128),
    _small("s_bf16_route_t40_e100", T=40, E=100, k=5, H=1152, F=128),
    _small("s_f32_route_e12", dtype="f32", T=70, E=12, k=3, H=200, F=40),
    _small("s_bf16_route_4tok_lane", T=130, E=128, k=8, H=256, F=128),
    _small("s_bf16_route_2tok_lane", T=70, E=128, k=8, H=2176, F=128),
    _small("s_bf16_route_deep", T=20, E=60, k=4, H=4224, F=128),
    _small("s_bf16_route_mfma_8waves", T=260, E=128, k=8, H=2176, F=128),
    _small("s_bf16_route_fused_long", T=6, E=8, k=2, H=4224, F=128),
    # FFN kernel choices not reached above: halved-contraction down, shared experts over 200 tokens
    # (tiled gate/up, several 64-row passes of the one-tile down form),
    # the tiled kernel as the gate/up kernel of wide experts at decode sizes
    _small("s_bf16_halves", T=40, E=4, k=2, H=256, F=512),
    _small("s_bf16_128row_passes", T=200, E=60, k=4, S=1, H=128, F=256, bias="zipf", bias_scale=1.1),
    _small("s_bf16_wide_decode", T=12, E=8, k=2, H=128, F=4096),
    _small("s_bf16_wide_halves", T=40, E=8, k=2, H=128, F=4096),
    # well-filled blocks: the eight-wave tiled form, all three pipeline remainders
    # (contraction lengths of 8, 10 and 12 stages), uneven and split blocks
    _small("s_bf16_filled_blocks", T=400, E=4, k=2, H=512, F=640, S=1, bias="zipf", bias_scale=0.7),
    _small("s_bf16_filled_blocks_12", T=300, E=2, k=1, H=768, F=768, S=1),
    # at most 64 tokens in the tiled kernels (both phases; the shortest contraction whose ring runs on
    # from item to item, several items per workgroup; shared experts; one bucket nearly full)
    _small("s_bf16_small_tiled", T=60, E=2, k=1, H=256, F=512),
    _small("s_bf16_small_tiled_two_items", T=64, E=2, k=2, H=512, F=8192, S=1),
]


def _route_gpu(B, cfg, L, X):
    sh = _shape(B, cfg, X.shape[0])
    T = X.shape[0]
    idx = torch.empty((T, cfg.k), dtype=torch.int32, device="cuda")
    w = torch.empty((T, cfg.k), dtype=torch.float32, device="cuda")
    lg = torch.empty((T, cfg.E), dtype=torch.float64, device="cuda")
    B.moe_route(sh, to_dev(X), to_dev(L["Wr"]), to_dev(L["b"]), idx, w, lg)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), w.cpu().numpy(), lg.cpu().numpy()


def _check_route(B, cfg, L, X):
    idx, w, lg = _route_gpu(B, cfg, L, X)
    ridx, rw, rlg = O.route(X, L["Wr"], L["b"], cfg.k)
    assert O.routing_margins(rlg, cfg.k).min() > 1e-9, "seed gives an ill-posed routing"
    assert np.array_equal(idx, ridx)
    assert np.abs(w - rw).max() <= 1e-5
    assert np.abs(lg - rlg).max() <= 1e-11 * max(1.0, np.abs(rlg).max())


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_route_small(B, cfg):
    L = make_layer(cfg)
    _check_route(B, cfg, L, L["X"])


@pytest.mark.parametrize("name", ["c1_tiny", "c2_mixtral", "c3_finegrained", "c4_dsv2lite_prefill",
                                  "c6_qwen3_a3b"])
def test_route_full_size(B, name):
    """Router at the real shapes (router weights only; no expert matrices)."""
    from workloads import make_router
    cfg = get_config(name)
    Wr, b = make_router(cfg)
    L = {"Wr": Wr, "b": b}
    for T in ([cfg.T] if name != "c2_mixtral" else [1, 8, 64, 256]):
        _check_route(B, cfg, L, make_hidden(cfg, T=T))


def test_route_logits_in_workspace(B):
    """Without logits_out the logits live in the caller's workspace between
    the two routing kernels; same indices and weights either way."""
    cfg = SMALL[3]
    L = make_layer(cfg)
    sh = _shape(B, cfg)
    idx, w, _ = _route_gpu(B, cfg, L, L["X"])
    idx2 = torch.empty((cfg.T, cfg.k), dtype=torch.int32, device="cuda")
    w2 = torch.empty((cfg.T, cfg.k), dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(sh)
    B.moe_route(sh, to_dev(L["X"]), to_dev(L["Wr"]), to_dev(L["b"]), idx2, w2, None, ws)
    torch.cuda.synchronize()
    assert np.array_equal(idx2.cpu().numpy(), idx) and np.array_equal(w2.cpu().numpy(), w)
    with pytest.raises(B.MoEError):
        B.moe_route(sh, to_dev(L["X"]), to_dev(L["Wr"]), to_dev(L["b"]), idx2, w2, None, None)


def test_route_exact_ties(B):
    """Wr = 0 makes the logits equal the bias, which repeats values: every
    round must take the lowest index among equals."""
    cfg = _small("ties", T=6, E=8, k=4)
    X = make_hidden(cfg)
    Wr = np.zeros((cfg.E, cfg.H), dtype=np.uint16)
    b = np.array([0.5, 1.0, 1.0, -1.0, 0.5, 1.0, -1.0, 0.5], dtype=np.float32)
    idx, w, lg = _route_gpu(B, cfg, {"Wr": Wr, "b": b}, X)
    ridx, rw, _ = O.route(X, Wr, b, cfg.k)
    assert np.array_equal(idx, ridx)
    assert np.all(idx == np.array([1, 2, 5, 0]))
    assert np.abs(w - rw).max() <= 1e-6
    # small-integer inputs: every precision agrees exactly, ties arise in the GEMM
    r = np.random.Generator(np.random.PCG64(7))
    Xi = r.integers(-2, 3, size=(32, cfg.H)).astype(np.float32)
    Wi = r.integers(-1, 2, size=(cfg.E, cfg.H)).astype(np.float32)
    Wi[3] = Wi[1]
    Wi[6] = Wi[1]
    from workloads import bf16_bits_from_f32
    Xb, Wb = bf16_bits_from_f32(Xi), bf16_bits_from_f32(Wi)
    idx, w, lg = _route_gpu(B, cfg, {"Wr": Wb, "b": np.zeros(cfg.E, np.float32)}, Xb)
    ridx, rw, rlg = O.route(Xb, Wb, None, cfg.k)
    assert np.array_equal(lg, rlg)
    assert np.array_equal(idx, ridx)


def test_permute(B):
    r = np.random.Generator(np.random.PCG64(11))
    for (T, E, k) in [(8, 8, 2), (1, 8, 2), (64, 8, 2), (128, 60, 4), (2048, 64, 6), (3, 128, 8),
                      (700, 5, 5), (1025, 128, 1)]:
        idx = np.stack([r.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
        if T >= 64:
            idx[:, 0] = np.where(r.random(T) < 0.5, idx[:, 0], idx[0, 0])  # skew one expert
            for t in range(T):                                             # keep rows distinct
                if len(set(idx[t])) < k:
                    idx[t] = r.permutation(E)[:k]
        sh = B.make_shape(T, 128, E, k, 128, 0, "bf16")
        A = T * k
        d = {n: torch.full((m,), -7, dtype=torch.int32, device="cuda")
             for n, m in [("count", E), ("offset", E + 1), ("perm", A), ("inv", A)]}
        B.moe_permute(sh, to_dev(idx), d["count"], d["offset"], d["perm"], d["inv"])
        torch.cuda.synchronize()
        count, offset, perm, inv = O.bucket_by_expert(idx, E)
        assert np.array_equal(d["count"].cpu().numpy(), count)
        assert np.array_equal(d["offset"].cpu().numpy(), offset)
        assert np.array_equal(d["perm"].cpu().numpy(), perm)
        assert np.array_equal(d["inv"].cpu().numpy(), inv)


def test_permute_drops_out_of_range_indices(B):
    r = np.random.Generator(np.random.PCG64(12))
    T, E, k = 300, 7, 3
    idx = r.integers(0, E, size=(T, k)).astype(np.int32)
    bad = r.random((T, k)) < 0.1
    idx[bad] = np.where(r.random(bad.sum()) < 0.5, -1, E + 3)
    sh = B.make_shape(T, 128, E, k, 128, 0, "bf16")
    A = T * k
    cnt = torch.empty(E, dtype=torch.int32, device="cuda")
    off = torch.empty(E + 1, dtype=torch.int32, device="cuda")
    perm = torch.full((A,), -7, dtype=torch.int32, device="cuda")
    inv = torch.full((A,), -7, dtype=torch.int32, device="cuda")
    B.moe_permute(sh, to_dev(idx), cnt, off, perm, inv)
    torch.cuda.synchronize()
    flat = idx.reshape(-1)
    valid = (flat >= 0) & (flat < E)
    ids = np.nonzero(valid)[0]
    want = ids[np.argsort(flat[ids], kind="stable")]
    nv = len(ids)
    assert np.array_equal(perm.cpu().numpy()[:nv], want)
    assert off.cpu().numpy()[-1] == nv
    assert np.array_equal(cnt.cpu().numpy(), np.bincount(flat[valid], minlength=E))
    invh = inv.cpu().numpy()
    assert np.all(invh[~valid] == -1)
    assert np.array_equal(invh[want], np.arange(nv))


def _ffn_and_combine(B, cfg, L, mask=None, layout="row_major"):
    """route/bucket on the CPU oracle, FFN + combine on the GPU."""
    sh = _shape(B, cfg, layout=layout)
    ridx, rw, _ = O.route(L["X"], L["Wr"], L["b"], cfg.k)
    count, offset, perm, inv = O.bucket_by_expert(ridx, cfg.E)
    rows = cfg.A + cfg.S * cfg.T
    Wg, Wu, Wd = _experts_dev(B, L, layout)
    tab = B.expert_table(sh, Wg, Wu, Wd)
    Y = torch.full((rows, cfg.H), float("nan"), dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(sh)
    X = to_dev(L["X"])
    B.moe_grouped_ffn(sh, X, to_dev(perm), to_dev(offset), tab, mask, Y, ws)
    torch.cuda.synchronize()
    Yref = O.grouped_ffn_rows(L["X"], perm, offset, cfg.k, L["Wg"], L["Wu"], L["Wd"], cfg.S)
    return sh, Y, Yref, (ridx, rw, count, offset, perm, inv), X


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_grouped_ffn_and_combine_small(B, cfg, layout):
    if layout == "tiled" and cfg.dtype != "bf16":
        pytest.skip("the tiled layout exists for bf16 storage only")
    L = make_layer(cfg)
    sh, Y, Yref, (ridx, rw, count, offset, perm, inv), X = _ffn_and_combine(B, cfg, L, layout=layout)
    Yh = Y.cpu().numpy()
    assert np.isfinite(Yh).all()
    assert row_rel_err(Yh, Yref) <= TOL[cfg.dtype]
    # combine (with and without residual) against the oracle's combine of the
    # oracle's rows, and against its combine of the GPU's own rows (tight)
    for residual in (None, L["X"]):
        out = torch.empty((cfg.T, cfg.H), dtype=X.dtype, device="cuda")
        B.moe_combine(sh, Y, to_dev(rw.astype(np.float32)), to_dev(inv),
                      None if residual is None else X, out)
        torch.cuda.synchronize()
        got = O.widen(to_host_bits(out))
        ref = O.combine_rows(Yref, rw, inv, cfg.T, cfg.k, cfg.S, residual)
        assert row_rel_err(got, ref) <= TOL[cfg.dtype]
        ref_own = O.combine_rows(Yh, rw.astype(np.float32), inv, cfg.T, cfg.k, cfg.S, residual)
        assert row_rel_err(got, ref_own) <= (4e-3 if cfg.dtype == "bf16" else 1e-6)


def test_grouped_ffn_mask_leaves_rows_untouched(B):
    cfg = SMALL[1]
    L = make_layer(cfg)
    mask = [e % 2 == 0 for e in range(cfg.E + cfg.S)]
    sh, Y, Yref, (ridx, rw, count, offset, perm, inv), X = _ffn_and_combine(B, cfg, L, mask)
    Yh = Y.cpu().numpy()
    for e in range(cfg.E + cfg.S):
        lo, hi = ((offset[e], offset[e + 1]) if e < cfg.E else
                  (cfg.A + (e - cfg.E) * cfg.T, cfg.A + (e - cfg.E + 1) * cfg.T))
        if mask[e]:
            if hi > lo:
                assert row_rel_err(Yh[lo:hi], Yref[lo:hi]) <= TOL[cfg.dtype]
        else:
            assert np.isnan(Yh[lo:hi]).all()


def test_small_tiled_kernel_splits_an_overfull_bucket(B):
    """The grouped FFN is public and takes any bucket list.  At most 64 tokens
    select the small tiled kernel, which multiplies 64-row blocks: a bucket of
    more than 64 rows (a caller's top-k list naming one expert twice per token)
    must be split into blocks, not cut off after the first."""
    cfg = _small("overfull", T=60, E=2, k=2, H=256, F=512, bias="none")
    L = make_layer(cfg)
    sh = _shape(B, cfg, layout="tiled")
    assert "small" in B.moe_ffn_kernel_name(sh, 0, cfg.E) and "small" in B.moe_ffn_kernel_name(sh, 1, cfg.E)
    A = cfg.A
    idx = np.zeros((cfg.T, cfg.k), dtype=np.int32)          # every assignment goes to expert 0
    count, offset, perm, inv = O.bucket_by_expert(idx, cfg.E)
    assert count[0] == A == 120
    Wg, Wu, Wd = _experts_dev(B, L, "tiled")
    tab = B.expert_table(sh, Wg, Wu, Wd)
    Y = torch.full((A, cfg.H), float("nan"), dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(sh)
    B.moe_grouped_ffn(sh, to_dev(L["X"]), to_dev(perm), to_dev(offset), tab, None, Y, ws)
    torch.cuda.synchronize()
    Yref = O.grouped_ffn_rows(L["X"], perm, offset, cfg.k, L["Wg"], L["Wu"], L["Wd"], 0)
    Yh = Y.cpu().numpy()
    assert np.isfinite(Yh).all()
    assert row_rel_err(Yh, Yref) <= TOL["bf16"]


def _layer_gpu(B, cfg, L, ctx=None, layout="row_major", dev_weights=None, want_rows=False, **kw):
    sh = _shape(B, cfg, L["X"].shape[0], layout=layout)
    own = ctx is None
    if own:
        ctx = B.Context(sh)
    Wg, Wu, Wd = dev_weights if dev_weights is not None else _experts_dev(B, L, layout)
    layer = B.make_layer_desc(sh, to_dev(L["Wr"]), to_dev(L["b"]), dev=(Wg, Wu, Wd))
    X = to_dev(L["X"])
    out = torch.empty_like(X)
    ws = B.alloc_workspace(sh)
    B.moe_layer_forward(ctx, sh, layer, X, out, ws, **kw)
    torch.cuda.synchronize()
    v = B.moe_workspace_views(sh, ws)
    res = {"out": O.widen(to_host_bits(out)), "topk_idx": v["topk_idx"].cpu().numpy(),
           "topk_w": v["topk_w"].cpu().numpy(), "count": v["count"].cpu().numpy()}
    if want_rows:
        res.update(Y=v["Y"].float().cpu().numpy(), offset=v["offset"].cpu().numpy(),
                   perm=v["perm"].cpu().numpy())
    if own:
        ctx.close()
    return res


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_layer_forward_small(B, cfg, layout):
    if layout == "tiled" and cfg.dtype != "bf16":
        pytest.skip("the tiled layout exists for bf16 storage only")
    L = make_layer(cfg)
    got = _layer_gpu(B, cfg, L, layout=layout)
    ref = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S)
    assert np.array_equal(got["topk_idx"], ref["topk_idx"])
    assert np.abs(got["topk_w"] - ref["topk_w"]).max() <= 1e-5
    assert row_rel_err(got["out"], ref["out"]) <= TOL[cfg.dtype]


def test_layer_forward_c1_tiny(B):
    cfg = get_config("c1_tiny")
    L = make_layer(cfg)
    got = _layer_gpu(B, cfg, L)
    ref = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S)
    assert np.array_equal(got["topk_idx"], ref["topk_idx"])
    assert np.abs(got["topk_w"] - ref["topk_w"]).max() <= 1e-5
    assert row_rel_err(got["out"], ref["out"]) <= 1e-5


@pytest.mark.parametrize("layout", LAYOUTS)
def test_layer_forward_c3_finegrained(B, layout):
    cfg = get_config("c3_finegrained")
    L = make_layer(cfg)
    got = _layer_gpu(B, cfg, L, layout=layout)
    ref = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S)
    assert np.array_equal(got["topk_idx"], ref["topk_idx"])
    assert np.abs(got["topk_w"] - ref["topk_w"]).max() <= 1e-5
    assert row_rel_err(got["out"], ref["out"]) <= TOL["bf16"]
    assert np.array_equal(got["count"], np.bincount(ref["topk_idx"].reshape(-1), minlength=cfg.E))


@pytest.mark.parametrize("layout", LAYOUTS)
def test_layer_forward_c6_qwen3_a3b(B, layout):
    """Qwen3-30B-A3B-shaped decode layer (128 experts, top-8, 9 MiB experts):
    the most fine-grained shape of Table 2, every token against the oracle."""
    cfg = get_config("c6_qwen3_a3b")
    L = make_layer(cfg)
    got = _layer_gpu(B, cfg, L, layout=layout)
    ref = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S)
    assert O.routing_margins(ref["logits"], cfg.k).min() > 1e-9
    assert np.array_equal(got["topk_idx"], ref["topk_idx"])
    assert np.abs(got["topk_w"] - ref["topk_w"]).max() <= 1e-5
    assert row_rel_err(got["out"], ref["out"]) <= TOL["bf16"]
    assert np.array_equal(got["count"], np.bincount(ref["topk_idx"].reshape(-1), minlength=cfg.E))


def _stratified_rows(offset, E, S, T, block=256, whole=()):
    """Rows of the grouped FFN's output that a tiling mistake would hit: for every
    routed expert's bucket and every shared expert's segment the first 16 and the
    last 16 rows (every position inside a 16-row tile, the ragged last tile), the
    rows on both sides of every `block`-row boundary, and every row of the groups
    named in `whole`.  Returns {group: sorted row list}."""
    A = int(offset[E])
    out = {}
    for g in range(E + S):
        lo, hi = (int(offset[g]), int(offset[g + 1])) if g < E else (A + (g - E) * T, A + (g - E + 1) * T)
        if hi <= lo:
            continue
        rows = set(range(lo, min(lo + 16, hi))) | set(range(max(hi - 16, lo), hi))
        for b in range(lo + block, hi, block):
            rows |= set(range(max(b - 2, lo), min(b + 2, hi)))
        if g in whole:
            rows |= set(range(lo, hi))
        out[g] = sorted(rows)
    return out


def _check_ffn_rows(cfg, L, X, got, rows_by_group):
    """Rows of Y against the oracle's expert FFN, one expert at a time."""
    Xd = O.widen(X)
    A = X.shape[0] * cfg.k
    worst = 0.0
    for g, rows in rows_by_group.items():
        W = (O.widen(L["Wg"][g]), O.widen(L["Wu"][g]), O.widen(L["Wd"][g]))
        for p in rows:
            t = got["perm"][p] // cfg.k if p < A else (p - A) % X.shape[0]
            if p < A:
                assert got["offset"][g] <= p < got["offset"][g + 1]
            ref = O.expert_ffn(Xd[t], *W)
            err = np.abs(got["Y"][p] - ref).max() / np.abs(ref).max()
            assert err <= TOL["bf16"], f"row {p} of group {g} (token {t}): {err}"
            worst = max(worst, err)
    return worst


@pytest.fixture(scope="module")
def c2_oracle(c2_weights):
    """Oracle results of the Mixtral-shaped layer per batch size, computed once
    for both layouts: every token at 1, 8, 10, 32 and 64 tokens (between them
    the sizes reach every decode form of the down projection at this shape:
    split-K with sixteen parts, with four parts and one or two weight tiles per
    wave, and the small tiled kernel with sparsely and with well filled blocks)."""
    cfg, L = c2_weights
    memo = {}

    def get(T):
        if T not in memo:
            X = make_hidden(cfg, T=T)
            memo[T] = (X, O.moe_layer(X, L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S))
        return memo[T]
    return get


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("T", [64, 1, 8, 10, 32])
def test_layer_forward_c2_mixtral_every_token(B, T, layout, c2_weights, c2_dev, c2_oracle):
    """Full Mixtral-shaped layer in the launch configuration the benchmark
    times: routing, gate weights and the output of EVERY token against the
    oracle (Section 2.1's block equation is per token)."""
    cfg, L = c2_weights
    X, ref = c2_oracle(T)
    assert O.routing_margins(ref["logits"], cfg.k).min() > 1e-9
    got = _layer_gpu(B, cfg, dict(L, X=X), layout=layout, dev_weights=c2_dev[layout])
    assert np.array_equal(got["topk_idx"], ref["topk_idx"])
    assert np.abs(got["topk_w"] - ref["topk_w"]).max() <= 1e-5
    assert row_rel_err(got["out"], ref["out"]) <= TOL["bf16"]
    assert np.array_equal(got["count"], np.bincount(ref["topk_idx"].reshape(-1), minlength=cfg.E))


@pytest.mark.parametrize("layout", LAYOUTS)
def test_layer_forward_c2_mixtral_256_tokens_stratified(B, layout, c2_weights, c2_dev):
    """256 tokens of the Mixtral-shaped layer (uneven buckets of 40-90 rows,
    items dealt round-robin): routing for every token; FFN rows chosen so that
    every expert's first and last 16 bucket rows are compared (every position of
    a 16-row tile, the ragged tail) plus the whole fullest and emptiest bucket;
    block outputs for the tokens that own each bucket's first and last row."""
    cfg, L = c2_weights
    T = 256
    X = make_hidden(cfg, T=T)
    got = _layer_gpu(B, cfg, dict(L, X=X), layout=layout, dev_weights=c2_dev[layout], want_rows=True)
    ridx, rw, rlg = O.route(X, L["Wr"], L["b"], cfg.k)
    assert O.routing_margins(rlg, cfg.k).min() > 1e-9
    assert np.array_equal(got["topk_idx"], ridx)
    assert np.abs(got["topk_w"] - rw).max() <= 1e-5
    count, offset, perm, inv = O.bucket_by_expert(ridx, cfg.E)
    assert np.array_equal(got["offset"], offset) and np.array_equal(got["perm"], perm)
    rows = _stratified_rows(offset, cfg.E, cfg.S, T,
                            whole=(int(np.argmax(count)), int(np.argmin(np.where(count > 0, count, 1 << 30)))))
    assert sum(len(v) for v in rows.values()) >= 32 * int((count > 0).sum())
    _check_ffn_rows(cfg, L, X, got, rows)
    ends = sorted({int(perm[p]) // cfg.k for e in range(cfg.E) if count[e]
                   for p in (offset[e], offset[e + 1] - 1)})
    ref = O.moe_layer(X, L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S, tokens=ends)
    assert row_rel_err(got["out"][ends], ref["out"][ends]) <= TOL["bf16"]


def test_layer_forward_c5_shape_streamed(B, c2_weights, c2_dev):
    """One layer of the streamed stack at its real shape (Mixtral experts,
    batch 32): half of the experts come from pinned host memory through the
    slots, two of them prefetched by an earlier call; the result must equal the
    all-resident result bit for bit and match the oracle on sampled tokens."""
    from paper_2509_23638_amd.stack import StreamedStack
    from workloads import make_residency_mask
    cfg, L = c2_weights
    cfg = cfg.with_(T=32)
    sh = _shape(B, cfg, 32)
    X = make_hidden(cfg, step=3, T=32)
    res = make_residency_mask(cfg, 0)
    ref = O.moe_layer(X, L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S, tokens=[0, 9, 31])
    active = np.bincount(ref["topk_idx"].reshape(-1), minlength=cfg.E) > 0
    stack = StreamedStack(sh, [L], [res, res], 2, 2, n_layers=2)
    Xd = to_dev(X)
    out0, out1 = torch.empty_like(Xd), torch.empty_like(Xd)
    pf = np.zeros(cfg.E, dtype=bool)
    pf[[e for e in range(cfg.E) if not res[e] and active[e]][:2]] = True
    # layer 0: everything non-resident is a miss; it also prefetches two experts for layer 1
    st0 = stack.layer_forward(0, Xd, out0, prefetch_next_mask=pf, next_l=1)
    st1 = stack.layer_forward(1, Xd, out1)            # same weights, same input
    torch.cuda.synchronize()
    n_nonres = int((active & ~res).sum())
    assert st0["n_miss"] == n_nonres and st0["n_hit"] == 0 and st0["n_prefetch_issued"] == int(pf.sum())
    assert st1["n_hit"] == int(pf.sum()) and st1["n_miss"] == n_nonres - int(pf.sum())
    full = _layer_gpu(B, cfg, dict(L, X=X), dev_weights=c2_dev["row_major"])
    got0 = O.widen(to_host_bits(out0))
    assert np.array_equal(got0, full["out"])
    assert torch.equal(out0.view(torch.int16), out1.view(torch.int16))
    assert row_rel_err(got0[[0, 9, 31]], ref["out"][[0, 9, 31]]) <= TOL["bf16"]
    stack.close()


@pytest.fixture(scope="module")
def c2_weights():
    cfg = get_config("c2_mixtral")
    return cfg, make_layer(cfg, with_hidden=False)


@pytest.fixture(scope="module")
def c2_dev(B, c2_weights):
    """The Mixtral-shaped layer's experts on the GPU, in both layouts."""
    cfg, L = c2_weights
    rm = _experts_dev(B, L, "row_major")
    return {"row_major": rm, "tiled": tuple(B.pack_experts(W) for W in rm)}


@pytest.fixture(scope="module")
def c4_case():
    """The prefill layer, its routing, and the oracle's block output for 160
    tokens: the owners of every expert's first and last bucket row plus a seeded
    random fill (computed once for both layouts)."""
    cfg = get_config("c4_dsv2lite_prefill")
    L = make_layer(cfg)
    ridx, rw, rlg = O.route(L["X"], L["Wr"], L["b"], cfg.k)
    count, offset, perm, inv = O.bucket_by_expert(ridx, cfg.E)
    ends = {int(perm[p]) // cfg.k for e in range(cfg.E) if count[e] for p in (offset[e], offset[e + 1] - 1)}
    r = np.random.Generator(np.random.PCG64(4))
    fill = [int(t) for t in r.permutation(cfg.T) if int(t) not in ends]
    tokens = sorted(ends | set(fill[:max(0, 160 - len(ends))]))
    ref = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S, tokens=tokens)
    return cfg, L, (count, offset, perm, inv), tokens, ref


@pytest.mark.parametrize("layout", LAYOUTS)
def test_layer_forward_c4_prefill_stratified(B, layout, c4_case):
    """DeepSeek-V2-Lite-shaped prefill (2048 tokens, the eight-wave kernels):
    routing for every token; rows of the grouped FFN per expert -- the first and
    last 16 rows of all 64 buckets and of both shared experts, both sides of
    every 256-row block boundary, every row of the fullest and the emptiest
    bucket (partly filled blocks) and of a shared expert (eight full blocks);
    block outputs of 160 tokens incl. the owners of every bucket's end rows."""
    cfg, L, (count, offset, perm, inv), tokens, ref = c4_case
    got = _layer_gpu(B, cfg, L, layout=layout, want_rows=True)
    assert O.routing_margins(ref["logits"], cfg.k).min() > 1e-9
    assert np.array_equal(got["topk_idx"], ref["topk_idx"])
    assert np.abs(got["topk_w"] - ref["topk_w"]).max() <= 1e-5
    assert np.array_equal(got["count"], count)
    assert np.array_equal(got["offset"], offset) and np.array_equal(got["perm"], perm)
    rows = _stratified_rows(offset, cfg.E, cfg.S, cfg.T,
                            whole=(int(np.argmax(count)), int(np.argmin(count)), cfg.E + 1))
    assert len(rows) == cfg.E + cfg.S and len(rows[cfg.E + 1]) == cfg.T
    _check_ffn_rows(cfg, L, L["X"], got, rows)
    assert len(tokens) >= 128
    assert row_rel_err(got["out"][tokens], ref["out"][tokens]) <= TOL["bf16"]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("name", ["s_bf16_filled_blocks", "s_bf16_filled_blocks_12"])
def test_prefill_layer_keeps_rows_of_y_in_bf16(B, name, layout):
    """Where the down projection runs its prefill form the block keeps Y in bf16:
    those rows must be exactly the float32 rows of moe_grouped_ffn rounded to
    nearest even (same kernel arithmetic, one more rounding), and the block's
    output must be the float32 weighted sum of the ROUNDED rows."""
    cfg = next(c for c in SMALL if c.name == name)
    L = make_layer(cfg)
    sh = _shape(B, cfg, layout=layout)
    assert B.moe_layer_y_dtype(sh) == torch.bfloat16
    assert B.moe_ffn_kernel_name(sh, 1, cfg.E + cfg.S) == "ffn_wide_kernel<down>"
    dev_w = _experts_dev(B, L, layout)
    ctx = B.Context(sh)
    layer = B.make_layer_desc(sh, to_dev(L["Wr"]), to_dev(L["b"]), dev=dev_w)
    X = to_dev(L["X"])
    out = torch.empty_like(X)
    ws = B.alloc_workspace(sh)
    B.moe_layer_forward(ctx, sh, layer, X, out, ws)
    torch.cuda.synchronize()
    v = B.moe_workspace_views(sh, ws)
    assert v["Y"].dtype == torch.bfloat16
    rows = cfg.T * cfg.k + cfg.S * cfg.T
    Y32 = torch.full((rows, cfg.H), float("nan"), dtype=torch.float32, device="cuda")
    ws2 = B.alloc_workspace(sh)
    tab = B.expert_table(sh, *dev_w)
    B.moe_grouped_ffn(sh, X, v["perm"], v["offset"], tab, None, Y32, ws2)
    torch.cuda.synchronize()
    assert torch.isfinite(Y32).all()
    assert torch.equal(v["Y"].view(torch.int16), Y32.to(torch.bfloat16).view(torch.int16))
    # the weighted sum of the rounded rows, in float64 (the kernel sums in float32 and rounds once)
    Yr = v["Y"].double().cpu().numpy()
    w = v["topk_w"].double().cpu().numpy()
    inv = v["inv_perm"].cpu().numpy().reshape(cfg.T, cfg.k)
    A = cfg.T * cfg.k
    want = (w[:, :, None] * Yr[inv]).sum(axis=1)
    for s_ in range(cfg.S):
        want += Yr[A + s_ * cfg.T:A + (s_ + 1) * cfg.T]
    got = O.widen(to_host_bits(out))
    assert row_rel_err(got, want) <= 2.0 ** -8       # one bf16 rounding of the sum
    ctx.close()


def test_small_configs_reach_every_ffn_kernel(B):
    """The element-wise parity cases above must between them run every kernel
    the grouped FFN can choose."""
    seen = set()
    for cfg in SMALL:
        sh = _shape(B, cfg, layout="tiled")
        for phase in (0, 1):
            seen.add(B.moe_ffn_kernel_name(sh, phase, cfg.E + cfg.S))
    want = {"ffn_tile_kernel<gate/up>", "ffn_tile_kernel<down>", "ffn_tile_small_kernel<gate/up>",
            "ffn_tile_small_kernel<down>", "ffn_wide_kernel<gate/up>",
            "ffn_wide_kernel<down>", "ffn_down_splitk_kernel",
            "ffn_stream_kernel<down, halved contraction>", "ffn_stream_kernel<gate/up, 64 rows>",
            "ffn_stream_kernel<down, 64 rows>", "ffn_f32_kernel<gate/up>", "ffn_f32_kernel<down>"}
    assert want <= seen, want - seen


def test_empty_batch_and_errors(B):
    cfg = SMALL[0]
    sh = _shape(B, cfg, 0)
    idx = torch.empty((0, cfg.k), dtype=torch.int32, device="cuda")
    w = torch.empty((0, cfg.k), dtype=torch.float32, device="cuda")
    L = make_layer(cfg)
    B.moe_route(sh, to_dev(L["X"][:0]), to_dev(L["Wr"]), None, idx, w)
    cnt = torch.full((cfg.E,), -1, dtype=torch.int32, device="cuda")
    off = torch.full((cfg.E + 1,), -1, dtype=torch.int32, device="cuda")
    B.moe_permute(sh, idx, cnt, off, idx.view(-1), idx.view(-1))
    torch.cuda.synchronize()
    assert not cnt.any() and not off.any()
    with pytest.raises(B.MoEError):
        B.moe_workspace_bytes(B.make_shape(4, 200, 4, 2, 384))        # H not a multiple of 128
    with pytest.raises(B.MoEError):
        B.moe_workspace_bytes(B.make_shape(4, 256, 4, 5, 384))        # k > E
    with pytest.raises(B.MoEError):
        B.moe_workspace_bytes(B.make_shape(4, 256, 200, 2, 384))      # E too large


def test_pack_weights_layout(B):
    """The tiled layout is exactly what the header says: tile (n16, ks) is one
    KiB, lane l = r + 16 g holds W[16 n16 + r][32 ks + 8 g .. + 7]."""
    r = np.random.Generator(np.random.PCG64(21))
    N, K = 48, 96
    W = r.integers(0, 65536, size=(N, K)).astype(np.uint16)
    src = to_dev(W)
    dst = torch.empty_like(src)
    B.moe_pack_weights(src, dst, N, K)
    torch.cuda.synchronize()
    got = to_host_bits(dst).reshape(-1)
    want = np.empty(N * K, dtype=np.uint16)
    for n16 in range(N // 16):
        for ks in range(K // 32):
            for lane in range(64):
                rr, g = lane % 16, lane // 16
                o = ((n16 * (K // 32) + ks) * 64 + lane) * 8
                want[o:o + 8] = W[16 * n16 + rr, 32 * ks + 8 * g: 32 * ks + 8 * g + 8]
    assert np.array_equal(got, want)
    with pytest.raises(B.MoEError):
        B.moe_pack_weights(src, dst, 40, 96)        # N not a multiple of 16
    with pytest.raises(B.MoEError):
        B.moe_workspace_bytes(B.make_shape(4, 72, 4, 2, 40, dtype="f32", layout="tiled"))


def test_batch_independence(B):
    """A token's output does not depend on what else is in the batch.  Alone in
    a batch a token is served by other kernels (other summation order), so that
    comparison is to rounding noise; inside a batch of the same size class the
    same kernels run and every output row is a fixed-order sum, so replacing the
    OTHER tokens must not change a single bit of the kept ones."""
    cfg = SMALL[0]
    L = make_layer(cfg)
    full = _layer_gpu(B, cfg, L)
    one = _layer_gpu(B, cfg, dict(L, X=L["X"][7:8]))
    assert np.array_equal(one["topk_idx"][0], full["topk_idx"][7])
    assert row_rel_err(one["out"], full["out"][7:8]) <= 1e-2
    keep = [0, 7, 13, 22, 39]
    other = make_hidden(cfg, step=77)
    X2 = other.copy()
    X2[keep] = L["X"][keep]
    mixed = _layer_gpu(B, cfg, dict(L, X=X2))
    assert not np.array_equal(mixed["out"], full["out"])
    assert np.array_equal(mixed["topk_idx"][keep], full["topk_idx"][keep])
    assert np.array_equal(mixed["topk_w"][keep], full["topk_w"][keep])
    assert np.array_equal(mixed["out"][keep], full["out"][keep])
    fewer = _layer_gpu(B, cfg, dict(L, X=np.ascontiguousarray(L["X"][:cfg.T - 1])))
    assert np.array_equal(fewer["out"], full["out"][:cfg.T - 1])


@pytest.mark.parametrize("cfg", [SMALL[0], SMALL[1], SMALL[3], SMALL[6]], ids=lambda c: c.name)
def test_token_permutation_equivariance_bitwise(B, cfg):
    """The block is defined per token (Section 2.1): shuffling the batch shuffles
    the outputs and nothing else.  Every output row is a fixed-order sum over
    the hidden / FFN dimension and over the k slots, so the bits must agree
    wherever a token lands in its bucket."""
    L = make_layer(cfg)
    order = np.random.Generator(np.random.PCG64(31)).permutation(cfg.T)
    a = _layer_gpu(B, cfg, L)
    b = _layer_gpu(B, cfg, dict(L, X=np.ascontiguousarray(L["X"][order])))
    assert np.array_equal(b["topk_idx"], a["topk_idx"][order])
    assert np.array_equal(b["topk_w"], a["topk_w"][order])
    assert np.array_equal(b["out"], a["out"][order])


@pytest.mark.parametrize("layout", LAYOUTS)
def test_down_projection_scales_linearly(B, layout):
    """Doubling every down projection (exact in bf16) doubles the block output
    exactly: the expert output is linear in Wd and the gate never sees it."""
    cfg = SMALL[1]
    L = make_layer(cfg)
    base = _layer_gpu(B, cfg, L, layout=layout)
    Wd = L["Wd"]
    Wd2 = np.where((Wd & 0x7F80) == 0, Wd, Wd + np.uint16(1 << 7)).astype(np.uint16)   # exponent + 1, zeros stay
    assert np.array_equal(O.widen(Wd2), 2.0 * O.widen(L["Wd"]))
    twice = _layer_gpu(B, cfg, dict(L, Wd=Wd2), layout=layout)
    assert np.array_equal(twice["topk_idx"], base["topk_idx"])
    assert np.array_equal(twice["out"], 2.0 * base["out"])


def test_layer_forward_random_shapes(B):
    """A seeded sweep over shapes the hand-picked cases may have missed: every
    case must route exactly and land within the bf16 bar."""
    r = np.random.Generator(np.random.PCG64(2026))
    worst, ran = 0.0, 0
    for i in range(24):
        E = int(r.choice([1, 2, 3, 4, 8, 20, 60, 64, 128]))
        k = int(r.integers(1, min(E, 8) + 1))
        S = int(r.choice([0, 0, 1, 3]))
        T = int(r.choice([1, 2, 7, 16, 33, 64, 100, 130, 257, 300, 520]))
        H = int(r.choice([128, 256, 384, 512]))
        F = int(r.choice([128, 256, 384, 640, 1408, 4096]))
        if T * (E + S) * F * H > 3e9:
            F = 128
        layout = str(r.choice(LAYOUTS))
        cfg = _small(f"rand{i}", T=T, E=E, k=k, S=S, H=H, F=F, seed=500 + i,
                     bias=str(r.choice(["none", "normal", "zipf"])), bias_scale=1.0)
        L = make_layer(cfg)
        ref = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S)
        if E > 1 and O.routing_margins(ref["logits"], cfg.k).min() <= 1e-9:
            continue
        ran += 1
        got = _layer_gpu(B, cfg, L, layout=layout)
        what = f"case {i}: {cfg} {layout}"
        assert np.array_equal(got["topk_idx"], ref["topk_idx"]), what
        assert np.abs(got["topk_w"] - ref["topk_w"]).max() <= 1e-5, what
        err = row_rel_err(got["out"], ref["out"])
        assert err <= TOL["bf16"], what
        worst = max(worst, err)
    assert worst > 0.0
    assert ran >= 22, f"only {ran} of 24 shapes had a well-posed routing"


def test_layer_forward_random_filled_shapes(B):
    """The same kind of sweep over shapes with well-filled blocks (about a
    hundred or more rows per expert, long enough contractions): the eight-wave
    tiled kernels with every pipeline remainder, split and partly filled
    blocks, shared experts, both layouts."""
    r = np.random.Generator(np.random.PCG64(4052))
    seen, ran = set(), 0
    for i in range(12):
        E = int(r.choice([1, 2, 3, 4, 6]))
        k = int(r.integers(1, min(E, 3) + 1))
        S = int(r.choice([0, 1, 2]))
        T = int(r.choice([230, 300, 411, 520, 700]))
        H = int(r.choice([512, 768, 1024]))
        F = int(r.choice([512, 640, 768, 896, 1152]))
        while T * (E + S) * F * H > 3e9:
            T = T * 2 // 3
        layout = str(r.choice(LAYOUTS))
        cfg = _small(f"filled{i}", T=T, E=E, k=k, S=S, H=H, F=F, seed=700 + i,
                     bias=str(r.choice(["none", "normal", "zipf"])), bias_scale=0.8)
        L = make_layer(cfg)
        ref = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S)
        if E > 1 and O.routing_margins(ref["logits"], cfg.k).min() <= 1e-9:
            continue
        ran += 1
        sh = _shape(B, cfg, layout=layout)
        seen.update(B.moe_ffn_kernel_name(sh, ph, cfg.E + cfg.S) for ph in (0, 1))
        got = _layer_gpu(B, cfg, L, layout=layout)
        what = f"case {i}: {cfg} {layout}"
        assert np.array_equal(got["topk_idx"], ref["topk_idx"]), what
        assert np.abs(got["topk_w"] - ref["topk_w"]).max() <= 1e-5, what
        assert row_rel_err(got["out"], ref["out"]) <= TOL["bf16"], what
    assert {"ffn_wide_kernel<gate/up>", "ffn_wide_kernel<down>"} <= seen, seen
    assert ran >= 11, f"only {ran} of 12 shapes had a well-posed routing"


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("case", [
    dict(T=40, E=8, k=2, H=256, F=512),             # decode sizes, six experts without a token
    dict(T=700, E=8, k=2, S=1, H=512, F=640),       # two buckets of 700 rows: three row blocks each
    dict(T=300, E=4, k=1, H=768, F=768),            # one expert takes every token
    dict(T=130, E=60, k=4, S=2, H=128, F=256),      # many experts, four in use
], ids=lambda c: f"T{c['T']}_E{c['E']}_k{c['k']}")
def test_layer_forward_every_token_to_the_same_experts(B, case, layout):
    """The most skewed routing there is: a router bias far above the logits
    sends every token to the same k experts, every other bucket is empty and
    the used ones hold T rows each (several row blocks at the larger sizes)."""
    cfg = _small("same_experts", seed=81, bias="none", **case)
    L = make_layer(cfg)
    b = np.zeros(cfg.E, dtype=np.float32)
    chosen = [(3 * j + 1) % cfg.E for j in range(cfg.k)]
    assert len(set(chosen)) == cfg.k
    for j, e in enumerate(chosen):
        b[e] = 40.0 + 0.75 * j
    L["b"] = b
    ref = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S)
    assert (np.sort(ref["topk_idx"], axis=1) == np.sort(chosen)).all()
    if cfg.E > cfg.k:
        assert O.routing_margins(ref["logits"], cfg.k).min() > 1e-6
    got = _layer_gpu(B, cfg, L, layout=layout)
    assert np.array_equal(got["topk_idx"], ref["topk_idx"])
    assert np.abs(got["topk_w"] - ref["topk_w"]).max() <= 1e-5
    count = np.zeros(cfg.E, dtype=np.int64)
    count[chosen] = cfg.T
    assert np.array_equal(got["count"], count)
    assert row_rel_err(got["out"], ref["out"]) <= TOL["bf16"]


@pytest.mark.parametrize("name", ["c2_mixtral", "c4_dsv2lite_prefill"])
def test_repeated_forwards_are_bit_identical(B, name):
    """Same inputs, same bits, run after run: the persistent kernels hand ring
    buffers from one work item to the next behind hand-counted waits, and a
    wait that let a stage start early would show up as run-to-run differences
    at the full sizes (many items per workgroup) long before it showed up as an
    error against the oracle."""
    cfg = get_config(name)
    L = make_layer(cfg)
    sh = _shape(B, cfg, layout="tiled")
    Wg, Wu, Wd = _experts_dev(B, L, "tiled")
    ctx = B.Context(sh)
    layer = B.make_layer_desc(sh, to_dev(L["Wr"]), to_dev(L["b"]), dev=(Wg, Wu, Wd))
    X = to_dev(L["X"])
    ws = B.alloc_workspace(sh)
    first = None
    for _ in range(25):
        out = torch.empty_like(X)
        B.moe_layer_forward(ctx, sh, layer, X, out, ws)
        torch.cuda.synchronize()
        if first is None:
            first = out
        else:
            assert torch.equal(out.view(torch.int16), first.view(torch.int16))
    ctx.close()



def test_phase_markers_count_the_layers_they_mark_and_leave_results_alone(B):
    """The measurement markers (all phases, gate/up only, gate/up on every fourth
    call) report the number of layers they marked and never change an output bit."""
    cfg = SMALL[1]
    L = make_layer(cfg)
    sh = _shape(B, cfg, L["X"].shape[0])
    ctx = B.Context(sh)
    Wg, Wu, Wd = _experts_dev(B, L, "row_major")
    layer = B.make_layer_desc(sh, to_dev(L["Wr"]), to_dev(L["b"]), dev=(Wg, Wu, Wd))
    X = to_dev(L["X"])
    ws = B.alloc_workspace(sh)
    outs = {}
    for mode, calls in ((0, 1), (1, 3), (2, 5), (3, 9)):
        out = torch.empty_like(X)
        ctx.phase_timing(mode)
        ctx.phase_times(reset=True)
        for _ in range(calls):
            B.moe_layer_forward(ctx, sh, layer, X, out, ws)
        torch.cuda.synchronize()
        t = ctx.phase_times(reset=True)
        outs[mode] = to_host_bits(out)
        want_all = calls if mode == 1 else 0
        want_gu = {0: 0, 1: 0, 2: calls, 3: (calls + 3) // 4}[mode]
        assert t["n_layers"] == want_all and t["gate_up_only_layers"] == want_gu, (mode, t)
        if want_all:
            assert min(t[k] for k in ("route_ms", "permute_ms", "gate_up_ms", "down_ms", "combine_ms")) > 0
        if want_gu:
            assert t["gate_up_only_ms"] > 0
    ctx.phase_timing(0)
    with pytest.raises(B.MoEError):
        ctx.phase_timing(4)
    for mode in (1, 2, 3):
        assert np.array_equal(outs[mode], outs[0])
    ctx.close()


@pytest.mark.gpu
def test_stage_probe_runs_and_leaves_its_inputs_alone(B):
    """The measurement aid reads its two buffers and writes nothing to global memory."""
    stages = 16
    w = torch.arange(256 * stages * 16384 // 4, dtype=torch.int32, device="cuda")
    tok = torch.arange((2 << 20) // 4, dtype=torch.int32, device="cuda")
    w0, t0 = w.clone(), tok.clone()
    for n in range(5):
        B.moe_probe_stage(w, tok, n, stages)
    torch.cuda.synchronize()
    assert torch.equal(w, w0) and torch.equal(tok, t0)
    with pytest.raises(B.MoEError):
        B.moe_probe_stage(w[:-1], tok, 1, stages)


@pytest.mark.gpu
@pytest.mark.parametrize("T", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("E,k,S", [(8, 2, 0), (8, 8, 0), (60, 4, 2), (128, 8, 0), (128, 16, 8), (1, 1, 0)])
def test_smallest_batches_are_bucketed_by_the_selecting_launch(B, E, k, S, T):
    """One token (any router), or up to four tokens when selection is a launch of its own (E > 8),
    are bucketed by the launch that selects -- there is no bucketing launch; five tokens, and two to
    four with the fused router of E <= 8, take the bucketing launch.  Either way count, offset, perm
    and inv_perm must be what the oracle's stable bucketing gives."""
    cfg = _small(f"few_{T}_{E}_{k}_{S}", T=T, E=E, k=k, S=S, H=256, F=128, bias="normal", bias_scale=1.0)
    L = make_layer(cfg)
    sh = _shape(B, cfg, T)
    ctx = B.Context(sh)
    Wg, Wu, Wd = _experts_dev(B, L, "row_major")
    layer = B.make_layer_desc(sh, to_dev(L["Wr"]), to_dev(L["b"]), dev=(Wg, Wu, Wd))
    X = to_dev(L["X"])
    out = torch.empty_like(X)
    ws = B.alloc_workspace(sh)
    ws.view(torch.uint8).fill_(0xAB)          # nothing may rely on what the workspace held
    B.moe_layer_forward(ctx, sh, layer, X, out, ws)
    torch.cuda.synchronize()
    v = B.moe_workspace_views(sh, ws)
    ref = O.moe_layer(L["X"], L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], k, S)
    if E > 1 and O.routing_margins(ref["logits"], k).min() <= 1e-9:
        pytest.skip("ill-posed routing for this seed")
    idx = v["topk_idx"].cpu().numpy()
    assert np.array_equal(idx, ref["topk_idx"])
    count, offset, perm, inv = O.bucket_by_expert(ref["topk_idx"], E)
    assert np.array_equal(v["count"].cpu().numpy(), count)
    assert np.array_equal(v["offset"].cpu().numpy(), offset)
    assert np.array_equal(v["perm"].cpu().numpy(), perm)
    assert np.array_equal(v["inv_perm"].cpu().numpy(), inv)
    assert row_rel_err(O.widen(to_host_bits(out)), ref["out"]) <= TOL["bf16"]
    ctx.close()
