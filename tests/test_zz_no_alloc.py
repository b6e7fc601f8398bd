"""The block for callers that cannot allocate: moe_layer_forward_static keeps
its workspace in a fixed device array inside the library.  Its output must be
bit for bit that of moe_layer_forward on the same inputs -- on two calls in a
row, the second with a smaller batch (the array keeps the first call's
contents), and for a shape that does not fit the array it must refuse."""
import numpy as np
import pytest
import torch

from workloads import MoEConfig, get_config, make_layer, make_hidden
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import paper_2509_23638_amd.binding as b
    return b


CASES = [
    # (config, first batch, second smaller batch, layout)
    (MoEConfig("na_tiled_small", T=64, H=512, E=8, k=2, F=8192, S=1, dtype="bf16", bias="normal",
               bias_scale=0.5, w_std=0.05, seed=11), 64, 17, "tiled"),
    (MoEConfig("na_stream", T=48, H=256, E=60, k=4, F=384, S=2, dtype="bf16", bias="zipf",
               bias_scale=1.1, w_std=0.05, seed=12), 48, 5, "row_major"),
    (get_config("c1_tiny"), 8, 3, "row_major"),
    (get_config("c3_finegrained"), 128, 40, "tiled"),
]


@pytest.mark.parametrize("cfg,T1,T2,layout", CASES, ids=lambda c: getattr(c, "name", str(c)))
def test_static_workspace_entry_point_matches_layer_forward(B, cfg, T1, T2, layout):
    L = make_layer(cfg, with_hidden=False)
    lay = layout if cfg.dtype == "bf16" else "row_major"
    W = [to_dev(L["Wg"]), to_dev(L["Wu"]), to_dev(L["Wd"])]
    if lay == "tiled":
        W = [B.pack_experts(w) for w in W]
    Wr, b = to_dev(L["Wr"]), to_dev(L["b"])
    for T in (T1, T2):                       # two calls in a row, the second smaller
        sh = B.make_shape(T, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, cfg.dtype, lay)
        assert B.moe_workspace_bytes(sh) - 256 <= B.moe_static_workspace_bytes()
        layer = B.make_layer_desc(sh, Wr, b, dev=tuple(W))
        X = to_dev(make_hidden(cfg, step=T, T=T))
        for residual in (None, X):
            ref = torch.empty_like(X)
            ctx = B.Context(sh)
            ws = B.alloc_workspace(sh)
            B.moe_layer_forward(ctx, sh, layer, X, ref, ws, residual=residual)
            torch.cuda.synchronize()
            ctx.close()
            got = torch.full_like(X, float("nan"))
            B.moe_layer_forward_static(sh, layer, X, got, residual=residual)
            torch.cuda.synchronize()
            assert torch.isfinite(got.float()).all()
            bits = torch.int16 if got.dtype == torch.bfloat16 else torch.int32
            assert torch.equal(got.view(bits), ref.view(bits)), f"T={T} residual={residual is not None}"


def test_static_workspace_entry_point_rejects_what_does_not_fit(B):
    cfg = get_config("c2_mixtral")
    sh = B.make_shape(256, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, cfg.dtype, "tiled")
    assert B.moe_workspace_bytes(sh) - 256 > B.moe_static_workspace_bytes()
    Wr = torch.zeros((cfg.E, cfg.H), dtype=torch.bfloat16, device="cuda")
    one = torch.zeros(8, dtype=torch.bfloat16, device="cuda")        # never read: the call must refuse first
    layer = B.moe_layer_desc()
    tab = (B.moe_expert_ptrs * cfg.E)()
    for e in range(cfg.E):
        tab[e].Wg = tab[e].Wu = tab[e].Wd = one.data_ptr()
    layer.Wr, layer.host_dev = Wr.data_ptr(), tab
    X = torch.zeros((256, cfg.H), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.MoEError) as ei:
        B.moe_layer_forward_static(sh, B.Layer(layer, (Wr, one, tab)), X, torch.empty_like(X))
    assert ei.value.status == -3 and "fixed array" in str(ei.value)
    # a missing expert is an argument error, not a fault
    sh2 = B.make_shape(8, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, cfg.dtype, "tiled")
    tab[3].Wu = None
    with pytest.raises(B.MoEError) as ei:
        B.moe_layer_forward_static(sh2, B.Layer(layer, (Wr, one, tab)), X[:8], torch.empty_like(X[:8]))
    assert ei.value.status == -1
