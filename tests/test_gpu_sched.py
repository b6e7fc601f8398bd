"""Scheduling-side calls that touch the GPU, through the C-ABI, against the
scheduling oracle: predicted token counts and counter totals bit-exact; the
online prefetch policies must not change a single output bit."""
import numpy as np
import pytest
import torch

import oracle.moe_oracle as O
import oracle.sched_oracle as S
from workloads import MoEConfig, get_config, make_layer, make_hidden, make_residency_mask
from gpu_util import to_dev

pytestmark = pytest.mark.gpu

CFG = MoEConfig("sched_small", T=24, H=256, E=8, k=2, F=384, S=0, dtype="bf16", bias="normal",
                bias_scale=0.5, w_std=0.05, seed=7, layers=4, steps=3)


@pytest.fixture(scope="module")
def B():
    import paper_2509_23638_amd.binding as b
    return b


def _shape(B, cfg, T=None):
    return B.make_shape(cfg.T if T is None else T, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, cfg.dtype)


@pytest.mark.parametrize("name,T", [("c5_stack", 32), ("c3_finegrained", 128), ("c6_qwen3_a3b", 64),
                                    ("c4_dsv2lite_prefill", 2048), ("c2_mixtral", 1), ("c2_mixtral", 0)])
def test_predict_counts_match_oracle(B, name, T):
    """The next layer's router applied to this layer's input, at the real
    routing shapes (expert matrices play no part)."""
    cfg = get_config(name).with_(T=T, F=128)
    sh = _shape(B, cfg)
    nxt = make_layer(cfg.with_(T=1), layer=1)            # router of the "next" layer
    X = make_hidden(cfg, step=2, T=T)
    pred = torch.full((cfg.E,), -7, dtype=torch.int32, device="cuda")
    ws = B.alloc_workspace(sh)
    B.moe_predict_counts(sh, to_dev(X) if T else None, to_dev(nxt["Wr"]), to_dev(nxt["b"]), pred, ws)
    torch.cuda.synchronize()
    ref = S.gate_based_counts(X, nxt["Wr"], nxt["b"], cfg.k)
    if T:
        assert O.routing_margins(O.router_logits(X, nxt["Wr"], nxt["b"]), cfg.k).min() > 1e-9
    assert np.array_equal(pred.cpu().numpy(), ref)
    assert int(ref.sum()) == T * cfg.k


def test_counter_totals_and_hot_table(B):
    """Counter of tokens per (layer, expert) over several batches, then the
    residency choice under a budget; both equal to the oracle's."""
    cfg = CFG
    sh = _shape(B, cfg)
    layers = [make_layer(cfg, layer=l, with_hidden=False) for l in range(cfg.layers)]
    ws = B.alloc_workspace(sh)
    pred = torch.zeros(cfg.E, dtype=torch.int32, device="cuda")
    total = torch.zeros((cfg.layers, cfg.E), dtype=torch.int64, device="cuda")
    ref = np.zeros((cfg.layers, cfg.E), dtype=np.int64)
    for step in range(5):
        X = make_hidden(cfg, step=step)
        for l, L in enumerate(layers):
            B.moe_predict_counts(sh, to_dev(X), to_dev(L["Wr"]), to_dev(L["b"]), pred, ws)
            B.moe_counter_add(sh, pred, total[l])
            ref[l] += S.gate_based_counts(X, L["Wr"], L["b"], cfg.k)
    torch.cuda.synchronize()
    got = total.cpu().numpy()
    assert np.array_equal(got, ref)
    for budget in (0, 5, cfg.layers * cfg.E // 2, cfg.layers * cfg.E):
        assert np.array_equal(B.moe_hot_table(got, budget), S.hot_expert_table(ref, budget))


@pytest.mark.parametrize("policy", ["gate_topn", "presched", "none"])
def test_online_policies_leave_the_output_bitwise_unchanged(B, policy):
    from paper_2509_23638_amd.stack import StreamedStack
    cfg = CFG
    sh = _shape(B, cfg)
    layers = [make_layer(cfg, layer=l, with_hidden=False) for l in range(cfg.layers)]
    ref_stack = StreamedStack(sh, layers, [[True] * cfg.E] * cfg.layers, 0, 0)
    res = [make_residency_mask(cfg, l) for l in range(cfg.layers)]
    stack = StreamedStack(sh, layers, res, 2, 2)
    # a window of 2.4 loads opens after each layer: PreSched plans two prefetches
    costs = B.moe_presched_costs(t_io=1.0, t_g=0.1, t_attn=100.0, beta=0.0, C=0.0, alpha=0.0,
                                 r_hit=0.9, cpu_executor=0)
    issued = hits = 0
    for step in range(cfg.steps):
        X = to_dev(make_hidden(cfg, step=step))
        want, _ = ref_stack.step(X, want_stats=False)
        want = want.clone()
        got, stats = stack.step_online(X, policy, costs=costs, n_prefetch=2, wrap_prefetch=True)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), want.view(torch.int16))
        for l, st in enumerate(stats):
            assert st["n_hit"] + st["n_miss"] + st["n_resident"] == st["n_active"]
            issued += st["n_prefetch_issued"]
            hits += st["n_hit"]
    if policy == "none":
        assert issued == 0 and hits == 0
    else:
        assert 0 < hits <= issued
    if policy == "presched":
        assert stack.sched_log["n_decisions"] == cfg.steps * cfg.layers
    # and without stats (no host wait where every non-resident expert was prefetched)
    X = to_dev(make_hidden(cfg, step=0))
    want, _ = ref_stack.step(X, want_stats=False)
    want = want.clone()
    got, stats = stack.step_online(X, policy, costs=costs, n_prefetch=2, wrap_prefetch=True,
                                   want_stats=False)
    torch.cuda.synchronize()
    assert stats == [] and torch.equal(got.view(torch.int16), want.view(torch.int16))
    stack.close()
    ref_stack.close()
