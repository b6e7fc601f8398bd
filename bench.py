#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

A step = one pass of the whole hot path (route -> permute -> grouped FFN ->
combine, i.e. one moe_layer_forward) over one batch of synthetic decode tokens
of the Mixtral-8x7B-shaped layer (hidden 4096, 8 experts, top-2, FFN 14336,
bf16 storage, fp32 accumulate), all experts resident in HBM.  Successive steps
rotate over several distinct weight sets so that no step finds its weights in
the 256 MB last-level cache.

Prints ONE JSON line.  `value` = tokens/s of the whole layer with inputs
already in HBM (mean over the K timed steps; `ms_per_step_median` comes from
a second, untimed pass with one event pair per step).  `roofline` prices the
dominant kernel (gate/up weight stream) against the 8 TB/s HBM peak using its
algorithmic bytes and its average duration measured with HIP events recorded
between the kernels inside the timed region (on every fourth step: an event
pair costs its step about 5 us); `roofline.layer` prices the whole
layer step the same way; `roofline.traffic` is read from the committed counter
summaries under profiles/ and is null unless one was measured on this very
kernel, workload and library version.  `cpu_baseline` times the fp64 CPU
oracle on a bounded sample of the same batch on this machine's host cores, and
`parity_err` compares the timed configuration's output with those oracle rows.
`other_workloads` appends short runs of the Mixtral batch sweep (1, 8, 256
tokens) and of the fine-grained, prefill and Qwen3-shaped layers.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--tokens", type=int, default=64, help="decode batch (tokens per step)")
    ap.add_argument("--tokens-all", action="store_true",
                    help="apply --tokens to every single-layer workload, not only to c2_mixtral")
    ap.add_argument("--weight-sets", type=int, default=3,
                    help="distinct layers' weights rotated through (cache defeat)")
    ap.add_argument("--workload", default="c2_mixtral",
                    choices=["c2_mixtral", "c3_finegrained", "c4_dsv2lite_prefill", "c5_stack",
                             "c6_qwen3_a3b"])
    ap.add_argument("--weight-period", type=int, default=4,
                    help="c5_stack: distinct layers' weights; layer l uses set l %% period")
    ap.add_argument("--c5-steps", type=int, default=16)
    ap.add_argument("--c5-layers", type=int, default=32)
    ap.add_argument("--c5-policy", default="noisy_top2",
                    choices=["noisy_top2", "gate_top2", "presched", "none"],
                    help="c5_stack prefetch policy: noisy copy of the true next-layer logits "
                         "(default), gate-based prediction, gate-based prediction + PreSched, "
                         "or on-demand loads only")
    ap.add_argument("--c5-residency", default="random", choices=["random", "hot"],
                    help="c5_stack resident experts: seeded 4 of 8 per layer, or the hot-expert "
                         "table of a profiling pass under the same budget")
    ap.add_argument("--c5-profile-steps", type=int, default=8)
    ap.add_argument("--c5-tokens", type=int, default=None,
                    help="c5_stack batch (default: the shape's own)")
    ap.add_argument("--c5-shape", default="c5_stack",
                    choices=["c5_stack", "c4_dsv2lite_prefill", "c6_qwen3_a3b", "c3_finegrained"],
                    help="c5_stack: layer shape of the streamed stack (default: Mixtral-shaped)")
    ap.add_argument("--c5-resident", type=int, default=None,
                    help="c5_stack: resident experts per layer (default: half)")
    ap.add_argument("--c5-prefetch-n", type=int, default=2,
                    help="c5_stack: experts prefetched per layer by the fixed-count policies")
    ap.add_argument("--c5-step-log", action="store_true", help="c5_stack: report wall time per step")
    ap.add_argument("--c5-repeat", type=int, default=1,
                    help="c5_stack: run the timed streamed pass this many times, report the last")
    ap.add_argument("--no-c5-warm", action="store_true",
                    help="c5_stack: skip the load-time pass that touches every pinned block once")
    ap.add_argument("--no-c5-controls", action="store_true",
                    help="c5_stack: skip the synchronous-copy and three-copies-per-expert reruns")
    ap.add_argument("--layout", default="tiled", choices=["tiled", "row_major"],
                    help="expert weight layout in HBM (tiled = packed once at load time)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the batch sweep and the other layer shapes")
    ap.add_argument("--other-steps", type=int, default=20)
    ap.add_argument("--probe", action="store_true",
                    help="also time a plain 1 GiB copy and a 4 GiB read (achievable HBM rate)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="0 = auto")
    return ap.parse_args()


def cpu_baseline(cfg, L, X, n_tokens):
    """The oracle as it stands, on a bounded sample of this batch."""
    import oracle.moe_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    # a short probe sizes the sample to roughly 20 s of CPU work
    probe = list(range(min(2, X.shape[0])))
    t0 = time.perf_counter()
    O.moe_layer(X, L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S, tokens=probe)
    per_tok = (time.perf_counter() - t0) / len(probe)
    if not n_tokens:
        n_tokens = int(max(2, min(X.shape[0], 20.0 / max(per_tok, 1e-6))))
    sample = list(range(min(n_tokens, X.shape[0])))
    t0 = time.perf_counter()
    ref = O.moe_layer(X, L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S, tokens=sample)
    dt = time.perf_counter() - t0
    return {"value": len(sample) / dt, "unit": "tokens/s", "cores": cores, "cpu_model": cpu_model(),
            "kind": "oracle",
            "sample": f"{len(sample)} of the batch's {X.shape[0]} tokens through the fp64 oracle "
                      f"(routing for all tokens, experts for the sample), {dt:.1f} s wall",
            "_ref": ref, "_sample": sample}


def hbm_probe(torch, B):
    """Plain streaming kernels of known size: achievable HBM rate of this machine."""
    out = {}
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    big = torch.empty(4 << 30, dtype=torch.uint8, device="cuda")
    big.view(torch.int32).random_(0, 1 << 30)
    sink = torch.zeros(4, dtype=torch.uint8, device="cuda")
    for name, fn, nbytes in (("copy_1GiB", lambda: B.moe_probe_copy(dst, src), 2 * (1 << 30)),
                             ("read_4GiB", lambda: B.moe_probe_read(big, sink), 4 << 30),
                             ("read_nt_4GiB", lambda: B.moe_probe_read_nt(big, sink), 4 << 30)):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name + "_GBps"] = nbytes * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    # the tiled kernels' stage loop on its own: 16 KiB of weights per stage and compute unit out of HBM,
    # beside 0 .. 32 KiB of token rows out of L2 (what bytes that hit in L2 cost an HBM-bound stream)
    stages = 448
    tokens = torch.zeros(2 << 20, dtype=torch.uint8, device="cuda")
    wbytes = 256 * stages * 16384
    for n in range(5):
        for _ in range(2):
            B.moe_probe_stage(big[:wbytes], tokens, n, stages)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            B.moe_probe_stage(big[:wbytes], tokens, n, stages)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / 5
        out[f"stage_loop_{8 * n}KiB_tokens"] = {"us_per_stage": us / stages, "weights_GBps": wbytes / us / 1e3}
    return out


def run_c5(args, torch, B):
    """Streamed 32-layer stack: half of every layer's experts live in pinned
    host memory.  Reports the link-bound throughput and the overlap metrics."""
    from workloads import get_config, make_layer, make_hidden, make_residency_mask, make_prefetch_noise
    from paper_2509_23638_amd.stack import StreamedStack, noisy_topk_prefetch_mask, _to_torch

    cfg = get_config(args.c5_shape)
    if args.c5_tokens:
        cfg = cfg.with_(T=args.c5_tokens)
    NL, NS, T, E = args.c5_layers, args.c5_steps, cfg.T, cfg.E
    NPF = args.c5_prefetch_n
    sh = B.make_shape(T, cfg.H, E, cfg.k, cfg.F, cfg.S, cfg.dtype, args.layout)
    P = min(args.weight_period, NL)
    hosts = [make_layer(cfg, layer=p, with_hidden=False, threads=16) for p in range(P)]
    res = [make_residency_mask(cfg, l, args.c5_resident) for l in range(NL)]
    ref = StreamedStack(sh, hosts, [[True] * E] * NL, 0, 0, n_layers=NL)
    hot_info = None
    if args.c5_residency == "hot":
        # Section 4.1: count tokens per (layer, expert) over profiling batches (other
        # seeds than the timed steps), keep the hottest resident under the same budget
        total = torch.zeros((NL, E), dtype=torch.int64, device="cuda")
        views = B.moe_workspace_views(sh, ref.ws)
        norm = torch.empty((T, cfg.H), dtype=torch.bfloat16, device="cuda")
        bufs = [torch.empty_like(norm), torch.empty_like(norm)]
        for s_ in range(args.c5_profile_steps):
            x = _to_torch(make_hidden(cfg, step=1000 + s_)).cuda()
            for l in range(NL):
                B.moe_rmsnorm(sh, x, norm)
                ref.layer_forward(l, norm, bufs[l & 1], residual=x, want_stats=False)
                B.moe_counter_add(sh, views["count"], total[l])
                x = bufs[l & 1]
        torch.cuda.synchronize()
        budget = int(sum(int(np.sum(m)) for m in res))
        tok = total.cpu().numpy()
        hot = B.moe_hot_table(tok, budget)
        hot_info = {"budget_experts": budget, "profile_steps": args.c5_profile_steps,
                    "tokens_covered_by_random_masks": int(sum(tok[l][res[l]].sum() for l in range(NL))),
                    "tokens_covered_by_hot_table": int(tok[hot].sum()), "tokens_total": int(tok.sum()),
                    "resident_per_layer_min_max": [int(hot.sum(1).min()), int(hot.sum(1).max())]}
        res = [hot[l] for l in range(NL)]
    stack = StreamedStack(sh, hosts, res, 2, max(NPF, 1), n_layers=NL)
    if not args.no_c5_warm:
        stack.warm_host_copies()       # load time: every pinned block crosses the link once
    Xs = [_to_torch(make_hidden(cfg, step=s)).cuda() for s in range(NS)]

    # recorded all-resident pass: true router logits of every (step, layer)
    lg = torch.empty((T, E), dtype=torch.float64, device="cuda")
    idx = torch.empty((T, cfg.k), dtype=torch.int32, device="cuda")
    w = torch.empty((T, cfg.k), dtype=torch.float32, device="cuda")
    logits = [[None] * NL for _ in range(NS)]
    finals = []
    norm, bufs = torch.empty_like(Xs[0]), [torch.empty_like(Xs[0]), torch.empty_like(Xs[0])]
    for s in range(NS):
        x = Xs[s]
        for l in range(NL):
            B.moe_rmsnorm(sh, x, norm)
            B.moe_route(sh, norm, ref.layers[l].keep[0], ref.layers[l].keep[1], idx, w, lg)
            logits[s][l] = lg.cpu().numpy()
            ref.layer_forward(l, norm, bufs[l & 1], residual=x, want_stats=False)
            x = bufs[l & 1]
        finals.append(x.clone())
    torch.cuda.synchronize()

    # prefetch masks: issued at layer l for layer l+1 (last layer: layer 0 of the next step)
    masks = [[None] * NL for _ in range(NS)]
    for s in range(NS):
        for l in range(NL):
            ns, nl = (s, l + 1) if l + 1 < NL else (s + 1, 0)
            if ns >= NS:
                continue
            noise = make_prefetch_noise(cfg, nl, ns)
            masks[s][l] = noisy_topk_prefetch_mask(logits[ns][nl], noise, cfg.k, NPF, res[nl])

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = fn()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, out

    def run_ref():
        for s in range(NS):
            ref.step(Xs[s], want_stats=False)

    costs = B.moe_presched_costs(t_io=1.0, t_g=0.0, t_attn=0.0, beta=0.0, C=0.0, alpha=0.0,
                                 r_hit=0.5, cpu_executor=0)

    step_log = []

    def run_streamed(want_stats=True):
        """One pass over all steps.  With want_stats the per-layer hit/miss counts come
        back (every layer then waits on the host for the router's counts); without, a
        layer whose non-resident experts are all prefetched never blocks the host."""
        agg = {"n_active": 0, "n_resident": 0, "n_hit": 0, "n_miss": 0, "n_wasted": 0,
               "n_prefetch_issued": 0, "bytes_on_demand": 0, "bytes_prefetch": 0}
        same = True
        t_prev = time.perf_counter()
        for s in range(NS):
            if args.c5_policy == "noisy_top2":
                x, st = stack.step(Xs[s], prefetch_masks=masks[s], wrap_prefetch=s + 1 < NS,
                                   want_stats=want_stats)
                st = st if want_stats else []
            else:
                if agg["n_prefetch_issued"]:
                    # hit rate of the prefetches so far, as the Timer/Counter would report it
                    costs.r_hit = agg["n_hit"] / agg["n_prefetch_issued"]
                pol = {"gate_top2": "gate_topn", "presched": "presched", "none": "none"}[args.c5_policy]
                x, st = stack.step_online(Xs[s], pol, costs=costs, n_prefetch=NPF,
                                          wrap_prefetch=False, want_stats=want_stats)
            for d in st:
                for k_ in agg:
                    agg[k_] += d[k_]
            same = same and bool(torch.equal(x.view(torch.int16), finals[s].view(torch.int16)))
            if args.c5_step_log:      # per-step wall time (the comparison above synchronises)
                now = time.perf_counter()
                step_log.append(round((now - t_prev) * 1e3, 3))
                t_prev = now
        return agg, same

    run_ref()
    t_c, _ = timed(run_ref)
    # Timer inputs of PreSched, measured: one layer's compute, one expert's load
    t_layer = t_c / (NS * NL)
    # (one untimed streamed step, prefetches included: it also absorbs the one-time cost
    # of the first cross-stream waits, ~80 ms in a fresh process)
    stack.step(Xs[0], prefetch_masks=masks[0], want_stats=False)
    torch.cuda.synchronize()
    # the load time of one expert, from a step whose copies run alone on the link
    stack.ctx.set_sync_copies(True)
    stack.ctx.stream_totals(reset=True)
    stack.step(Xs[0], prefetch_masks=masks[0], want_stats=False)
    torch.cuda.synchronize()
    cal = stack.ctx.stream_totals(reset=True)
    stack.ctx.set_sync_copies(False)
    costs.t_io = cal["copy_ms"] * 1e-3 / max(1, cal["n_copies"])
    costs.t_g = t_layer / E
    costs.t_attn = t_layer          # the only time per layer the link has no on-demand work
    # hit / miss accounting from an untimed pass with stats; the timed passes run without
    # (a layer whose non-resident experts were all prefetched then needs no host wait; the
    # online policies wait for their prediction only after the layer has been queued)
    _, (agg, same0) = timed(run_streamed)
    stack.ctx.stream_totals(reset=True)
    fast = True
    earlier = []
    for rep in range(args.c5_repeat):
        t_wall, (agg_t, same) = timed(lambda: run_streamed(want_stats=not fast))
        same = same and same0
        tot = stack.ctx.stream_totals(reset=True)
        earlier.append({"T_wall_s": t_wall, "T_x_s": tot["copy_ms"] * 1e-3})
    t_x = tot["copy_ms"] * 1e-3
    sched_log = dict(stack.sched_log)
    if args.no_c5_controls:
        t_sync, same2, tot2 = None, True, {"bytes": 0, "copy_ms": 0.0}
        t_wall3, same3, tot3 = None, True, {"bytes": 0, "copy_ms": 0.0}
    else:
        stack.ctx.set_sync_copies(True)
        t_sync, (agg2, same2) = timed(lambda: run_streamed(want_stats=not fast))
        tot2 = stack.ctx.stream_totals(reset=True)
        stack.ctx.set_sync_copies(False)
        # Section 4.4's sub-tensor granularity: three copies per expert, phase 1 gated on gate+up
        stack.ctx.set_copy_split(3)
        t_wall3, (agg3, same3) = timed(lambda: run_streamed(want_stats=not fast))
        tot3 = stack.ctx.stream_totals(reset=True)
        stack.ctx.set_copy_split(1)

    tokens = T * NS
    res_json = {
        "metric": f"streamed MoE stack tokens/sec ({NL}-layer {args.c5_shape}-shaped stack, batch {T}, "
                  f"{int(np.sum(res[0]))} of {E} routed experts per layer resident, the rest in pinned host memory)",
        "value": tokens / t_wall, "unit": "tokens/s", "n_gpus": 1, "steps": NS, "warmup": 0,
        "ms_per_step": t_wall / NS * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"c5_stack ({args.c5_shape} layers): {NL} layers x {NS} steps, T={T}, weights repeat "
                               f"with period {P} layers, 2 on-demand + 2x{max(NPF, 1)} prefetch slots, "
                               f"{args.layout} weight layout, prefetch policy {args.c5_policy}, "
                               f"{args.c5_residency} residency"},
        "prefetch": {"policy": args.c5_policy, "issued": agg["n_prefetch_issued"], "hits": agg["n_hit"],
                     "wasted": agg["n_wasted"], "misses": agg["n_miss"],
                     "hit_rate_of_issued": agg["n_hit"] / agg["n_prefetch_issued"]
                     if agg["n_prefetch_issued"] else None,
                     "presched": {"t_io_ms": costs.t_io * 1e3, "t_g_ms": costs.t_g * 1e3,
                                  "t_attn_ms": costs.t_attn * 1e3, **sched_log}
                     if args.c5_policy == "presched" else None},
        "hot_table": hot_info,
        "overlap": {
            "T_c_s": t_c, "T_x_s": t_x, "T_wall_s": t_wall, "T_wall_sync_s": t_sync,
            "hidden_literal_A": 1.0 - (t_wall - t_c) / t_x if t_x > 0 else None,
            "A_ceiling_Tc_over_Tx": t_c / t_x if t_x > 0 else None,
            "B1_overlap_efficiency": (t_c + t_x - t_wall) / min(t_c, t_x) if t_x > 0 else None,
            "B2_link_busy_fraction": t_x / t_wall,
            "B2_wire_time_fraction": (tot["bytes"] / (tot2["bytes"] / (tot2["copy_ms"] * 1e-3))) / t_wall
            if tot2["copy_ms"] else None,
            "B3_h2d_GBps_per_copy": tot["bytes"] / t_x / 1e9 if t_x > 0 else None,
            "h2d_bytes": tot["bytes"], "n_copies": tot["n_copies"],
            "sync_control_h2d_GBps": tot2["bytes"] / (tot2["copy_ms"] * 1e-3) / 1e9 if tot2["copy_ms"] else None,
        },
        "three_copies_per_expert": {
            "T_wall_s": t_wall3, "T_x_s": tot3["copy_ms"] * 1e-3,
            "h2d_GBps_per_copy": tot3["bytes"] / (tot3["copy_ms"] * 1e-3) / 1e9 if tot3["copy_ms"] else None,
            "B1_overlap_efficiency": (t_c + tot3["copy_ms"] * 1e-3 - t_wall3) / min(t_c, tot3["copy_ms"] * 1e-3)
            if tot3["copy_ms"] else None},
        "stats": agg,
        "bitwise_equal_to_all_resident": bool(same and same2 and same3),
        "timed_passes": earlier, "step_wall_ms": step_log or None,
    }
    ref.close()
    stack.close()
    print(json.dumps(res_json))


def traffic_from_profiles(kernel, workload, T, layout, lib):
    """HBM bytes per launch of `kernel` from the committed counter summaries
    (profiles/*.md): lines of the form
        traffic_bytes: kernel=<name> workload=<w> tokens=<T> layout=<l> lib=<version> total=<bytes>
    (no blanks inside a value: blanks of the version string are written as underscores)
    written next to the rocprofv3 --pmc tables they summarise.  A figure is only
    reported for the very kernel, workload and library version it was measured
    on; anything else (a changed kernel bumps the version) gives None."""
    import glob
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        for line in open(path):
            if not line.startswith("traffic_bytes:"):
                continue
            kv = dict(tok.split("=", 1) for tok in line.split()[1:] if "=" in tok)
            if (kv.get("kernel") == kernel and kv.get("workload") == workload
                    and kv.get("tokens") == str(T) and kv.get("layout") == layout
                    and kv.get("lib") == lib.replace(" ", "_")):
                return {"bytes": int(kv["total"]), "source": os.path.relpath(path, ROOT)}
    return None


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def run_layer(args, torch, B, workload, T, steps, warmup, weight_sets, headline):
    """One single-layer workload: K timed steps of the whole hot path."""
    from workloads import get_config, make_layer, make_hidden
    cfg = get_config(workload).with_(T=T)
    sh = B.make_shape(T, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, cfg.dtype, args.layout)

    def dev(a):
        t = torch.from_numpy(a.view(np.int16)).view(torch.bfloat16) if a.dtype == np.uint16 \
            else torch.from_numpy(a)
        return t.cuda()

    layers, host0 = [], None
    for i in range(weight_sets):
        L = make_layer(cfg, layer=i, with_hidden=False, threads=16)
        if i == 0 and headline:
            host0 = L
        Wg, Wu, Wd = dev(L["Wg"]), dev(L["Wu"]), dev(L["Wd"])
        if args.layout == "tiled":   # the one-time load-time re-layout, outside the timed region
            Wg, Wu, Wd = B.pack_experts(Wg), B.pack_experts(Wu), B.pack_experts(Wd)
        layers.append(B.make_layer_desc(sh, dev(L["Wr"]), dev(L["b"]), dev=(Wg, Wu, Wd), layer_id=i))
        del L
    Xh = make_hidden(cfg, step=0, T=T)
    X = dev(Xh)
    out = torch.empty_like(X)
    ws = B.alloc_workspace(sh)
    ctx = B.Context(sh)
    views = B.moe_workspace_views(sh, ws)

    # active experts per weight set (decides the algorithmic bytes)
    n_active = []
    for L in layers:
        B.moe_layer_forward(ctx, sh, L, X, out, ws)
        torch.cuda.synchronize()
        n_active.append(int((views["count"] > 0).sum().item()))

    es = cfg.itemsize
    rows = cfg.rows
    ys = 2 if B.moe_layer_y_dtype(sh) == torch.bfloat16 else 4   # bytes per element of Y in this block

    def gate_up_bytes(na):
        return (na + cfg.S) * 2 * cfg.F * cfg.H * es + T * cfg.H * es + rows * cfg.F * es

    def layer_bytes(na):
        return ((na + cfg.S) * 3 * cfg.F * cfg.H * es      # expert weights, once
                + 2 * T * cfg.H * es                        # X in, out
                + cfg.E * cfg.H * es                        # router weights
                + 2 * rows * cfg.F * es                     # h written, read
                + 2 * rows * cfg.H * ys)                    # Y written, read

    for i in range(warmup):
        B.moe_layer_forward(ctx, sh, layers[i % len(layers)], X, out, ws)
    torch.cuda.synchronize()

    # the timed region: K layer steps; on every fourth of them two HIP event markers
    # around the dominant kernel (gate/up), recorded on the kernels' own stream (a
    # pair costs about 5 us of the step it is in)
    ctx.phase_timing(3)
    ctx.phase_times(reset=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        B.moe_layer_forward(ctx, sh, layers[i % len(layers)], X, out, ws)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ph2 = ctx.phase_times(reset=True)
    ctx.phase_timing(0)
    # informational passes outside the timed region: one event pair per step (median
    # step time), then all five phases (six markers per step)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
             for _ in range(steps)]
    for i, (e0, e1) in enumerate(pairs):
        e0.record()
        B.moe_layer_forward(ctx, sh, layers[i % len(layers)], X, out, ws)
        e1.record()
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in pairs)
    ctx.phase_timing(1)
    for i in range(steps):
        B.moe_layer_forward(ctx, sh, layers[i % len(layers)], X, out, ws)
    torch.cuda.synchronize()
    ph = ctx.phase_times(reset=True)
    ctx.phase_timing(0)

    ms_per_step = dt / steps * 1e3
    used = [n_active[i % len(layers)] for i in range(steps)]
    # the marked launches are those of steps 0, 4, 8, ...: their bytes
    gu_bytes = float(np.mean([gate_up_bytes(n) for n in used[::4]]))
    all_bytes = float(np.mean([layer_bytes(n) for n in used]))
    flops = 6.0 * rows * cfg.H * cfg.F
    gu_ms = ph2["gate_up_only_ms"] / max(1, ph2["gate_up_only_layers"])
    achieved = gu_bytes / (gu_ms * 1e-3) / 1e9 if gu_ms > 0 else 0.0
    kernel = B.moe_ffn_kernel_name(sh, 0, cfg.E + cfg.S)
    tr = traffic_from_profiles(kernel, workload, T, args.layout, B.moe_version())
    res = {
        "workload": workload, "tokens": T, "ms_per_step": ms_per_step,
        "ms_per_step_median": per_step[len(per_step) // 2],
        "tokens_per_s": T / (ms_per_step / 1e3), "active_experts": float(np.mean(used)),
        "kernels": {"gate_up": kernel, "down": B.moe_ffn_kernel_name(sh, 1, cfg.E + cfg.S)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": tr["bytes"] if tr else None,
                     "traffic_source": tr["source"] if tr else None,
                     "kernel": kernel, "kernel_ms": gu_ms, "kernel_launches_timed": int(ph2["gate_up_only_layers"]),
                     "algorithmic_bytes": gu_bytes,
                     "layer": {"algorithmic_bytes": all_bytes,
                               "achieved": all_bytes / (ms_per_step * 1e-3) / 1e9,
                               "frac": all_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                               "flops": flops,
                               "mfma_frac": flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}},
        "phases_ms": {k: ph[k] / max(1, ph["n_layers"]) for k in
                      ("route_ms", "permute_ms", "gate_up_ms", "down_ms", "combine_ms")},
    }
    if headline:
        res["_cfg"], res["_host0"], res["_Xh"] = cfg, host0, Xh
        # the timed configuration's own output on weight set 0, for the parity figure
        B.moe_layer_forward(ctx, sh, layers[0], X, out, ws)
        torch.cuda.synchronize()
        res["_out"] = out.cpu()
        res["_topk_idx"] = views["topk_idx"].cpu().numpy().copy()
        if args.probe:
            res["hbm_probe"] = hbm_probe(torch, B)
    ctx.close()
    del layers, ws, X, out
    torch.cuda.empty_cache()
    return res


def parity_of_timed_output(res, base):
    """Row-normalised error of the timed configuration's output against the
    oracle rows the cpu_baseline leg computed (same weights, same tokens)."""
    import torch
    import oracle.moe_oracle as O
    ref, sample = base.pop("_ref"), base.pop("_sample")
    got = res["_out"]
    got = O.widen(got.view(torch.int16).numpy().view(np.uint16)) if got.dtype == torch.bfloat16 \
        else got.numpy().astype(np.float64)
    num = np.abs(got[sample] - ref["out"][sample]).max(axis=1)
    den = np.abs(ref["out"][sample]).max(axis=1)
    return {"max_row_rel_err": float((num / den).max()), "tol": 2e-2 if res["_cfg"].dtype == "bf16" else 1e-5,
            "routing_exact": bool(np.array_equal(res["_topk_idx"], ref["topk_idx"])),
            "tokens_compared": len(sample)}


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the hot path is a single-GPU "
              "kernel path; sharding by expert is a design note only). Run with --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    import paper_2509_23638_amd.binding as B
    from workloads import get_config

    if args.workload == "c5_stack":
        return run_c5(args, torch, B)
    T = args.tokens if (args.workload == "c2_mixtral" or args.tokens_all) else get_config(args.workload).T
    r = run_layer(args, torch, B, args.workload, T, args.steps, args.warmup, args.weight_sets, True)
    cfg = r["_cfg"]
    res = {
        "metric": "MoE-layer decode tokens/sec, Mixtral shape batch 64"
                  if args.workload == "c2_mixtral" else f"MoE-layer tokens/sec, {args.workload}",
        "value": r["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": r["ms_per_step"],
        "ms_per_step_median": r["ms_per_step_median"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload} single MoE layer, T={T} decode tokens, "
                               f"H={cfg.H} E={cfg.E} top-{cfg.k} F={cfg.F} S={cfg.S}, all experts "
                               f"resident ({args.layout} weight layout), {args.weight_sets} weight sets rotated",
                   "tokens": T, "active_experts": r["active_experts"], "library": B.moe_version()},
        "roofline": r["roofline"], "phases_ms": r["phases_ms"], "kernels": r["kernels"],
    }
    if "hbm_probe" in r:
        res["hbm_probe"] = r["hbm_probe"]
    if not args.no_cpu_baseline:
        base = cpu_baseline(cfg, r["_host0"], r["_Xh"], args.cpu_sample_tokens)
        res["parity_err"] = parity_of_timed_output(r, base)
        res["cpu_baseline"] = base
    for k_ in [k_ for k_ in r if k_.startswith("_")]:
        del r[k_]
    # the other single-layer workloads, a few steps each (same harness, untouched kernels):
    # the Mixtral batch sweep, the fine-grained, prefill and Qwen3-shaped layers
    if not args.no_other_workloads and args.workload == "c2_mixtral" and T == 64:
        others = []
        plan = [("c2_mixtral", t, args.weight_sets) for t in (1, 8, 256)] + \
               [(w, get_config(w).T, 2) for w in ("c3_finegrained", "c4_dsv2lite_prefill", "c6_qwen3_a3b")]
        for w, t, sets in plan:
            o = run_layer(args, torch, B, w, t, args.other_steps, 30, sets, False)
            others.append({"workload": w, "tokens": t, "ms_per_step": o["ms_per_step"],
                           "ms_per_step_median": o["ms_per_step_median"],
                           "tokens_per_s": o["tokens_per_s"], "active_experts": o["active_experts"],
                           "layer_hbm_frac": o["roofline"]["layer"]["frac"],
                           "layer_mfma_frac": o["roofline"]["layer"]["mfma_frac"],
                           "gate_up_hbm_frac": o["roofline"]["frac"], "kernels": o["kernels"],
                           "phases_ms": o["phases_ms"]})
        res["other_workloads"] = others
    print(json.dumps(res))


if __name__ == "__main__":
    main()
