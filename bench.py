#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

A step = one pass of the whole hot path (route -> permute -> grouped FFN ->
combine, i.e. one moe_layer_forward) over one batch of synthetic decode tokens
of the Mixtral-8x7B-shaped layer (hidden 4096, 8 experts, top-2, FFN 14336,
bf16 storage, fp32 accumulate), all experts resident in HBM.  Successive steps
rotate over several distinct weight sets so that no step finds its weights in
the 256 MB last-level cache.

Prints ONE JSON line.  `value` = tokens/s of the whole layer with inputs
already in HBM.  `roofline` prices the dominant kernel (gate/up weight stream)
against the 8 TB/s HBM peak using its algorithmic bytes and its average
duration measured with HIP events recorded between the kernels inside the
timed region.  `cpu_baseline` times the fp64 CPU oracle on a bounded sample of
the same batch on this machine's host cores.
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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=12)
    ap.add_argument("--tokens", type=int, default=64, help="decode batch (tokens per step)")
    ap.add_argument("--weight-sets", type=int, default=3,
                    help="distinct layers' weights rotated through (cache defeat)")
    ap.add_argument("--workload", default="c2_mixtral",
                    choices=["c2_mixtral", "c3_finegrained", "c4_dsv2lite_prefill"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    O.moe_layer(X, L["Wr"], L["b"], L["Wg"], L["Wu"], L["Wd"], cfg.k, cfg.S, tokens=sample)
    dt = time.perf_counter() - t0
    return {"value": len(sample) / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{len(sample)} of the batch's {X.shape[0]} tokens through the fp64 oracle "
                      f"(routing for all tokens, experts for the sample), {dt:.1f} s wall"}


def hbm_probe(torch, B):
    """Plain streaming kernels of known size: achievable HBM rate of this machine."""
    out = {}
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    big = torch.empty(4 << 30, dtype=torch.uint8, device="cuda")
    big.view(torch.int32).random_(0, 1 << 30)
    sink = torch.zeros(4, dtype=torch.uint8, device="cuda")
    for name, fn, nbytes in (("copy_1GiB", lambda: B.moe_probe_copy(dst, src), 2 * (1 << 30)),
                             ("read_4GiB", lambda: B.moe_probe_read(big, sink), 4 << 30)):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name + "_GBps"] = nbytes * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    return out


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the hot path is a single-GPU "
              "kernel path; see DESIGN.md for how it would shard). Run with --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    import paper_2509_23638_amd.binding as B
    from workloads import get_config, make_layer, make_hidden

    cfg = get_config(args.workload)
    T = args.tokens if args.workload == "c2_mixtral" else cfg.T
    cfg = cfg.with_(T=T)
    sh = B.make_shape(T, cfg.H, cfg.E, cfg.k, cfg.F, cfg.S, cfg.dtype)

    def dev(a):
        t = torch.from_numpy(a.view(np.int16)).view(torch.bfloat16) if a.dtype == np.uint16 \
            else torch.from_numpy(a)
        return t.cuda()

    layers, hosts = [], []
    for i in range(args.weight_sets):
        L = make_layer(cfg, layer=i, with_hidden=False, threads=16)
        if i == 0:
            hosts.append(L)
        Wg, Wu, Wd = dev(L["Wg"]), dev(L["Wu"]), dev(L["Wd"])
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
    A, rows = cfg.A, cfg.rows

    def gate_up_bytes(na):
        return (na + cfg.S) * 2 * cfg.F * cfg.H * es + T * cfg.H * es + rows * cfg.F * es

    def layer_bytes(na):
        return ((na + cfg.S) * 3 * cfg.F * cfg.H * es      # expert weights, once
                + 2 * T * cfg.H * es                        # X in, out
                + cfg.E * cfg.H * es                        # router weights
                + 2 * rows * cfg.F * es                     # h written, read
                + 2 * rows * cfg.H * 4)                     # Y written, read (fp32)

    for i in range(args.warmup):
        B.moe_layer_forward(ctx, sh, layers[i % len(layers)], X, out, ws)
    torch.cuda.synchronize()

    ctx.phase_timing(True)
    ctx.phase_times(reset=True)
    t0 = time.perf_counter()
    for i in range(args.steps):
        B.moe_layer_forward(ctx, sh, layers[i % len(layers)], X, out, ws)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ph = ctx.phase_times(reset=True)
    ctx.phase_timing(False)

    ms_per_step = dt / args.steps * 1e3
    value = T / (ms_per_step / 1e3)
    used = [n_active[i % len(layers)] for i in range(args.steps)]
    gu_bytes = float(np.mean([gate_up_bytes(n) for n in used]))
    all_bytes = float(np.mean([layer_bytes(n) for n in used]))
    gu_ms = ph["gate_up_ms"] / max(1, ph["n_layers"])
    achieved = gu_bytes / (gu_ms * 1e-3) / 1e9 if gu_ms > 0 else 0.0

    res = {
        "metric": "MoE-layer decode tokens/sec, Mixtral shape batch 64"
                  if args.workload == "c2_mixtral" else f"MoE-layer tokens/sec, {args.workload}",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload} single MoE layer, T={T} decode tokens, "
                               f"H={cfg.H} E={cfg.E} top-{cfg.k} F={cfg.F} S={cfg.S}, all experts "
                               f"resident, {len(layers)} weight sets rotated",
                   "tokens": T, "active_experts": float(np.mean(used))},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "ffn_stream_kernel<gate/up>", "kernel_ms": gu_ms,
                     "algorithmic_bytes": gu_bytes},
        "phases_ms": {k: ph[k] / max(1, ph["n_layers"]) for k in
                      ("route_ms", "permute_ms", "gate_up_ms", "down_ms", "combine_ms")},
        "layer_hbm": {"algorithmic_bytes": all_bytes,
                      "achieved_GBps": all_bytes / (ms_per_step * 1e-3) / 1e9,
                      "frac_of_peak": all_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    if args.probe:
        res["hbm_probe"] = hbm_probe(torch, B)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg, hosts[0], Xh, args.cpu_sample_tokens)
    ctx.close()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
