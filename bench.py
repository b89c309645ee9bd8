"""Benchmark of the C2T tree-construction hot path on one MI355X.

A step is one whole draft phase over one batch of synthetic logits: reset, max_depth x
expand_layer (one launch per layer: logits pass, row scoring and sequence pruning in the same
kernel), finalize_tree, with every input resident in HBM.
Prints ONE JSON line: whole-job throughput in draft-tree nodes scored per second on the headline
workload (cfg4), the HBM roofline of the layer kernel (timed with HIP events on its own stream inside
the timed region; its algorithmic bytes are the logits rows it reads), the same figures for the
other configurations under `secondary` (bounded legs, outside the timed region) and the CPU oracle
timed on a bounded sample of the headline workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E bandwidth


def esz_of(cfg):
    return 4 if cfg["dtype"] == "f32" else 2


def make_layers(W, cfg, dev, n_layers=None):
    """Logits of the first n_layers layers, resident on the device.  Small configurations come from
    the CPU generator, the stream the classifier seeds were chosen on (torch's CPU and GPU generators
    differ; a GPU-generated cfg3 tree dies at the root)."""
    B, V, F, D = (cfg[k] for k in ("B", "V", "F", "D"))
    n = D if n_layers is None else min(D, n_layers)
    gen = "cpu" if B * F * V * D * esz_of(cfg) <= (256 << 20) else dev
    layers = [W.logits_layer(cfg, l, device=gen).to(dev) for l in range(n)]
    return layers + [layers[-1]] * (D - n)          # layers past n_layers have no live row to read


def new_context(C2TContext, cfg, cls, dev, beta=None, a=None):
    ctx = C2TContext(cfg["B"], cfg["V"], cfg["F"], cfg["K"], cfg["D"], cfg["N"], cfg["h"], 0 if cfg["dtype"] == "f32" else 1,
                     cfg["beta"] if beta is None else beta,
                     entropy_top_m=a.entropy_top_m if a else 0, rerank=1 if (a and a.rerank) else 0, device=dev)
    ctx.set_classifier(*cls)
    if a and a.splits:
        ctx.set_row_splits(*[int(x) for x in a.splits.split(",")])
    return ctx


def time_phases(torch, np, ctx, cfg, layers, out, steps, warmup, profile_every, rerank=0, graph=False):
    """warmup untimed + steps timed draft phases; per-launch kernel times from events attached to the
    launches of every profile_every-th timed step.  Returns (seconds, per-launch ms [sampled][D], rows per layer)."""
    D = cfg["D"]

    def step():
        ctx.reset()
        for l in range(D):
            ctx.expand_layer(layers[l])
        if rerank:
            ctx.finalize_tree_reranked(rerank, out)
        else:
            ctx.finalize_tree(out)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                                   # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        n_ev = min(steps, 20)
        ctx.profile_enable(n_ev * D)                 # events cannot be attached inside a graph: un-captured phases afterwards
        for _ in range(n_ev):
            step()
        torch.cuda.synchronize()
        k_ms = ctx.profile_read(n_ev * D)
    else:
        # the per-dispatch events cost the host about 20 us a launch, which shows in the step time: they
        # are attached to every profile_every-th step of the timed region only
        ctx.profile_enable(steps * D)
        every = profile_every if steps >= profile_every else 1
        ctx.profile_sample(every, every // 2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        k_ms = ctx.profile_read(steps * D)
    ctx.profile_enable(0)
    rows = ctx.layer_rows().cpu().numpy()[:D].astype(np.int64)       # rows consumed by each layer's expand
    n_s = len(k_ms) // D
    return dt, np.array(k_ms[:n_s * D], np.float64).reshape(n_s, D), rows


def time_full_layers(torch, np, C2TContext, cfg, cls, layers, dev, reps, a=None):
    """The layer kernel on FULL layers (every sequence with F rows), the unit the HBM roofline is stated
    on: the same logits and classifier with beta = 0, so that every candidate survives the first
    pruning and the frontiers stay full until the budget is used up."""
    B, V, F, D, N = (cfg[k] for k in ("B", "V", "F", "D", "N"))
    n_full = min(D - 1, N // F) if B > 1 else 0
    if n_full < 1:
        return None
    f = new_context(C2TContext, cfg, cls, dev, beta=0.0, a=a)
    for timed in (False, True):
        if timed:
            f.profile_enable(reps * (1 + n_full))
        for _ in range(reps):
            f.reset()
            for l in range(1 + n_full):
                f.expand_layer(layers[l])
        torch.cuda.synchronize()
    f_ms = np.array(f.profile_read(reps * (1 + n_full)), np.float64).reshape(reps, 1 + n_full)[:, 1:]
    f_rows = f.layer_rows().cpu().numpy()[1:1 + n_full].astype(np.int64)
    assert (f_rows == B * F).all(), f_rows
    f.profile_enable(0)
    fb = float(B * F * V * esz_of(cfg))
    us = float(f_ms.mean() * 1e3)
    return {"rows": int(B * F), "bytes": fb, "launches": int(f_ms.size), "us": us, "min_us": float(f_ms.min() * 1e3),
            "gbps": fb / us / 1e3, "frac": fb / us / 1e3 / HBM_PEAK_GBPS}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg4", help="cfg1..cfg5 (default: batched serving, B=64, V=128256)")
    ap.add_argument("--splits", default="", help="row splits 'first,other' (0 = default)")
    ap.add_argument("--entropy-top-m", type=int, default=0,
                    help="M > 0: entropy over the M most probable tokens (Eq. 2, second line) instead of the whole row")
    ap.add_argument("--rerank", type=int, default=0,
                    help="n > 0: finish with the EAGLE-2-style reranking of all scored candidates (Sec. 2.2), n nodes out")
    ap.add_argument("--mask-frac", type=float, default=0.0,
                    help="fraction of the vocabulary (a seeded, scattered set of tokens, the same in every row) whose "
                         "logits are -inf, as under constrained decoding")
    ap.add_argument("--graph", action="store_true",
                    help="capture one draft phase in a HIP graph and time K replays (the per-launch kernel times for "
                         "the roofline then come from further, un-captured phases after the timed region)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-full-layer", action="store_true",
                    help="skip the extra full-layer launches (roofline.full_layer), so that a kernel trace of the run "
                         "holds the warm-up and timed draft phases only")
    ap.add_argument("--only-full-layer", action="store_true",
                    help="run nothing but the full-layer launches (for a kernel trace whose average of the four-per-CU "
                         "build of the layer kernel is the full-layer figure)")
    ap.add_argument("--no-secondary", action="store_true", help="skip the bounded legs on the other configurations")
    ap.add_argument("--profile-every", type=int, default=4, help="steps of the timed region between two steps whose launches carry timing events")
    ap.add_argument("--cpu-seqs", type=int, default=0, help="sequences the oracle is timed on (0 = auto)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (sequences are independent: the path would shard by "
              "splitting the batch over GPUs, with no exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as W
    from paper_2502_13652_amd import C2TContext, stream_read, stream_read_rows

    assert torch.cuda.is_available(), "bench.py needs a GPU (no CPU fallback)"
    dev = torch.device("cuda:0")
    cfg = W.CONFIGS[a.workload]
    B, V, F, K, D, N, h = (cfg[k] for k in ("B", "V", "F", "K", "D", "N", "h"))
    esz = esz_of(cfg)
    cls = W.classifier(cfg, W.classifier_seed(a.workload))
    layers = make_layers(W, cfg, dev)
    if a.mask_frac > 0:
        g = torch.Generator(device="cpu").manual_seed(20250213)
        masked = (torch.rand(V, generator=g) < a.mask_frac).to(dev)
        for x in layers:
            x[..., :V].masked_fill_(masked, float("-inf"))

    if a.only_full_layer:
        fl = time_full_layers(torch, np, C2TContext, cfg, cls, layers, dev, max(3, a.steps // 2), a)
        print(json.dumps({"full_layer": fl}))
        return

    ctx = new_context(C2TContext, cfg, cls, dev, a=a)
    out = ctx.new_tree_out(a.rerank or None)
    dt, k1_ms, rows = time_phases(torch, np, ctx, cfg, layers, out, a.steps, a.warmup, a.profile_every, a.rerank, a.graph)
    scored_per_step = int(rows.sum()) * K
    n_sampled = k1_ms.shape[0]
    bytes_layer = rows * V * esz
    achieved = bytes_layer.sum() * n_sampled / (k1_ms.sum() / 1e3) / 1e9       # GB/s over every logits-pass launch
    per_layer = [dict(layer=int(l), rows=int(rows[l]), mbytes=round(bytes_layer[l] / 1e6, 2),
                      us=round(float(k1_ms[:, l].mean() * 1e3), 2),
                      gbps=round(float(bytes_layer[l] / (k1_ms[:, l].mean() / 1e3) / 1e9), 1)) for l in range(D)]
    n_nodes = out["n_nodes"].cpu().numpy()

    full_layer = None
    if not a.mask_frac and not a.no_full_layer:
        full_layer = time_full_layers(torch, np, C2TContext, cfg, cls, layers, dev, max(3, min(a.steps // 2, 20)), a)

    # practical ceiling: plain streaming read of a buffer larger than the last-level cache
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    acc = torch.zeros(1, dtype=torch.int32, device=dev)
    for _ in range(2):
        stream_read(big, acc)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        stream_read(big, acc)
    e1.record()
    torch.cuda.synchronize()
    stream_gbps = 5 * big.numel() / (e0.elapsed_time(e1) / 1e3) / 1e9
    # the same bytes read with the layer kernel's access pattern (one workgroup per row of V logits,
    # as many rows as a full layer has, rotating over the buffer) and no other work
    row_bytes = (V * esz + 15) // 16 * 16
    n_rows = min(B * F, big.numel() // row_bytes)
    groups = max(1, min(4, big.numel() // (n_rows * row_bytes)))
    for i in range(2 + 5):
        if i == 2:
            e0.record()
        stream_read_rows(big[(i % groups) * n_rows * row_bytes:], n_rows, row_bytes, acc)
    e1.record()
    torch.cuda.synchronize()
    row_read_gbps = 5 * n_rows * row_bytes / (e0.elapsed_time(e1) / 1e3) / 1e9
    del big

    # HBM traffic per launch: NOT measured in this run.  It is the FETCH_SIZE counter of the committed
    # rocprofv3 pass on this workload (profiles/k_logits_hist_cfg4_pmc.md says on which build and how it
    # was scaled), quoted for the default workload only.
    traffic, traffic_source = None, None
    if a.workload == "cfg4" and not a.splits and not a.entropy_top_m and not a.rerank and not a.mask_frac:
        try:
            import re
            with open(os.path.join(ROOT, "profiles", "k_logits_hist_cfg4_pmc.md")) as f:
                traffic = float(re.search(r"traffic_bytes_per_launch = (\d+)", f.read()).group(1))
            traffic_source = "profiles/k_logits_hist_cfg4_pmc.md (rocprofv3 --pmc FETCH_SIZE, committed pass; not measured in this run)"
        except (OSError, AttributeError):
            traffic = None

    rec = {
        "metric": "draft-tree nodes scored/sec + logits-pass HBM GB/s (fraction of peak), 1 GPU",
        "value": scored_per_step * a.steps / dt,
        "unit": "nodes scored/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": dt / a.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": "%s: %s" % (a.workload, cfg["desc"]), "B": B, "V": V, "logits": cfg["dtype"], "D": D,
                   "F": F, "K": K, "h": h, "beta": cfg["beta"], "N": N,
                   "arithmetic": "%s logits compared as stored; exact integer value counts; fp64 sums (Z, S, p, H); fp32 classifier" % cfg["dtype"],
                   "entropy_top_m": a.entropy_top_m, "rerank": a.rerank, "mask_frac": a.mask_frac, "hip_graph": bool(a.graph),
                   "profile_every": a.profile_every, "classifier_seed": W.classifier_seed(a.workload),
                   "nodes_scored_per_step": scored_per_step, "tree_nodes_mean": float(n_nodes.mean()),
                   "workgroups_per_row": list(ctx.row_workgroups())},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "k_logits_hist<512,false,*,*>" if cfg["dtype"] == "bf16" else "k_logits_generic<0,512>",
                     "launches": int(n_sampled * D), "sampled_steps": int(n_sampled),
                     "avg_launch_us": float(k1_ms.mean() * 1e3),
                     "algorithmic_bytes_per_launch": float(bytes_layer.mean()),
                     # the same kernel on full layers (every sequence with F rows), the unit the target is stated on
                     "frac_full_layer": full_layer["frac"] if full_layer else None,
                     "full_layer_us": full_layer["us"] if full_layer else None,
                     "full_layer_gbps": full_layer["gbps"] if full_layer else None,
                     "full_layer": full_layer,
                     "stream_read_gbps": stream_gbps, "row_read_gbps": row_read_gbps, "per_layer": per_layer},
    }
    del ctx, layers, out
    torch.cuda.empty_cache()

    # ---- the other configurations, bounded legs outside the timed region ----
    if not a.no_secondary and a.workload == "cfg4" and not (a.splits or a.entropy_top_m or a.rerank or a.mask_frac or a.graph):
        sec = {}
        for name in ("cfg5", "cfg1", "cfg2", "cfg3"):
            c2 = W.CONFIGS[name]
            cls2 = W.classifier(c2, W.classifier_seed(name))
            # cfg5's budget (N = 4 F) ends every tree after layer 4: layers 5.. have no row to read
            lay2 = make_layers(W, c2, dev, n_layers=(1 + c2["N"] // c2["F"]) if c2["B"] > 1 else None)
            x2 = new_context(C2TContext, c2, cls2, dev)
            o2 = x2.new_tree_out()
            st = 10 if c2["B"] > 1 else 50
            d2, k2, r2 = time_phases(torch, np, x2, c2, lay2, o2, st, 2, 2)
            live = r2 > 0
            b2 = r2 * c2["V"] * esz_of(c2)
            s = {"ms_per_step": d2 / st * 1e3, "nodes_scored_per_s": int(r2.sum()) * c2["K"] * st / d2, "steps": st,
                 "rows_per_layer": r2.tolist(), "us_per_layer": [round(float(v), 2) for v in (k2.mean(0) * 1e3)],
                 "us_per_live_layer_mean": float(k2.mean(0)[live].mean() * 1e3),
                 "workgroups_per_row": list(x2.row_workgroups())}     # (first layer, later layers): above 1 on the bf16 path = rows shared by workgroups
            if c2["B"] > 1:
                s["achieved_gbps"] = float(b2.sum() * k2.shape[0] / (k2.sum() / 1e3) / 1e9)
                s["frac"] = s["achieved_gbps"] / HBM_PEAK_GBPS
                fl = time_full_layers(torch, np, C2TContext, c2, cls2, lay2, dev, 5)
                s["full_layer_us"], s["full_layer_gbps"], s["frac_full_layer"] = fl["us"], fl["gbps"], fl["frac"]
            else:
                # a single sequence is bound by launch latency: the same phases replayed from a HIP graph
                dg, _, _ = time_phases(torch, np, x2, c2, lay2, o2, st, 2, 2, graph=True)
                s["graph_ms_per_step"] = dg / st * 1e3
            sec[name] = s
            del x2, lay2, o2
            torch.cuda.empty_cache()
        rec["secondary"] = sec

    if not a.no_cpu_baseline:
        from oracle import RefTree
        layers = make_layers(W, cfg, dev)
        # bounded sample: whole draft phases of the first n sequences, one thread
        per_seq_elems = (1 + (D - 1) * F) * V
        nseq = a.cpu_seqs or max(1, min(B, int(1.0e9 / per_seq_elems)))
        sl = [W.as_numpy_bits(x[:nseq].cpu()) for x in layers]
        t = RefTree(nseq, V, F, K, D, N, h, 0 if cfg["dtype"] == "f32" else 1, cfg["beta"])
        if a.entropy_top_m:
            t.set_entropy_top_m(a.entropy_top_m)
        t.set_classifier(*cls)
        # the sample's draft phases are repeated until about ten seconds of CPU work are timed
        cdt, scored, passes = 0.0, 0, 0
        while cdt < 10.0 and passes < 200:
            t.reset()
            c0 = time.perf_counter()
            for l in range(D):
                if t.frontier()["n_frontier"].sum() == 0:
                    break
                t.expand_layer(sl[l], threads=1)
            if a.rerank:
                t.finalize_rerank(a.rerank)
            else:
                t.finalize()
            cdt += time.perf_counter() - c0
            scored += int(t.audit()["scored"].sum())
            passes += 1
        rec["cpu_baseline"] = {"value": scored / cdt, "unit": "nodes scored/s", "cores": 1, "kind": "oracle",
                               "sample": "whole draft phases of the first %d of %d sequences of %s, %d passes, %d candidates, %.1f s"
                                         % (nseq, B, a.workload, passes, scored, cdt)}
        # the same oracle with the (independent) sequences sharded over the host's cores
        nthr = min(16, os.cpu_count() or 1, B)
        if nthr > 1:
            nseq_all = min(B, nseq * nthr)
            sl = [W.as_numpy_bits(x[:nseq_all].cpu()) for x in layers]
            t = RefTree(nseq_all, V, F, K, D, N, h, 0 if cfg["dtype"] == "f32" else 1, cfg["beta"])
            if a.entropy_top_m:
                t.set_entropy_top_m(a.entropy_top_m)
            t.set_classifier(*cls)
            t.reset()
            c0 = time.perf_counter()
            for l in range(D):
                if t.frontier()["n_frontier"].sum() == 0:
                    break
                t.expand_layer(sl[l], threads=nthr)
            t.finalize_rerank(a.rerank) if a.rerank else t.finalize()
            cdt = time.perf_counter() - c0
            scored = int(t.audit()["scored"].sum())
            rec["cpu_baseline"]["sharded"] = {"value": scored / cdt, "cores": nthr,
                                              "sample": "%d sequences, %d candidates, %.1f s" % (nseq_all, scored, cdt)}
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
