"""Benchmark of the C2T tree-construction hot path on one MI355X.

A step is one whole draft phase over one batch of synthetic logits: reset, max_depth x
expand_layer (one launch per layer: logits pass, row scoring and sequence pruning in the same
kernel), finalize_tree, with every input resident in HBM.
Prints ONE JSON line: whole-job throughput in draft-tree nodes scored per second, the HBM
roofline of the layer kernel (timed with HIP events on its own stream inside the timed region;
its algorithmic bytes are the logits rows it reads) and the CPU oracle timed on a bounded sample
of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E bandwidth


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
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
                         "the roofline then come from K further, un-captured phases after the timed region)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-full-layer", action="store_true",
                    help="skip the extra full-layer launches (roofline.full_layer), so that a kernel trace of the run "
                         "holds the warm-up and timed draft phases only")
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
    esz = 4 if cfg["dtype"] == "f32" else 2
    cls = W.classifier(cfg, W.classifier_seed(a.workload))
    # Small configurations are generated with the CPU generator, the stream the classifier seed was
    # chosen on (torch's CPU and GPU generators differ; a GPU-generated cfg3 tree dies at the root).
    gen = "cpu" if B * F * V * D * esz <= (256 << 20) else dev
    layers = [W.logits_layer(cfg, l, device=gen).to(dev) for l in range(D)]
    if a.mask_frac > 0:
        g = torch.Generator(device="cpu").manual_seed(20250213)
        masked = (torch.rand(V, generator=g) < a.mask_frac).to(dev)
        for x in layers:
            x[..., :V].masked_fill_(masked, float("-inf"))
    ctx = C2TContext(B, V, F, K, D, N, h, 0 if cfg["dtype"] == "f32" else 1, cfg["beta"],
                     entropy_top_m=a.entropy_top_m, rerank=1 if a.rerank else 0, device=dev)
    ctx.set_classifier(*cls)
    if a.splits:
        ctx.set_row_splits(*[int(x) for x in a.splits.split(",")])
    out = ctx.new_tree_out(a.rerank or None)

    def step():
        ctx.reset()
        for l in range(D):
            ctx.expand_layer(layers[l])
        if a.rerank:
            ctx.finalize_tree_reranked(a.rerank, out)
        else:
            ctx.finalize_tree(out)

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    if a.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                                   # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ctx.profile_enable(a.steps * D)
        for _ in range(a.steps):
            step()
        torch.cuda.synchronize()
    else:
        # the per-dispatch events cost the host about 20 us a launch, which shows in the step time: they
        # are attached to every --profile-every-th step of the timed region only
        ctx.profile_enable(a.steps * D)
        every = a.profile_every if a.steps >= a.profile_every else 1
        ctx.profile_sample(every, every // 2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    k1_ms = ctx.profile_read(a.steps * D)
    ctx.profile_enable(0)
    rows = ctx.layer_rows().cpu().numpy()[:D].astype(np.int64)      # rows consumed by each layer's expand
    scored_per_step = int(rows.sum()) * K
    n_sampled = len(k1_ms) // D                                     # steps whose launches carried events
    k1_ms = np.array(k1_ms[:n_sampled * D], np.float64).reshape(n_sampled, D)
    bytes_layer = rows * V * esz
    k1_total_s = k1_ms.sum() / 1e3
    achieved = bytes_layer.sum() * n_sampled / k1_total_s / 1e9       # GB/s over every logits-pass launch
    per_layer = [dict(layer=int(l), rows=int(rows[l]), mbytes=round(bytes_layer[l] / 1e6, 2),
                      us=round(float(k1_ms[:, l].mean() * 1e3), 2),
                      gbps=round(float(bytes_layer[l] / (k1_ms[:, l].mean() / 1e3) / 1e9), 1)) for l in range(D)]

    # Full layers (every sequence with F valid rows), the unit the HBM roofline is stated on: the same
    # logits and classifier with beta = 0, so that every candidate survives the first pruning and the
    # frontiers stay full until the budget is used up.  Outside the timed region.
    full_layer = None
    n_full = min(D - 1, N // F) if B > 1 else 0
    if n_full >= 1 and not a.mask_frac and not a.no_full_layer:
        fctx = C2TContext(B, V, F, K, D, N, h, 0 if cfg["dtype"] == "f32" else 1, 0.0,
                          entropy_top_m=a.entropy_top_m, device=dev)
        fctx.set_classifier(*cls)
        if a.splits:
            fctx.set_row_splits(*[int(x) for x in a.splits.split(",")])
        reps = max(3, a.steps // 2)
        for timed in (False, True):
            if timed:
                fctx.profile_enable(reps * (1 + n_full))
            for _ in range(reps):
                fctx.reset()
                for l in range(1 + n_full):
                    fctx.expand_layer(layers[l])
            torch.cuda.synchronize()
        f_ms = np.array(fctx.profile_read(reps * (1 + n_full)), np.float64).reshape(reps, 1 + n_full)[:, 1:]
        f_rows = fctx.layer_rows().cpu().numpy()[1:1 + n_full].astype(np.int64)
        assert (f_rows == B * F).all(), f_rows
        fctx.profile_enable(0)
        fb = float(B * F * V * esz)
        full_layer = {"rows": int(B * F), "bytes": fb, "launches": int(f_ms.size), "us": float(f_ms.mean() * 1e3),
                      "gbps": fb / (f_ms.mean() / 1e3) / 1e9, "frac": fb / (f_ms.mean() / 1e3) / 1e9 / HBM_PEAK_GBPS}
        del fctx

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

    # HBM traffic per launch from the committed counter pass (rocprofv3 --pmc FETCH_SIZE, scaled by the
    # factor the same counter shows for the plain read kernel); only for the workload it was taken on
    traffic = None
    if a.workload == "cfg4" and not a.splits and not a.entropy_top_m and not a.rerank and not a.mask_frac:
        try:
            import re
            with open(os.path.join(ROOT, "profiles", "k_logits_hist_cfg4_pmc.md")) as f:
                traffic = float(re.search(r"traffic_bytes_per_launch = (\d+)", f.read()).group(1))
        except (OSError, AttributeError):
            traffic = None

    n_nodes = out["n_nodes"].cpu().numpy()
    rec = {
        "metric": "draft-tree nodes scored/sec + logits-pass HBM GB/s (fraction of peak), 1 GPU",
        "value": scored_per_step * a.steps / dt,
        "unit": "nodes scored/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": dt / a.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": "%s: %s" % (a.workload, cfg["desc"]), "B": B, "V": V, "logits": cfg["dtype"], "D": D,
                   "F": F, "K": K, "h": h, "beta": cfg["beta"], "N": N, "entropy_top_m": a.entropy_top_m, "rerank": a.rerank, "mask_frac": a.mask_frac, "hip_graph": bool(a.graph), "profile_every": a.profile_every, "classifier_seed": W.classifier_seed(a.workload),
                   "nodes_scored_per_step": scored_per_step, "tree_nodes_mean": float(n_nodes.mean())},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "kernel": "k_logits_hist<512>" if cfg["dtype"] == "bf16" else "k_logits_generic<0,256>", "launches": int(n_sampled * D), "sampled_steps": int(n_sampled),
                     "avg_launch_us": float(k1_ms.mean() * 1e3),
                     "algorithmic_bytes_per_launch": float(bytes_layer.mean()),
                     "full_layer": full_layer,
                     "stream_read_gbps": stream_gbps, "row_read_gbps": row_read_gbps, "per_layer": per_layer},
    }

    if not a.no_cpu_baseline:
        from oracle import RefTree
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
