"""Where a layer launch's time goes: builds the library with -DC2T_PHASE_TIMES into
lib/libc2t_hip_phase_times.so, runs draft phases of a benchmark configuration up to one layer and prints,
per phase boundary of the layer kernel, when the workgroups pass it (microseconds after the first
workgroup's start), the mean time between boundaries and the timeline of the workgroup that finishes last.

    python -m paper_2502_13652_amd.phase_times cfg4 2 --full     # a full layer (beta = 0) of cfg4
    python -m paper_2502_13652_amd.phase_times cfg3 2            # 16 rows, five workgroups each, all alone on their CUs
    python -m paper_2502_13652_amd.phase_times cfg3 2 --unshared # 16 workgroups, one per row
"""
import argparse
import ctypes
import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
sys.path.insert(0, _ROOT)

MARKS = ["start", "own stream ends", "histogram complete", "sums", "K-th largest known", "cells listed", "cells re-read",
         "top K ranked", "row scored, handed over", "sequence ticket", "sequence pruned",
         "  candidates loaded", "  first pruning done", "  preselected", "  ranked and appended",
         "  (split rows) row merged"]


def build():
    from paper_2502_13652_amd import binding
    out = os.path.join(_HERE, "lib", "libc2t_hip_phase_times.so")
    os.makedirs(os.path.dirname(out), exist_ok=True)
    cmd = ["hipcc"] + binding.HIPCC_FLAGS + ["-DC2T_PHASE_TIMES", "-I", os.path.join(_ROOT, "include"), "-o", out,
                                              os.path.join(_HERE, "csrc", "c2t_lib.hip")]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode:
        print(r.stdout)
        raise RuntimeError("hipcc failed")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("workload")
    ap.add_argument("layer", type=int)
    ap.add_argument("--full", action="store_true", help="beta = 0: every frontier stays full until the budget is used up")
    ap.add_argument("--unshared", action="store_true", help="one workgroup per row also where rows would be shared")
    ap.add_argument("--no-build", action="store_true")
    a = ap.parse_args()
    import numpy as np
    import torch
    import workloads as W
    from paper_2502_13652_amd import binding
    lib = os.path.join(_HERE, "lib", "libc2t_hip_phase_times.so")
    if not a.no_build or not os.path.exists(lib):
        build()
    L = binding.load_library(lib)
    dev = torch.device("cuda:0")
    cfg = W.CONFIGS[a.workload]
    B, V, F, K, D, N, h = (cfg[k] for k in ("B", "V", "F", "K", "D", "N", "h"))
    cls = W.classifier(cfg, W.classifier_seed(a.workload))
    gen = "cpu" if B == 1 else dev
    layers = [W.logits_layer(cfg, l, device=gen).to(dev) for l in range(a.layer + 1)]
    ctx = binding.C2TContext(B, V, F, K, D, N, h, 0 if cfg["dtype"] == "f32" else 1, 0.0 if a.full else cfg["beta"], device=dev)
    ctx.set_classifier(*cls)
    if a.unshared:
        ctx.set_row_splits(1, 1)
    per_row = ctx.row_workgroups()[0 if a.layer == 0 else 1]
    for _ in range(3):
        ctx.reset()
        for l in range(a.layer + 1):
            ctx.expand_layer(layers[l])
        torch.cuda.synchronize()
    rows = int(ctx.layer_rows().cpu().numpy()[a.layer])
    nwg = min(8192, B * (F if a.layer > 0 else 1) * per_row)
    buf = (ctypes.c_uint64 * (nwg * 16))()
    L.c2t_phase_times_read.argtypes = [ctypes.c_void_p, ctypes.c_int32]
    rc = L.c2t_phase_times_read(buf, nwg)
    assert rc == 0, rc
    t = np.array(buf, dtype=np.int64).reshape(nwg, 16)[:, :len(MARKS)].astype(np.float64)
    t = t[t[:, 0] > 0]                                    # workgroups that had a live row in the last launch
    t0 = t[:, 0].min()
    t[t < t0] = np.nan                                    # slots not passed in this launch hold older times
    us = (t - t0) / 100.0
    print("%s layer %d%s: %d rows consumed, %d workgroups with a row (%d per row)" % (a.workload, a.layer, " (full)" if a.full else "", rows, len(us), per_row))
    if per_row > 1:
        print("(the workgroups that hand a segment's counts over end after 'histogram complete'; 'sums' includes the hand-over)")
    print("%-26s %8s %8s %8s %6s" % ("boundary", "mean us", "min", "max", "n"))
    for i, nm in enumerate(MARKS):
        c = us[:, i]
        if np.all(np.isnan(c)):
            continue
        print("%-26s %8.2f %8.2f %8.2f %6d" % (nm, np.nanmean(c), np.nanmin(c), np.nanmax(c), int(np.sum(~np.isnan(c)))))
    d = np.diff(us[:, :9], axis=1)   # the row's own boundaries
    print("mean time between boundaries (start .. handed over):", np.round(np.nanmean(d, axis=0), 2).tolist())
    last = int(np.nanargmax(us[:, 8]))
    print("workgroup that hands its row over last:", np.round(us[last], 2).tolist())
    pr = ~np.isnan(us[:, 10])
    if pr.any():
        print("pruning workgroups (%d): handed over -> ticket %.2f us, ticket -> pruned %.2f us (means)"
              % (int(pr.sum()), np.nanmean(us[pr, 9] - us[pr, 8]), np.nanmean(us[pr, 10] - us[pr, 9])))
        seq = us[pr][:, [9, 11, 12, 13, 14, 10]]
        print("  inside the sequence step (ticket, candidates loaded, first pruning, preselected, ranked and appended, frontier stored), mean steps:",
              np.round(np.nanmean(np.diff(seq, axis=1), axis=0), 2).tolist())
    n_cus = torch.cuda.get_device_properties(dev).multi_processor_count
    if n_cus < len(us) <= 4 * n_cus and len(us) == nwg:
        # a launch of one round is placed statically: workgroups w, w + n_cus, w + 2 n_cus, ... share a CU
        hc = np.full(4 * n_cus, np.nan); hc[:len(us)] = us[:, 2]
        per_cu = np.nanmax(hc.reshape(4, n_cus), axis=0)
        print("per CU, when the last of its workgroups has its histogram complete: min %.1f, 10 %% %.1f, median %.1f, 90 %% %.1f, max %.1f us"
              % (per_cu.min(), np.percentile(per_cu, 10), np.median(per_cu), np.percentile(per_cu, 90), per_cu.max()))
        print("workgroups still streaming at", ", ".join("%d us: %d" % (t, int((us[:, 2] > t).sum())) for t in range(int(per_cu.min()) - 4, int(per_cu.max()) + 2, 2)))
    print("first start -> last boundary: %.2f us" % np.nanmax(us))


if __name__ == "__main__":
    main()
