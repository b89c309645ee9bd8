"""Writes tests/golden/classifier_seeds.json.  Calls only the oracle (never the HIP path).

A random 3->h->1 MLP drawn N(0, 0.5) is often degenerate as a pruning classifier (it keeps
every candidate or none).  Rule (it consults the oracle only, never the HIP path; its part (b) was
added, and every seed chosen again, once after the first HIP path existed, because seeds chosen by
(a) alone gave trees that die at the root, and such workloads exercise one layer of the path and
nothing else): for each config take the smallest seed s >= 0 for which the oracle, run on the first min(B, 4) sequences of workload instance 0,
  (a) lets between 20% and 80% of the second layer's candidates pass the threshold beta, and
  (b) builds, for every one of those sequences, a tree that uses the whole node budget or is still
      growing in the last layer (so the workload exercises every layer, not a tree that dies early).
For the chain configuration (F = K = 1, Sec. 5.5) the trees are chains that are meant to stop early:
there the rule is, on the first 64 sequences, (a) as above and (b') at least three distinct chain
lengths whose mean lies between a quarter and three quarters of the maximum depth.
Configurations already in the file keep their seed unless --all is given.
Usage: python tests/golden/make_classifier_seeds.py [--all]
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import workloads as W  # noqa: E402
from oracle import RefTree, ref_logit_of_beta  # noqa: E402


def evaluate(cfg, seed, logits):
    ns = logits[0].shape[0]
    t = RefTree(ns, cfg["V"], cfg["F"], cfg["K"], cfg["D"], cfg["N"], cfg["h"], 0 if cfg["dtype"] == "f32" else 1, cfg["beta"])
    t.set_classifier(*W.classifier(cfg, seed))
    t.reset()
    zb = ref_logit_of_beta(cfg["beta"])
    frac = None
    for l in range(cfg["D"]):
        if t.frontier()["n_frontier"].sum() == 0:
            break
        t.expand_layer(logits[l], threads=ns)
        if l == 1:
            c = t.candidates()
            tot = int(c["n_cand"].sum())
            surv = sum(int((c["z"][b, :c["n_cand"][b]] > zb).sum()) for b in range(ns))
            frac = surv / max(tot, 1)
    alive = t.frontier()["n_frontier"].tolist() if t.layer == cfg["D"] else [0] * ns
    out = t.finalize()
    return frac, out["n_nodes"].tolist(), alive


def main():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "classifier_seeds.json")
    result = {}
    if "--all" not in sys.argv and os.path.exists(path):
        with open(path) as f:
            result = json.load(f)
    for name, cfg in W.CONFIGS.items():
        if name in result:
            continue
        chain = cfg["F"] == 1 and cfg["K"] == 1
        ns = min(cfg["B"], 64 if chain else 4)
        logits = [W.as_numpy_bits(W.logits_layer(cfg, l, seqs=range(ns))) for l in range(cfg["D"])]
        for seed in range(2000):
            frac, nn, alive = evaluate(cfg, seed, logits)
            if chain:
                ok = (frac is not None and 0.2 <= frac <= 0.8 and len(set(nn)) >= 3
                      and 0.25 * cfg["D"] <= float(np.mean(nn)) <= 0.75 * cfg["D"])
            else:
                ok = frac is not None and 0.2 <= frac <= 0.8 and all(n == cfg["N"] or a > 0 for n, a in zip(nn, alive))
            print(name, seed, frac, nn if not chain else sorted(set(nn)), alive if not chain else "", "OK" if ok else "", flush=True)
            if ok:
                result[name] = dict(seed=seed, layer1_pass_fraction=frac, n_nodes=nn)
                break
        else:
            raise SystemExit("no seed found for " + name)
    with open(path, "w") as f:
        json.dump(result, f, indent=1)


if __name__ == "__main__":
    main()
