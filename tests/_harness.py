"""Shared helpers of the GPU parity tests: run the HIP path and the oracle on the same
seeded inputs and compare them element by element."""
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402

RTOL = 1e-5          # relative tolerance for probabilities, features, confidences (fp64 definition rounded to fp32)
ORACLE_THREADS = 16  # the GPU machine's CPU share


def dtype_code(cfg):
    return 0 if cfg["dtype"] == "f32" else 1


def make_gpu(cfg, cls, B=None, device="cuda:0"):
    from paper_2502_13652_amd import C2TContext
    ctx = C2TContext(B or cfg["B"], cfg["V"], cfg["F"], cfg["K"], cfg["D"], cfg["N"], cfg["h"], dtype_code(cfg),
                     cfg["beta"], entropy_top_m=cfg.get("entropy_top_m", 0), rerank=cfg.get("rerank", 0), device=device)
    ctx.set_classifier(*cls)
    return ctx


def make_oracle(cfg, cls, B=None):
    from oracle import RefTree
    t = RefTree(B or cfg["B"], cfg["V"], cfg["F"], cfg["K"], cfg["D"], cfg["N"], cfg["h"], dtype_code(cfg), cfg["beta"])
    if cfg.get("entropy_top_m", 0):
        t.set_entropy_top_m(cfg["entropy_top_m"])
    t.set_classifier(*cls)
    return t


def close(a, b, rtol=RTOL, atol=0.0):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return np.abs(a - b) <= rtol * np.abs(b) + atol


def compare_layer(gc, gf, oc, of, seqs, K, tag):
    """gc/gf: GPU candidates/frontier (numpy, full batch); oc/of: oracle's (batch = len(seqs))."""
    for i, b in enumerate(seqs):
        n = int(oc["n_cand"][i])
        assert int(gc["n_cand"][b]) == n, "%s seq %d: n_cand gpu %d oracle %d" % (tag, b, gc["n_cand"][b], n)
        np.testing.assert_array_equal(gc["token"][b, :n], oc["token"][i, :n], err_msg="%s seq %d tokens" % (tag, b))
        for k in ("p", "P", "H", "z"):
            # z is a sum of O(1) terms: compare it on the scale of 1 (absolute floor) as well
            ok = close(gc[k][b, :n], oc[k][i, :n], atol=1e-5 if k == "z" else 1e-30)
            assert ok.all(), "%s seq %d %s: worst %g vs %g" % (tag, b, k, gc[k][b, :n][~ok][0], oc[k][i, :n][~ok][0])
        np.testing.assert_array_equal(gc["kept"][b, :n], oc["kept"][i, :n], err_msg="%s seq %d kept" % (tag, b))
        nf = int(of["n_frontier"][i])
        assert int(gf["n_frontier"][b]) == nf, "%s seq %d n_frontier" % (tag, b)
        np.testing.assert_array_equal(gf["tokens"][b, :nf], of["tokens"][i, :nf], err_msg="%s seq %d frontier" % (tag, b))
        np.testing.assert_array_equal(gf["parent_slot"][b, :nf], of["parent_slot"][i, :nf])


def compare_final(go, oo, seqs, tag):
    for i, b in enumerate(seqs):
        n = int(oo["n_nodes"][i])
        assert int(go["n_nodes"][b]) == n, "%s seq %d: n_nodes gpu %d oracle %d" % (tag, b, go["n_nodes"][b], n)
        for k in ("tokens", "parent", "position"):
            np.testing.assert_array_equal(go[k][b], oo[k][i], err_msg="%s seq %d %s" % (tag, b, k))
        np.testing.assert_array_equal(go["mask"][b], oo["mask"][i], err_msg="%s seq %d mask" % (tag, b))
        assert int(go["status"][b]) & 1 == int(oo["status"][i])      # bit 1 is informational (slow path taken)
        for k in ("conf", "joint_prob", "entropy"):
            ok = close(go[k][b], oo[k][i], atol=1e-30)
            assert ok.all(), "%s seq %d %s" % (tag, b, k)


def to_np(d):
    return {k: v.detach().cpu().numpy() for k, v in d.items()}


def run_both(cfg, cls, layer_logits, seqs=None, splits=None, per_layer=True, tag=""):
    """layer_logits(l) -> device tensor [B][F][V].  GPU runs the whole batch; the oracle runs
    the sequences `seqs` (default all).  Returns (gpu_out, oracle_out, oracle_audit)."""
    B = cfg["B"]
    seqs = list(range(B)) if seqs is None else list(seqs)
    g = make_gpu(cfg, cls)
    if splits:
        g.set_row_splits(*splits)
    o = make_oracle(cfg, cls, B=len(seqs))
    g.reset(); o.reset()
    for l in range(cfg["D"]):
        x = layer_logits(l)
        g.expand_layer(x)
        torch.cuda.synchronize()
        xs = W.as_numpy_bits(x if len(seqs) == B and seqs == list(range(B)) else x[seqs])
        if o.frontier()["n_frontier"].sum() > 0:
            o.expand_layer(xs, threads=ORACLE_THREADS)
            if per_layer:
                compare_layer(to_np(g.candidates()), to_np(g.frontier()), o.candidates(), o.frontier(), seqs, cfg["K"],
                              "%s layer %d" % (tag, l))
        else:
            gf = to_np(g.frontier())
            assert all(int(gf["n_frontier"][b]) == 0 for b in seqs)
        del x
    go = to_np(g.finalize_tree())
    torch.cuda.synchronize()
    oo = o.finalize()
    compare_final(go, oo, seqs, tag)
    return go, oo, o.audit()
