"""GPU parity of whole draft phases (reset -> expand x D -> finalize) on the five benchmark
configurations: discrete outputs bit-exact with the oracle, reals within 1e-5 relative.  The two
batched configurations run at full size on the GPU; the oracle replays a sample of their
(independent) sequences."""
import numpy as np
import pytest
import torch

import workloads as W
from _harness import run_both, to_np, make_gpu

pytestmark = pytest.mark.gpu


def _layers(cfg, name, instance=0, keep=True):
    cache = {}

    def get(l):
        if l not in cache:
            if not keep:
                cache.clear()
            cache[l] = W.logits_layer(cfg, l, device="cuda", instance=instance)
        return cache[l]
    return get


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3"])
@pytest.mark.parametrize("instance", [0, 1, 2])
def test_single_sequence_configs(name, instance):
    cfg = W.CONFIGS[name]
    cls = W.classifier(cfg, W.classifier_seed(name))
    print("config", name, "instance", instance, flush=True)
    go, oo, audit = run_both(cfg, cls, _layers(cfg, name, instance), tag=name)
    print(name, "n_nodes", oo["n_nodes"], "scored", audit["scored"], "margins", audit["min_thr_margin"], audit["min_rank_gap"])


@pytest.mark.parametrize("name,sample", [("cfg4", 8), ("cfg5", 6)])
def test_batched_configs_full_size_sampled_oracle(name, sample):
    cfg = W.CONFIGS[name]
    cls = W.classifier(cfg, W.classifier_seed(name))
    rng = np.random.default_rng(7)
    seqs = sorted(rng.choice(cfg["B"], sample, replace=False).tolist())
    print("config", name, "oracle on sequences", seqs, flush=True)
    go, oo, audit = run_both(cfg, cls, _layers(cfg, name, keep=False), seqs=seqs, tag=name)
    n = go["n_nodes"]
    assert (n <= cfg["N"]).all() and n.sum() > 0
    # properties that hold for every sequence of the full batch, not only the sampled ones
    for b in range(cfg["B"]):
        k = int(n[b])
        par = go["parent"][b, :k]
        assert (par < np.arange(k)).all()
        m = go["mask"][b]
        assert (m.sum(axis=1)[:k] == go["position"][b, :k]).all()     # ancestors + self = depth + 1
        assert not m[k:].any()
    print(name, "nodes/seq mean %.1f" % n.mean(), "min margins", audit["min_thr_margin"].min(), audit["min_rank_gap"].min())


def test_split_rows_give_the_same_tree_and_reruns_are_bitwise_equal():
    cfg = dict(W.CONFIGS["cfg3"])
    cls = W.classifier(cfg, W.classifier_seed("cfg3"))
    layers = [W.logits_layer(cfg, l, device="cuda") for l in range(cfg["D"])]
    outs = []
    for splits in ((0, 0), (0, 0), (1, 1), (7, 3), (64, 16)):
        g = make_gpu(cfg, cls)
        if splits != (0, 0):
            g.set_row_splits(*splits)
        g.reset()
        for l in range(cfg["D"]):
            g.expand_layer(layers[l])
        outs.append(to_np(g.finalize_tree()))
        torch.cuda.synchronize()
    for k in outs[0]:
        np.testing.assert_array_equal(outs[0][k], outs[1][k], err_msg="rerun differs in " + k)   # determinism
    for o in outs[2:]:
        for k in ("tokens", "parent", "position", "n_nodes", "mask", "status"):
            np.testing.assert_array_equal(outs[0][k], o[k], err_msg="split changes " + k)
        for k in ("conf", "joint_prob", "entropy"):
            np.testing.assert_allclose(outs[0][k], o[k], rtol=1e-5)
