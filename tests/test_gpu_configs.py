"""GPU parity of whole draft phases (reset -> expand x D -> finalize) on the five benchmark
configurations: discrete outputs bit-exact with the oracle, reals within 1e-5 relative.  The two
batched configurations run at full size on the GPU; the oracle replays a sample of their
(independent) sequences."""
import numpy as np
import pytest
import torch

import workloads as W
from _harness import run_both, to_np, make_gpu, ORACLE_THREADS

pytestmark = pytest.mark.gpu


def _as_signed(t):
    return t.view(torch.int32) if t.dtype == torch.uint32 else t     # status is a uint32 bit field


def _layers(cfg, name, instance=0, keep=True):
    cache = {}

    def get(l):
        if l not in cache:
            if not keep:
                cache.clear()
            # single sequences: the CPU generator's stream, on which the classifier seeds were chosen
            # (torch's GPU generator gives other rows, and e.g. a cfg3 tree that dies at the root)
            gen = "cpu" if cfg["B"] == 1 else "cuda"
            cache[l] = W.logits_layer(cfg, l, device=gen, instance=instance).cuda()
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


@pytest.mark.parametrize("name,instance", [("cfg4", 0), ("cfg4", 1), ("cfg5", 0), ("cfg5", 1)])
def test_batched_configs_every_sequence_against_oracle(name, instance):
    # full batch on the GPU, and the oracle replays EVERY sequence (sharded over the host's threads),
    # layer by layer and at the end
    cfg = W.CONFIGS[name]
    cls = W.classifier(cfg, W.classifier_seed(name))
    print("config", name, "instance", instance, "oracle on all", cfg["B"], "sequences", flush=True)
    go, oo, audit = run_both(cfg, cls, _layers(cfg, name, instance=instance, keep=False), tag="%s inst %d" % (name, instance))
    n = go["n_nodes"]
    assert (n <= cfg["N"]).all() and n.sum() > 0
    assert int(audit["scored"].sum()) > cfg["B"] * cfg["K"]            # the trees grow beyond the root layer
    print(name, "instance", instance, "nodes/seq mean %.1f" % n.mean(), "scored", int(audit["scored"].sum()),
          "min margins", audit["min_thr_margin"].min(), audit["min_rank_gap"].min())


@pytest.mark.parametrize("name,sample,frac", [("cfg2", 1, 0.3), ("cfg4", 64, 0.01), ("cfg4", 64, 0.9)])
def test_masked_vocabulary_whole_trees(name, sample, frac):
    """Constrained decoding: the same scattered set of tokens has logit -inf in every row (probability
    0, ranked after every finite logit).  The bf16 rows stay on the histogram path."""
    cfg = W.CONFIGS[name]
    cls = W.classifier(cfg, W.classifier_seed(name))
    rng = np.random.default_rng(11)
    seqs = sorted(rng.choice(cfg["B"], sample, replace=False).tolist())
    masked = torch.from_numpy(rng.random(cfg["V"]) < frac).cuda()
    plain = _layers(cfg, name, keep=False)

    def layers(l):
        x = plain(l).clone()
        x.masked_fill_(masked, float("-inf"))
        return x
    print("config", name, "masked fraction", frac, "oracle on sequences", seqs, flush=True)
    go, oo, audit = run_both(cfg, cls, layers, seqs=seqs, tag="%s masked %g" % (name, frac))
    assert go["n_nodes"].sum() > 0
    k = int(go["n_nodes"][seqs[0]])
    assert not masked[torch.from_numpy(go["tokens"][seqs[0], 1:k].astype(np.int64)).cuda()].any()   # no masked token drafted
    if cfg["dtype"] == "bf16":
        assert not (go["status"] & 2).any()               # no row left the histogram path


@pytest.mark.parametrize("name,sample", [("cfg1", 1), ("cfg2", 1), ("cfg3", 1), ("cfg4", 64), ("cfg5", 256)])
def test_entropy_over_top_1000_whole_trees(name, sample):
    # the paper's own configuration of the H feature: Eq. 2, second line with M = 1000
    cfg = dict(W.CONFIGS[name], entropy_top_m=1000)
    rng = np.random.default_rng(3)
    seqs = sorted(rng.choice(cfg["B"], sample, replace=False).tolist())
    total = 0
    # the stored seeds were chosen for the full-vocabulary entropy; with another H feature the same
    # classifier may prune everything at the root, so a few neighbouring seeds are run as well
    for ds in range(1 if cfg["B"] > 1 else 4):
        cls = W.classifier(cfg, W.classifier_seed(name) + ds)
        print("config", name, "top-1000 entropy, classifier seed +%d, oracle on sequences" % ds, seqs, flush=True)
        go, oo, audit = run_both(cfg, cls, _layers(cfg, name, keep=cfg["B"] == 1), seqs=seqs, tag="%s M=1000 seed+%d" % (name, ds))
        print(name, "M=1000 n_nodes", go["n_nodes"][seqs].tolist())
        total += int(go["n_nodes"].sum())
    assert total > 0


def _compare_reranked(g, o, seqs, n_out, tag):
    go = to_np(g.finalize_tree_reranked(n_out))
    torch.cuda.synchronize()
    oo = o.finalize_rerank(n_out)
    for j, b in enumerate(seqs):
        n = int(oo["n_nodes"][j])
        assert int(go["n_nodes"][b]) == n, "%s n_out=%d seq %d: %d vs %d nodes" % (tag, n_out, b, go["n_nodes"][b], n)
        for k in ("tokens", "parent", "position"):
            np.testing.assert_array_equal(go[k][b], oo[k][j], err_msg="%s n_out=%d seq %d %s" % (tag, n_out, b, k))
        np.testing.assert_array_equal(go["mask"][b], oo["mask"][j], err_msg="%s mask" % tag)
        assert (go["status"][b] & 1) == (oo["status"][j] & 1)
        for k in ("conf", "joint_prob", "entropy"):
            np.testing.assert_allclose(go[k][b, :n], oo[k][j, :n], rtol=1e-5, err_msg="%s %s" % (tag, k))
    return go


@pytest.mark.parametrize("name,sample,eagle2", [("cfg1", 1, False), ("cfg2", 1, True), ("cfg3", 1, False), ("cfg4", 64, False),
                                                ("cfg4", 64, True), ("cfg5", 256, False), ("cfg5", 48, True)])
def test_reranked_finalize_against_oracle(name, sample, eagle2):
    # Sec. 2.2, EAGLE-2's reranking phase over every scored candidate.  eagle2: the classifier is the
    # joint probability itself and beta = 0, i.e. EAGLE-2's own expansion and rerank.
    cfg = dict(W.CONFIGS[name], rerank=1)
    if eagle2:
        cfg["beta"] = 0.0
        cfg["N"] = cfg["D"] * cfg["F"]                # the budget binds at the rerank, not in the expansion
        W1 = np.zeros((cfg["h"], 3), np.float32); W1[0, 0] = 1
        w2 = np.zeros(cfg["h"], np.float32); w2[0] = 1
        cls = (W1, np.zeros(cfg["h"], np.float32), w2, 0.0)
    else:
        cls = W.classifier(cfg, W.classifier_seed(name))
    rng = np.random.default_rng(5)
    seqs = sorted(rng.choice(cfg["B"], sample, replace=False).tolist())
    print("config", name, "rerank, eagle2 =", eagle2, "oracle on sequences", seqs, flush=True)
    from _harness import make_oracle
    layers = _layers(cfg, name, keep=cfg["B"] == 1)
    g = make_gpu(cfg, cls)
    o = make_oracle(cfg, cls, B=len(seqs))
    g.reset(); o.reset()
    for l in range(cfg["D"]):
        x = layers(l)
        g.expand_layer(x)
        if o.frontier()["n_frontier"].sum() > 0:
            o.expand_layer(W.as_numpy_bits(x if len(seqs) == cfg["B"] else x[seqs]), threads=ORACLE_THREADS)
        del x
    torch.cuda.synchronize()
    total = int(o.audit()["scored"].max())
    for n_out in sorted({1, 7, min(60, 1024), min(1024, max(1, total // 2)), min(1024, total + 3)}):
        go = _compare_reranked(g, o, seqs, n_out, name)
    print(name, "rerank: scored per sequence up to", total, "; last n_nodes", go["n_nodes"][seqs].tolist())


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_first_pruning_is_strict_at_equality(dtype):
    # Algorithm 1 keeps C_i > beta: a candidate whose classifier logit EQUALS logit(beta) is dropped.
    # Zero weights give z = b2 for every candidate.
    cfg = dict(idx=98, B=3, V=2008, dtype=dtype, D=3, F=4, K=4, h=4, beta=0.5, N=20,
               zipf_s=1.0, sigma=(1.0, 4.0), spike_frac=0.0, desc="equality at the threshold")
    zero = (np.zeros((4, 3), np.float32), np.zeros(4, np.float32), np.zeros(4, np.float32))
    layers = _layers(cfg, "eq")
    go, oo, _ = run_both(cfg, zero + (0.0,), layers, tag="z == logit(beta)")
    assert (go["n_nodes"] == 0).all() and (oo["n_nodes"] == 0).all()
    up = float(np.nextafter(np.float32(0), np.float32(1)))
    go, oo, _ = run_both(cfg, zero + (up,), layers, tag="z one ulp above logit(beta)")
    assert (go["n_nodes"] == 4 + 2 * 4).all()
    go, oo, _ = run_both(cfg, zero + (-up,), layers, tag="z one ulp below logit(beta)")
    assert (go["n_nodes"] == 0).all()
    cfg3 = dict(cfg, beta=0.3)
    from oracle import ref_logit_of_beta
    zb = np.float32(ref_logit_of_beta(0.3))
    go, oo, _ = run_both(cfg3, zero + (float(zb),), layers, tag="z == logit(0.3)")
    assert (go["n_nodes"] == 0).all()
    go, oo, _ = run_both(cfg3, zero + (float(np.nextafter(zb, np.float32(1))),), layers, tag="z above logit(0.3)")
    assert (go["n_nodes"] > 0).all()


@pytest.mark.parametrize("F,K,N", [(10, 10, 30), (32, 32, 100), (64, 32, 200)])
def test_candidates_with_equal_confidence_are_ranked_by_token_and_slot(F, K, N):
    # Equal classifier logits are the rule deep in a tree (P too small to move the fp32 sum: the K children of a row
    # share H and d).  The extreme cases: every candidate of a layer with the same z (zero weights), and z a function
    # of the row alone (one unit on H): the second pruning is then decided by token id and frontier slot alone.
    cfg = dict(idx=96, B=3, V=5000, dtype="bf16", D=4, F=F, K=K, h=4, beta=0.5, N=N,
               zipf_s=1.0, sigma=(1.0, 4.0), spike_frac=0.0, desc="equal confidences")
    layers = _layers(cfg, "ties")
    zero = (np.zeros((4, 3), np.float32), np.zeros(4, np.float32), np.zeros(4, np.float32), 1.0)
    go, oo, audit = run_both(cfg, zero, layers, tag="all z equal F=%d K=%d" % (F, K))
    assert (go["n_nodes"] == N).all() and len(np.unique(go["conf"][:, :N])) == 1
    W1 = np.zeros((4, 3), np.float32); W1[0, 1] = 1.0
    on_h = (W1, np.zeros(4, np.float32), np.array([1, 0, 0, 0], np.float32), 0.25)
    go, oo, audit = run_both(cfg, on_h, layers, tag="z from H alone F=%d K=%d" % (F, K))
    assert (go["n_nodes"] == N).all()

    # every frontier node of a sequence with the same logits row: the same K tokens under every parent, with the
    # same z: the selection is decided by the frontier slot, the last tie-break
    def same_rows(l):
        x = layers(l).clone()
        x[:, 1:, :] = x[:, :1, :]
        return x
    go, oo, audit = run_both(cfg, zero, same_rows, tag="equal rows, all z equal F=%d K=%d" % (F, K))
    assert (go["n_nodes"] == N).all()
    for b in range(cfg["B"]):                           # layer 1: the lowest token ids, each from every slot in turn
        first = min(F, K)
        t = go["tokens"][b, first:first + min(F, N - first)]
        assert (np.diff(t) >= 0).all() and len(set(t.tolist())) == -(-len(t) // first)


def test_reranked_finalize_with_whole_families_tied():
    # a classifier that grows with the depth: most children score above their parent, so their path
    # minimum equals the parent's and the reranking is decided by its tie rules (depth, then scoring order)
    from _harness import make_oracle
    cfg = dict(idx=99, B=6, V=3000, dtype="bf16", D=5, F=8, K=8, h=2, beta=0.3, N=40, rerank=1,
               zipf_s=1.0, sigma=(1.0, 4.0), spike_frac=0.0, desc="rerank ties")
    W1 = np.zeros((2, 3), np.float32); W1[0] = (0.4, 0.0, 0.75); W1[1] = (-1.0, 0.1, 0.0)
    cls = (W1, np.array([0.1, 0.3], np.float32), np.array([1.0, -0.7], np.float32), -0.5)
    layers = _layers(cfg, "rerank_ties")
    g = make_gpu(cfg, cls)
    o = make_oracle(cfg, cls)
    g.reset(); o.reset()
    for l in range(cfg["D"]):
        x = layers(l)
        g.expand_layer(x)
        if o.frontier()["n_frontier"].sum() > 0:
            o.expand_layer(W.as_numpy_bits(x), threads=4)
    torch.cuda.synchronize()
    total = int(o.audit()["scored"].max())
    everything = o.finalize_rerank(total)
    s = everything["path_min_z"][0, :int(everything["n_nodes"][0])]
    assert (np.diff(s) == 0).sum() > 20, "the classifier is meant to tie whole families"
    for n_out in (1, 9, total // 3, total // 2, total, min(1024, total + 5)):
        _compare_reranked(g, o, list(range(cfg["B"])), n_out, "rerank ties")


def test_batched_chain_mode_ragged_lengths():
    # Sec. 5.5: one child per node; the classifier is an early-exit rule and sequences stop at
    # different depths.  Full batch on the GPU, and the oracle replays every sequence.
    cfg = W.CONFIGS["chain"]
    cls = W.classifier(cfg, W.classifier_seed("chain"))
    rng = np.random.default_rng(11)
    seqs = list(range(cfg["B"]))                        # every one of the 1024 chains
    print("config chain, oracle on all", len(seqs), "sequences", flush=True)
    go, oo, audit = run_both(cfg, cls, _layers(cfg, "chain"), seqs=seqs, tag="chain")
    n = go["n_nodes"]
    assert len(set(n.tolist())) >= 3, "the workload is meant to have ragged chain lengths"
    for b in range(cfg["B"]):
        k = int(n[b])
        np.testing.assert_array_equal(go["parent"][b, :k], np.arange(k) - 1)          # a chain
        np.testing.assert_array_equal(go["position"][b, :k], np.arange(k) + 1)
        np.testing.assert_array_equal(go["mask"][b, :k, :k], np.tril(np.ones((k, k), np.uint8)))
    print("chain lengths: mean %.2f, histogram" % n.mean(), np.bincount(n, minlength=cfg["D"] + 1).tolist())


def test_split_rows_give_the_same_tree_and_reruns_are_bitwise_equal():
    cfg = dict(W.CONFIGS["cfg3"])
    cls = W.classifier(cfg, W.classifier_seed("cfg3"))
    layers = [W.logits_layer(cfg, l, device="cuda") for l in range(cfg["D"])]
    outs = []
    for splits in ((0, 0), (0, 0), (1, 1), (7, 3), (64, 16)):
        g = make_gpu(cfg, cls)
        if splits != (0, 0):
            g.set_row_splits(*splits)
        # by default the 16 rows of a layer (and the root row) are shared by four workgroups each; a count that is set is taken literally
        assert g.row_workgroups() == ((4, 4) if splits == (0, 0) else splits)
        g.reset()
        for l in range(cfg["D"]):
            g.expand_layer(layers[l])
        outs.append(to_np(g.finalize_tree()))
        torch.cuda.synchronize()
    for k in outs[0]:
        np.testing.assert_array_equal(outs[0][k], outs[1][k], err_msg="rerun differs in " + k)   # determinism
    for k in outs[0]:                                   # shared rows add the same counts up: nothing differs from unshared rows
        np.testing.assert_array_equal(outs[0][k], outs[2][k], err_msg="sharing rows changes " + k)
    for o in outs[2:]:
        for k in ("tokens", "parent", "position", "n_nodes", "mask", "status"):
            np.testing.assert_array_equal(outs[0][k], o[k], err_msg="split changes " + k)
        for k in ("conf", "joint_prob", "entropy"):
            np.testing.assert_allclose(outs[0][k], o[k], rtol=1e-5)


@pytest.mark.parametrize("name,opts", [("cfg2", {}), ("cfg3", {}), ("cfg4", {}), ("cfg4", {"entropy_top_m": 1000}), ("cfg2", {"rerank": 1})])
def test_a_draft_phase_replayed_from_a_hip_graph(name, opts):
    """reset -> D x expand -> finalize captured once and replayed: every replay, with eager work of
    the same context and synchronisations in between, gives the eager result bit for bit (the
    library enqueues kernels only: no memset nodes, no allocation, nothing host-side per call
    that a replay would miss)."""
    cfg = dict(W.CONFIGS[name]); cfg.update(opts)
    cls = W.classifier(cfg, W.classifier_seed(name))
    gen = "cpu" if cfg["B"] == 1 else "cuda"
    layers = [W.logits_layer(cfg, l, device=gen).cuda() for l in range(cfg["D"])]
    other = [W.logits_layer(cfg, l, device=gen, instance=1).cuda() for l in range(cfg["D"])]
    g = make_gpu(cfg, cls)
    n_out = 48 if opts.get("rerank") else None
    out_graph, out_eager = g.new_tree_out(n_out), g.new_tree_out(n_out)

    def phase(ls, out):
        g.reset()
        for l in range(cfg["D"]):
            g.expand_layer(ls[l])
        return g.finalize_tree_reranked(n_out, out) if n_out else g.finalize_tree(out)

    eager = {k: v.clone() for k, v in phase(layers, out_eager).items()}
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        phase(layers, out_graph)                          # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        phase(layers, out_graph)
    for replay in range(4):
        for v in out_graph.values():
            _as_signed(v).fill_(-7)                       # a replay must rewrite every output
        graph.replay()
        torch.cuda.synchronize()
        for k in eager:
            assert torch.equal(_as_signed(out_graph[k]), _as_signed(eager[k])), "replay %d differs in %s" % (replay, k)
        phase(other, out_eager)                           # eager work on other inputs between the replays
        torch.cuda.synchronize()
    assert int(eager["n_nodes"].sum()) > 0


LIMIT_CASES = {
    # name: (B, V, dtype, D, F, K, h, beta, N): the compiled limits of the kernels, odd vocabularies
    "max_candidates_bf16": (3, 20011, "bf16", 3, 64, 32, 256, 0.2, 1024),
    "max_topk_bf16": (2, 5003, "bf16", 3, 32, 64, 64, 0.3, 100),
    "max_candidates_f32": (2, 4099, "f32", 3, 64, 32, 16, 0.2, 200),
    "wide_frontier_keep_all": (2, 9000, "bf16", 3, 64, 16, 8, 0.0, 1024),
    "tiny_vocab": (5, 70, "bf16", 4, 8, 8, 4, 0.1, 30),
    # a vocabulary of one 16-byte chunk or less, and as many children as tokens
    "one_chunk_vocab_bf16": (3, 8, "bf16", 3, 4, 8, 3, 0.0, 12),
    "sub_chunk_vocab_bf16": (3, 5, "bf16", 3, 3, 5, 3, 0.0, 9),
    "sub_chunk_vocab_f32": (3, 3, "f32", 3, 3, 3, 3, 0.0, 9),
    "budget_one": (4, 1000, "f32", 3, 4, 4, 4, 0.0, 1),
    # launches of one round with more workgroups than CUs deal the live rows round the CUs: batch sizes
    # that are not multiples of the wave size, small budgets (frontiers of very different lengths,
    # sequences without a frontier in the later layers), both kernels, the largest such batch
    "dealt_rows_b100": (100, 3001, "bf16", 5, 8, 8, 8, 0.3, 12),
    "dealt_rows_b200_f32": (200, 1003, "f32", 4, 4, 4, 4, 0.3, 6),
    "dealt_rows_b256": (256, 517, "bf16", 4, 4, 4, 4, 0.4, 5),
    # few long rows: several workgroups count one row and hand their histograms over.  Five sequences with ragged
    # frontiers and small budgets (sequences without a frontier among shared rows), five workgroups per row, the last
    # with nothing but the row's partial chunk; a hundred one-row sequences, two workgroups per row
    "shared_rows_b5": (5, 65541, "bf16", 4, 8, 8, 8, 0.3, 14),
    "shared_rows_b100": (100, 49163, "bf16", 3, 1, 4, 4, 0.3, 3),
    # hidden widths that are not multiples of four: the classifier's arrays then start off 16 bytes
    "odd_hidden_7": (3, 1500, "bf16", 3, 4, 4, 7, 0.3, 10),
    "odd_hidden_1": (2, 900, "bf16", 3, 4, 4, 1, 0.3, 10),
}


@pytest.mark.parametrize("case", sorted(LIMIT_CASES))
def test_limits_of_the_kernels(case):
    B, V, dtype, D, F, K, h, beta, N = LIMIT_CASES[case]
    cfg = dict(idx=90 + sorted(LIMIT_CASES).index(case), B=B, V=V, dtype=dtype, D=D, F=F, K=K, h=h, beta=beta, N=N,
               zipf_s=1.0, sigma=(1.0, 4.0), spike_frac=0.1, desc=case)
    total = 0
    for seed in range(3):
        cls = W.classifier(cfg, seed)
        print("limits", case, "classifier seed", seed, flush=True)
        base = _layers(cfg, case)

        def padded(l, base=base):
            # row stride rounded up to 16 bytes plus one spare chunk, padding poisoned with +inf
            x = base(l)
            epc = 8 if dtype == "bf16" else 4
            stride = (V + epc - 1) // epc * epc + epc
            xp = torch.full((B, F, stride), float("inf"), dtype=x.dtype, device=x.device)
            xp[:, :, :V] = x
            return xp[:, :, :V]
        go, oo, audit = run_both(cfg, cls, padded, tag="%s seed %d" % (case, seed))
        total += int(go["n_nodes"].sum())
        print(case, "n_nodes", go["n_nodes"].tolist(), "scored", audit["scored"].tolist())
    assert total > 0


def test_reranked_finalize_at_the_history_limit():
    # max_depth * max_frontier * top_k = 32768 = C2T_MAX_HISTORY, 1024 nodes out; keep-all classifier
    # with many equal confidences (saturating hidden unit), so that ties at the n-th key occur
    from _harness import make_oracle
    B, V, D, F, K, h = 2, 5003, 16, 64, 32, 4
    cfg = dict(idx=97, B=B, V=V, dtype="bf16", D=D, F=F, K=K, h=h, beta=0.0, N=1024, rerank=1,
               zipf_s=1.0, sigma=(1.0, 4.0), spike_frac=0.0, desc="rerank limit")
    W1 = np.zeros((h, 3), np.float32); W1[0, 0] = -1e6        # relu(b1 - 1e6 P) is 0 for all but vanishing P
    b1 = np.zeros(h, np.float32); b1[0] = 1e-3
    w2 = np.zeros(h, np.float32); w2[0] = 1.0
    cls = (W1, b1, w2, 0.25)
    base = _layers(cfg, "rerank_limit")

    def padded(l):
        x = base(l)
        xp = torch.full((B, F, V + 13), float("inf"), dtype=x.dtype, device=x.device)
        xp[:, :, :V] = x
        return xp[:, :, :V]
    g = make_gpu(cfg, cls)
    o = make_oracle(cfg, cls)
    g.reset(); o.reset()
    for l in range(D):
        x = padded(l)
        g.expand_layer(x)
        if o.frontier()["n_frontier"].sum() > 0:
            o.expand_layer(W.as_numpy_bits(x), threads=4)
    torch.cuda.synchronize()
    print("scored per sequence", o.audit()["scored"].tolist(), flush=True)
    for n_out in (1024, 333, 1):
        _compare_reranked(g, o, list(range(B)), n_out, "rerank limit")
