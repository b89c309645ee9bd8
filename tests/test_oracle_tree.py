"""Pins for the oracle's classifier (Eq. 3), layer loop (Algorithm 1, Sec. 4.2) and tree
emission: hand-computable cases, the EAGLE-2 reduction (Sec. 2.2), chain mode (Sec. 5.5),
the paper's tree-size arithmetic (Appendix B.1), invariants and brute force on tiny inputs.
CPU only."""
import json
import math
import os

import numpy as np
import pytest
from scipy.special import softmax

import _second_impl as second
from oracle import RefTree, ref_logit_of_beta, ref_mlp_logit

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.json")))
f32 = np.float32


def identity_on_P(h):
    """z = P exactly: one unit with W1 = (1,0,0), b1 = 0, w2 = 1 (P >= 0 so ReLU is transparent)."""
    W1 = np.zeros((h, 3), f32); W1[0, 0] = 1
    return W1, np.zeros(h, f32), np.eye(1, h, 0, dtype=f32)[0], 0.0


def random_logits(rng, D, F, V, scale=2.0, bf16=False):
    x = (scale * rng.standard_normal((D, 1, F, V)) - 1.1 * np.log(rng.permutation(V) + 1.0)).astype(f32)
    if bf16:
        u = x.view(np.uint32).astype(np.uint64)
        x = ((u + ((u >> 16) & 1) + 0x7FFF) >> 16).astype(np.uint16)
    return x


def run(tree, logits):
    tree.reset()
    for l in range(tree.D):
        if tree.frontier()["n_frontier"].sum() == 0:
            break
        tree.expand_layer(logits[l])
    return tree.finalize()


# ---------------- classifier ----------------
def test_mlp_hand_cases():
    h = 4
    Z = np.zeros((h, 3), f32)
    assert ref_mlp_logit(Z, np.zeros(h, f32), np.zeros(h, f32), 0.75, 0.3, 2.0, 1.0) == f32(0.75)
    # single active unit: z = b2 + w2*(w.P + b1)
    W1 = Z.copy(); W1[2] = (0.5, 0.25, -1.0)
    b1 = np.zeros(h, f32); b1[2] = 0.125
    w2 = np.zeros(h, f32); w2[2] = 2.0
    assert ref_mlp_logit(W1, b1, w2, -1.0, 0.5, 2.0, 0.0) == f32(-1.0 + 2.0 * (0.25 + 0.5 + 0.125))
    # ReLU kills a negative pre-activation
    assert ref_mlp_logit(W1, b1, w2, -1.0, 0.5, 2.0, 3.0) == f32(-1.0)
    # sigmoid(0) = 0.5  <=>  logit(0.5) = 0 ; beta = 0 keeps everything
    assert ref_logit_of_beta(0.5) == 0.0
    assert ref_logit_of_beta(0.0) == -np.inf
    assert abs(ref_logit_of_beta(0.3) - math.log(0.3 / 0.7)) < 1e-7


def test_mlp_against_float64_and_second_impl():
    rng = np.random.default_rng(11)
    for h in (2, 12, 48, 64):
        W1 = (0.5 * rng.standard_normal((h, 3))).astype(f32)
        b1 = (0.5 * rng.standard_normal(h)).astype(f32)
        w2 = (0.5 * rng.standard_normal(h)).astype(f32)
        b2 = f32(0.1)
        for _ in range(20):
            P, H, d = f32(rng.random()), f32(10 * rng.random()), f32(rng.integers(0, 11))
            z = ref_mlp_logit(W1, b1, w2, b2, P, H, d)
            feat = np.array([P, H, d], np.float64)
            z64 = float(b2) + w2.astype(np.float64) @ np.maximum(W1.astype(np.float64) @ feat + b1, 0)
            assert abs(z - z64) < 1e-5 * max(1.0, abs(z64))
            assert z == second.mlp_logit(W1, b1, w2, b2, P, H, d)   # same fused order, numpy emulation


def test_mlp_flop_model_matches_paper_arithmetic():
    # Appendix E.2: 3h (input layer) + h (activation) + h (output layer) = 5h per token
    g = GOLD["overhead_model"]
    per_token = 3 * g["h"] + g["h"] + g["h"]
    assert per_token == 5 * g["h"]
    assert g["K"] * g["d_max"] * per_token == g["classifier_ops"]
    assert g["K"] * g["d_max"] * g["M"] == g["entropy_ops"]
    assert g["entropy_ops"] + g["classifier_ops"] == g["total_ops"]


# ---------------- EAGLE-2 reduction ----------------
def test_identity_classifier_reproduces_eagle2_expansion():
    # Sec. 2.2: each node generates TopK children, then the TopK of all generated tokens by
    # joint probability form the next layer; the joint probability never grows along a path.
    rng = np.random.default_rng(21)
    V, F, K, D, h = 300, 4, 4, 5, 3
    logits = random_logits(rng, D, F, V)
    t = RefTree(1, V, F, K, D, 100, h, 0, 0.0)
    t.set_classifier(*identity_on_P(h))
    out = run(t, logits)
    # independent expansion: scipy softmax, plain sort by joint probability
    frontier = [(1.0, -1)]           # (P, node index)
    nodes = []
    for l in range(D):
        children = []
        for slot, (Pp, par) in enumerate(frontier):
            p = softmax(logits[l][0][slot].astype(np.float64))
            for tok in np.lexsort((np.arange(V), -logits[l][0][slot]))[:K]:
                children.append((f32(f32(Pp) * f32(p[tok])), int(tok), slot, par))
        children.sort(key=lambda c: (-float(c[0]), c[1], c[2]))
        frontier = []
        for c in children[:F]:
            frontier.append((c[0], len(nodes)))
            nodes.append(c)
    n = out["n_nodes"][0]
    assert n == len(nodes) == F * (D - 1) + K
    np.testing.assert_array_equal(out["tokens"][0, :n], [c[1] for c in nodes])
    np.testing.assert_array_equal(out["parent"][0, :n], [c[3] for c in nodes])
    np.testing.assert_array_equal(out["joint_prob"][0, :n], np.array([c[0] for c in nodes], f32))
    np.testing.assert_array_equal(out["z"][0, :n], out["joint_prob"][0, :n])      # z == P exactly
    for i in range(n):
        par = out["parent"][0, i]
        if par >= 0:
            assert out["joint_prob"][0, i] <= out["joint_prob"][0, par]


def test_rerank_with_identity_classifier_is_eagle2_top_n():
    # Sec. 2.2, reranking phase: with value = joint probability, all candidate nodes of the
    # expansion are reranked and the top N selected; the joint probability never grows along a path,
    # so the selection is a tree.  Independent construction: scipy softmax, plain sort.
    rng = np.random.default_rng(23)
    V, F, K, D, h = 200, 3, 3, 4, 2
    logits = random_logits(rng, D, F, V)
    t = RefTree(1, V, F, K, D, 100, h, 0, 0.0)
    t.set_classifier(*identity_on_P(h))
    run(t, logits)
    frontier = [(1.0, -1)]
    cands = []                        # every generated token: (P, depth, order, token, parent cand index)
    for l in range(D):
        children = []
        for slot, (Pp, par) in enumerate(frontier):
            p = softmax(logits[l][0][slot].astype(np.float64))
            for tok in np.lexsort((np.arange(V), -logits[l][0][slot]))[:K]:
                children.append((f32(f32(Pp) * f32(p[tok])), int(tok), slot, par))
        base = len(cands)
        for i, c in enumerate(children):
            cands.append((c[0], l, base + i, c[1], c[3]))
        ranked = sorted(range(len(children)), key=lambda i: (-float(children[i][0]), children[i][1], children[i][2]))
        frontier = [(children[i][0], base + i) for i in ranked[:F]]
    assert len(cands) == K + (D - 1) * F * K
    for n_out in (1, 5, 12, len(cands), len(cands) + 7):
        out = t.finalize_rerank(n_out)
        want = sorted(cands, key=lambda c: (-float(c[0]), c[1], c[2]))[:n_out]
        n = int(out["n_nodes"][0])
        assert n == len(want)
        np.testing.assert_array_equal(out["tokens"][0, :n], [c[3] for c in want])
        np.testing.assert_array_equal(out["joint_prob"][0, :n], np.array([c[0] for c in want], f32))
        np.testing.assert_array_equal(out["position"][0, :n], [c[1] + 1 for c in want])
        pos = {c[2]: i for i, c in enumerate(want)}
        np.testing.assert_array_equal(out["parent"][0, :n], [-1 if c[4] < 0 else pos[c[4]] for c in want])
        assert not out["mask"][0, n:].any() and (out["tokens"][0, n:] == -1).all()


def test_rerank_selection_is_a_tree_for_any_classifier():
    # a classifier that is not monotone along paths: ranking by the path minimum of z keeps the
    # selection closed under "parent of"; brute force over the recorded forest
    rng = np.random.default_rng(24)
    V, F, K, D, h = 64, 4, 3, 5, 6
    for trial in range(6):
        logits = random_logits(rng, D, F, V)
        cls = ((0.8 * rng.standard_normal((h, 3))).astype(f32), (0.5 * rng.standard_normal(h)).astype(f32),
               (0.8 * rng.standard_normal(h)).astype(f32), f32(0.2))
        t = RefTree(1, V, F, K, D, 100, h, 0, 0.3)
        t.set_classifier(*cls)
        run(t, logits)
        total = int(t.audit()["scored"][0])
        everything = t.finalize_rerank(total + 3)
        assert int(everything["n_nodes"][0]) == total
        for n_out in (1, 7, total // 2, total):
            out = t.finalize_rerank(n_out)
            n = int(out["n_nodes"][0])
            assert n == min(n_out, total)
            par, s, z = out["parent"][0, :n], out["path_min_z"][0, :n], everything
            assert (par < np.arange(n)).all()                                     # parents come first
            assert (np.diff(s) <= 0).all()                                        # best path minimum first
            for i in range(n):
                zi = -np.log(1.0 / np.float64(out["conf"][0, i]) - 1.0)           # conf = sigmoid(z)
                want = zi if par[i] < 0 else min(s[par[i]], zi)
                assert abs(s[i] - want) <= 1e-5 * max(1.0, abs(want))            # s = min over the path
                anc = {i}; j = i
                while par[j] >= 0:
                    j = par[j]; anc.add(j)
                assert set(np.nonzero(out["mask"][0, i])[0].tolist()) == anc
                assert out["position"][0, i] == len(anc)
            # nothing left out beats something selected
            if n < total:
                assert everything["path_min_z"][0, n:total].max() <= s.min()
            # a prefix of the full ranking
            np.testing.assert_array_equal(out["tokens"][0, :n], everything["tokens"][0, :n])


def _independent_rerank(layers_dump, F, N, zb):
    """Every scored candidate of a draft phase, rebuilt from the per-layer candidate dumps alone
    (z, token, slot in scoring order), with its parent and s = smallest z on its path, and the
    frontier of each layer re-derived with python's sort.  Returns the candidates in the order of
    Sec. 2.2's reranking as this build reads it: (s desc, depth asc, scoring order asc)."""
    cands = []                 # dict(idx, depth, token, z, s, parent)
    frontier = [-1]            # history index of the node in each frontier slot; -1 = root
    n_nodes = 0
    for depth, c in enumerate(layers_dump):
        base = len(cands)
        for i in range(len(c["z"])):
            par = frontier[int(c["slot"][i])]
            z = float(c["z"][i])
            cands.append(dict(idx=base + i, depth=depth, token=int(c["token"][i]), z=z, parent=par,
                              s=z if par < 0 else min(cands[par]["s"], z), slot=int(c["slot"][i])))
        layer = cands[base:]
        surv = sorted((q for q in layer if q["z"] > zb), key=lambda q: (-q["z"], q["token"], q["slot"]))
        keep = surv[:max(0, min(F, N - n_nodes))]
        n_nodes += len(keep)
        frontier = [q["idx"] for q in keep]
        if not frontier:
            break
    return sorted(cands, key=lambda q: (-q["s"], q["depth"], q["idx"]))


def test_rerank_tie_order_against_an_independent_sort():
    # Sec. 2.2's reranking with a classifier that is NOT monotone along paths and grows with depth:
    # most children score above their parent, so their path minimum s equals the parent's and whole
    # families tie in s.  The order among equal s (depth first, then scoring order) is checked against
    # python's sort over the candidate dumps, not against the oracle's own full ranking.
    rng = np.random.default_rng(29)
    V, F, K, D, h, N = 80, 4, 3, 5, 2, 100
    ties_seen = 0
    for trial in range(8):
        logits = random_logits(rng, D, F, V)
        W1 = np.zeros((h, 3), f32); W1[0] = (0.5 * rng.standard_normal(), 0.0, 0.75)      # z rises with the depth
        W1[1] = (-1.0, 0.1, 0.0)
        cls = (W1, np.array([0.1, 0.3], f32), np.array([1.0, float(rng.standard_normal())], f32), f32(-0.5))
        beta = 0.3
        t = RefTree(1, V, F, K, D, N, h, 0, beta)
        t.set_classifier(*cls)
        t.reset()
        dumps = []
        for l in range(D):
            if t.frontier()["n_frontier"].sum() == 0:
                break
            t.expand_layer(logits[l])
            c = t.candidates()
            n = int(c["n_cand"][0])
            dumps.append({k: c[k][0, :n].copy() for k in ("z", "token", "slot")})
        want_all = _independent_rerank(dumps, F, N, ref_logit_of_beta(beta))
        total = len(want_all)
        assert total == int(t.audit()["scored"][0])
        s_all = [q["s"] for q in want_all]
        ties_seen += sum(1 for a, b in zip(s_all, s_all[1:]) if a == b)
        for n_out in (1, 4, total // 3, total // 2, total, total + 2):
            out = t.finalize_rerank(n_out)
            want = want_all[:n_out]
            n = int(out["n_nodes"][0])
            assert n == len(want)
            np.testing.assert_array_equal(out["tokens"][0, :n], [q["token"] for q in want])
            np.testing.assert_array_equal(out["position"][0, :n], [q["depth"] + 1 for q in want])
            np.testing.assert_array_equal(out["path_min_z"][0, :n], np.array([q["s"] for q in want], f32))
            pos = {q["idx"]: i for i, q in enumerate(want)}
            np.testing.assert_array_equal(out["parent"][0, :n], [-1 if q["parent"] < 0 else pos[q["parent"]] for q in want])
    assert ties_seen > 50, "the classifier is meant to produce many equal path minima"


def test_first_pruning_is_strict_at_equality():
    # Algorithm 1: the loop runs while C_i > beta and removes C_i < beta; at C_i == beta this build
    # drops the node (strict '>').  All-zero weights give z = b2 for every candidate: with b2 = 0 and
    # beta = 0.5, z == logit(beta) == 0 exactly and the tree stays empty; one ulp above, everything passes.
    rng = np.random.default_rng(30)
    V, F, K, D, h, N = 50, 3, 4, 3, 2, 20
    logits = random_logits(rng, D, F, V)
    zero = (np.zeros((h, 3), f32), np.zeros(h, f32), np.zeros(h, f32))
    t = RefTree(1, V, F, K, D, N, h, 0, 0.5)
    t.set_classifier(*zero, 0.0)
    t.reset()
    t.expand_layer(logits[0])
    c = t.candidates()
    assert c["n_cand"][0] == K and (c["z"][0, :K] == 0.0).all() and not c["kept"][0].any()
    assert t.frontier()["n_frontier"][0] == 0
    assert t.finalize()["n_nodes"][0] == 0
    t.set_classifier(*zero, float(np.nextafter(f32(0), f32(1))))
    out = run(t, logits)
    assert out["n_nodes"][0] == min(F, K) + (D - 1) * F        # every layer keeps max_frontier nodes
    t.set_classifier(*zero, float(np.nextafter(f32(0), f32(-1))))
    assert run(t, logits)["n_nodes"][0] == 0
    # a threshold other than 0.5: z equal to the rounded logit(beta) is dropped as well
    zb = ref_logit_of_beta(0.3)
    t = RefTree(1, V, F, K, D, N, h, 0, 0.3)
    t.set_classifier(*zero, float(zb))
    assert run(t, logits)["n_nodes"][0] == 0
    t.set_classifier(*zero, float(np.nextafter(f32(zb), f32(1))))
    assert run(t, logits)["n_nodes"][0] > 0


def test_candidate_count_matches_paper_tree_size():
    # Appendix B.1: K = 10, d_max = 11 gives complete trees of 1011 nodes = root + K + (d_max-1)*K*K
    g = GOLD["training_tree"]
    K, D = g["K"], g["d_max"]
    assert g["trees"] * g["nodes_with_root"] == g["entries"]
    rng = np.random.default_rng(22)
    V, h = 64, 2
    logits = random_logits(rng, D, K, V)
    t = RefTree(1, V, K, K, D, 2000, h, 0, 0.0)         # beta = 0, budget never binds: full frontiers
    t.set_classifier(*identity_on_P(h))
    run(t, logits)
    scored = int(t.audit()["scored"][0])
    assert scored == K + (D - 1) * K * K
    assert scored + 1 == g["nodes_with_root"]


# ---------------- chain mode ----------------
def test_chain_mode_is_argmax_path_with_early_exit():
    # Sec. 5.5: with one child per node the tree is a chain and C2T is an early-exit rule
    rng = np.random.default_rng(23)
    V, D, h = 200, 8, 3
    logits = random_logits(rng, D, 1, V, scale=1.0)
    beta = 0.02
    t = RefTree(1, V, 1, 1, D, 100, h, 0, beta)
    W1, b1, w2, _ = identity_on_P(h)
    # z = P + logit(beta): confidence sigmoid(z) > beta  <=>  P > 0 ... use z = 8*P - 4 instead
    W1[0, 0] = 8.0
    t.set_classifier(W1, b1, w2, -4.0)
    out = run(t, logits)
    zb = math.log(beta / (1 - beta))
    P, expect = 1.0, []
    for l in range(D):
        p = softmax(logits[l][0][0].astype(np.float64))
        tok = int(np.argmax(logits[l][0][0]))
        P = float(f32(f32(P) * f32(p[tok])))
        if not (float(f32(8.0) * f32(P) + f32(-4.0)) > zb):
            break
        expect.append(tok)
    n = out["n_nodes"][0]
    assert 0 < n < D, "choose the test so that the chain stops early"
    np.testing.assert_array_equal(out["tokens"][0, :n], expect)
    np.testing.assert_array_equal(out["parent"][0, :n], np.arange(n) - 1)
    np.testing.assert_array_equal(out["position"][0, :n], np.arange(n) + 1)


# ---------------- invariants on random instances ----------------
@pytest.mark.parametrize("bf16", [False, True])
def test_tree_invariants(bf16):
    rng = np.random.default_rng(31)
    V, F, K, D, N, h, beta = 500, 6, 5, 6, 20, 12, 0.45
    B = 3
    logits = np.concatenate([random_logits(rng, D, F, V, bf16=bf16) for _ in range(B)], axis=1)
    found = False
    for seed in range(40):
        r2 = np.random.default_rng(1000 + seed)
        cls = ((0.5 * r2.standard_normal((h, 3))).astype(f32), (0.5 * r2.standard_normal(h)).astype(f32),
               (0.5 * r2.standard_normal(h)).astype(f32), float(0.5 * r2.standard_normal()))
        t = RefTree(B, V, F, K, D, N, h, 1 if bf16 else 0, beta)
        t.set_classifier(*cls)
        t.reset()
        zb = ref_logit_of_beta(beta)
        for l in range(D):
            nf = t.frontier()["n_frontier"].copy()
            if nf.sum() == 0:
                break
            t.expand_layer(logits[l])
            c = t.candidates()
            for b in range(B):
                kept = c["kept"][b, :c["n_cand"][b]] == 1
                z = c["z"][b, :c["n_cand"][b]]
                assert kept.sum() <= F
                assert np.all(z[kept] > zb)                      # first pruning is strict
                if kept.sum() < min(F, (z > zb).sum()):          # fewer kept only because of the budget
                    assert t.finalize()["n_nodes"][b] == N
                if kept.any() and (~kept & (z > zb)).any():      # second pruning keeps the best z
                    assert z[kept].min() >= z[~kept & (z > zb)].max()
                assert c["n_cand"][b] == nf[b] * K
        out = t.finalize()
        for b in range(B):
            n = out["n_nodes"][b]
            assert n <= N
            par, dep = out["parent"][b, :n], out["position"][b, :n] - 1
            assert np.all(par < np.arange(n))                    # BFS order: parents come first
            assert np.all(np.diff(dep) >= 0)
            m = out["mask"][b]
            assert not m[n:].any() and not m[:, n:].any()
            for i in range(n):
                row = np.zeros(N, np.uint8); row[i] = 1
                if par[i] >= 0:
                    row |= m[par[i]]                             # mask[i] = mask[parent] + {i}
                    assert dep[i] == dep[par[i]] + 1
                    # Eq. 1 as a running product, one fp32 multiply per edge
                    assert out["joint_prob"][b, i] == f32(out["joint_prob"][b, par[i]] * out["p"][b, i])
                else:
                    assert dep[i] == 0 and out["joint_prob"][b, i] == out["p"][b, i]
                np.testing.assert_array_equal(m[i], row)
                assert m[i].sum() == dep[i] + 1
                assert abs(out["conf"][b, i] - 1 / (1 + math.exp(-float(out["z"][b, i])))) < 1e-6
            assert np.array_equal(np.tril(m), m)                 # ancestors have smaller indices
            if 0 < n < N:
                found = True
    assert found, "no classifier seed produced a non-trivial tree"


# ---------------- equal confidences: the second pruning's tie order ----------------
@pytest.mark.parametrize("equal_rows", [False, True])
def test_equal_confidences_are_ranked_by_token_then_slot(equal_rows):
    # Sec. 4.2.2 ranks by confidence only; with every confidence equal (zero weights) the order is this build's
    # tie rule alone: token id ascending, then frontier slot ascending.  Expected trees from plain python sorts.
    rng = np.random.default_rng(77)
    V, F, K, D, N, h = 40, 4, 5, 3, 11, 2
    logits = random_logits(rng, D, F, V, scale=2.0)
    if equal_rows:
        logits[:, :, 1:, :] = logits[:, :, :1, :]            # the same K tokens under every parent
    t = RefTree(1, V, F, K, D, N, h, 0, 0.5)
    t.set_classifier(np.zeros((h, 3), f32), np.zeros(h, f32), np.zeros(h, f32), 1.0)
    out = run(t, logits)
    tokens, parents, frontier = [], [], [-1]
    for l in range(D):
        cand = []
        for slot, par in enumerate(frontier):
            x = logits[l][0][slot]
            top = sorted(range(V), key=lambda j: (-float(x[j]), j))[:K]
            cand += [(tok, slot, par) for tok in top]
        keep = sorted(cand, key=lambda c: (c[0], c[1]))[:min(F, N - len(tokens))]
        frontier = []
        for tok, slot, par in keep:
            frontier.append(len(tokens)); tokens.append(tok); parents.append(par)
        if not frontier:
            break
    n = out["n_nodes"][0]
    assert n == len(tokens) == N
    np.testing.assert_array_equal(out["tokens"][0, :n], tokens)
    np.testing.assert_array_equal(out["parent"][0, :n], parents)
    if equal_rows:                                           # layer 1: the lowest token id, from slots 0, 1, 2, 3
        assert tokens[4] == tokens[5] == tokens[6] == tokens[7] and parents[4:8] == [0, 1, 2, 3]


# ---------------- brute force on tiny inputs ----------------
@pytest.mark.parametrize("case", range(12))
def test_against_second_implementation_tiny(case):
    rng = np.random.default_rng(4000 + case)
    V = int(rng.integers(3, 17))
    F, K = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    K = min(K, V)
    D = int(rng.integers(1, 4))
    N = int(rng.integers(1, 10))
    h = int(rng.integers(1, 5))
    beta = float(rng.choice([0.0, 0.3, 0.5, 0.6]))
    bf16 = bool(case % 2)
    logits = random_logits(rng, D, F, V, scale=1.5, bf16=bf16)
    if case % 3 == 0:                       # force exact ties
        logits[:, :, :, 1::2] = logits[:, :, :, 0:1] if V > 1 else logits[:, :, :, :1]
    cls = ((0.7 * rng.standard_normal((h, 3))).astype(f32), (0.5 * rng.standard_normal(h)).astype(f32),
           (0.9 * rng.standard_normal(h)).astype(f32), float(0.5 * rng.standard_normal() + 0.5))
    t = RefTree(1, V, F, K, D, N, h, 1 if bf16 else 0, beta)
    t.set_classifier(*cls)
    out = run(t, logits)
    nodes = second.build_tree([logits[l][0] for l in range(D)], F, K, D, N, cls, beta)
    n = out["n_nodes"][0]
    assert n == len(nodes)
    np.testing.assert_array_equal(out["tokens"][0, :n], [c["token"] for c in nodes])
    np.testing.assert_array_equal(out["parent"][0, :n], [c["parent"] for c in nodes])
    np.testing.assert_array_equal(out["position"][0, :n], [c["depth"] + 1 for c in nodes])
    np.testing.assert_allclose(out["joint_prob"][0, :n], [c["P"] for c in nodes], rtol=2e-7)
    np.testing.assert_allclose(out["entropy"][0, :n], [c["H"] for c in nodes], rtol=2e-7, atol=1e-7)
    np.testing.assert_array_equal(out["mask"][0], second.mask_of(nodes, N))
