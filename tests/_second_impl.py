"""A second, differently structured statement of the C2T layer loop, used only to pin
the oracle on tiny inputs: scipy's softmax / entropy library routines, Python's sort on
tuple keys, and an ancestor walk by recursion.  Small sizes only (pure Python).
"""
import numpy as np
from scipy.special import softmax
from scipy.stats import entropy

f32 = np.float32


def widen(row):
    """float32 stays; uint16 bf16 bit patterns -> float32 (exact)."""
    row = np.asarray(row)
    if row.dtype == np.uint16:
        return (row.astype(np.uint32) << 16).view(np.float32)
    return row.astype(np.float32)


def fma32(a, b, c):
    # a*b is exact in float64 (24+24 bits); one rounding to 53 bits, then to 24
    return f32(np.float64(a) * np.float64(b) + np.float64(c))


def mlp_logit(W1, b1, w2, b2, P, H, d):
    z = f32(b2)
    for j in range(len(b1)):
        a = fma32(W1[j][0], P, b1[j])
        a = fma32(W1[j][1], H, a)
        a = fma32(W1[j][2], d, a)
        a = a if a > 0 else f32(0)
        z = fma32(w2[j], a, z)
    return z


def logit_of_beta(beta):
    return f32(-np.inf) if beta <= 0 else f32(np.log(np.float64(beta) / (1.0 - np.float64(beta))))


def build_tree(logits_per_layer, F, K, D, N, cls, beta):
    """logits_per_layer[l]: array [F][V] for ONE sequence.  Returns list of nodes (dicts)."""
    W1, b1, w2, b2 = cls
    zb = logit_of_beta(beta)
    nodes = []
    frontier = [None]               # None = root
    for layer in range(D):
        if not frontier:
            break
        cands = []
        for slot, parent in enumerate(frontier):
            x = widen(logits_per_layer[layer][slot]).astype(np.float64)
            p = softmax(x)
            H = f32(entropy(p))                    # natural log
            order = sorted(range(len(x)), key=lambda j: (-x[j], j))[:K]
            Pp = f32(1.0) if parent is None else nodes[parent]["P"]
            for tok in order:
                p32 = f32(p[tok])
                P = f32(Pp * p32)
                z = mlp_logit(W1, b1, w2, b2, P, H, f32(layer))
                cands.append(dict(token=tok, slot=slot, parent=-1 if parent is None else parent,
                                  p=p32, P=P, H=H, z=z, depth=layer))
        surv = [c for c in cands if c["z"] > zb]
        surv.sort(key=lambda c: (-float(c["z"]), c["token"], c["slot"]))
        keep = surv[:max(0, min(F, N - len(nodes)))]
        frontier = []
        for c in keep:
            frontier.append(len(nodes))
            nodes.append(c)
    return nodes


def ancestors(nodes, i):
    return {i} if nodes[i]["parent"] < 0 else {i} | ancestors(nodes, nodes[i]["parent"])


def mask_of(nodes, N):
    m = np.zeros((N, N), np.uint8)
    for i in range(len(nodes)):
        for j in ancestors(nodes, i):
            m[i, j] = 1
    return m
