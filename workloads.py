"""Seeded synthetic workloads for the C2T tree-construction path.

Holds no arithmetic of the method itself: only input generation, shared by the
oracle-side and the HIP-side tests and by bench.py.  The inputs stand in for the
paper's workloads (EAGLE draft heads over LLaMA-2 / Vicuna vocabularies on
MT-bench etc.), whose models and data are not available: each logits row is
Gaussian noise of a per-row scale on top of a Zipf-shaped bias over a
per-sequence random permutation of the token ids, which gives rows whose
entropy ranges from near one-hot to several nats, like a draft model's.

Row (b, layer, f):  x_t = sigma * g_t + bias_t,  g_t ~ N(0,1) iid,
sigma ~ U[sigma_lo, sigma_hi] per row,  bias_t = -s * ln(rank_pi_b(t)),
pi_b a seeded permutation per sequence; optionally a fraction of rows gets +20
on one random token (near one-hot rows).  fp32 is rounded to bf16 (nearest
even) for the bf16 configs.  The "draft model" is thereby replaced by rows that
depend only on (config, sequence, layer, slot), not on the tokens chosen.
"""
import json
import os

import numpy as np
import torch

BASE_SEED = 250213652

# B sequences, V vocabulary, D max depth, F max frontier, K children per node,
# h classifier hidden width, beta threshold, N node budget (root excluded)
CONFIGS = {
    "cfg1": dict(idx=1, B=1, V=32000, dtype="f32", D=6, F=10, K=10, h=12, beta=0.5, N=60,
                 zipf_s=1.1, sigma=(1.0, 6.0), spike_frac=0.0,
                 desc="tiny CPU-seconds case, fp32 logits"),
    "cfg2": dict(idx=2, B=1, V=32000, dtype="bf16", D=8, F=10, K=10, h=12, beta=0.5, N=60,
                 zipf_s=1.1, sigma=(1.0, 6.0), spike_frac=0.0,
                 desc="Llama-2-chat-sized draft step"),
    "cfg3": dict(idx=3, B=1, V=128256, dtype="bf16", D=8, F=16, K=16, h=32, beta=0.4, N=96,
                 zipf_s=1.05, sigma=(1.0, 6.0), spike_frac=0.0,
                 desc="Llama-3-sized vocabulary"),
    "cfg4": dict(idx=4, B=64, V=128256, dtype="bf16", D=6, F=16, K=16, h=32, beta=0.4, N=64,
                 zipf_s=1.05, sigma=(1.0, 6.0), spike_frac=0.0,
                 desc="batched serving, 64 sequences"),
    "cfg5": dict(idx=5, B=256, V=152064, dtype="bf16", D=10, F=32, K=32, h=64, beta=0.3, N=128,
                 zipf_s=1.0, sigma=(0.5, 8.0), spike_frac=0.05,
                 desc="large-vocabulary stress case, 256 sequences"),
    # Sec. 5.5 (chain mode): one child per node, so the tree is a chain and the classifier is an
    # early-exit rule; many sequences, ragged lengths.  Not one of the five benchmark configurations.
    "chain": dict(idx=6, B=1024, V=32000, dtype="bf16", D=8, F=1, K=1, h=12, beta=0.5, N=8,
                  zipf_s=1.1, sigma=(1.0, 6.0), spike_frac=0.0,
                  desc="batched chain mode, 1024 sequences, one child per node"),
}


def _mix(*xs):
    """splitmix64-style hash of a tuple of small integers -> 63-bit seed."""
    h = 0x9E3779B97F4A7C15
    for x in xs:
        h = (h ^ (int(x) & 0xFFFFFFFFFFFFFFFF)) & 0xFFFFFFFFFFFFFFFF
        h = (h * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        h ^= h >> 31
        h = (h * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
        h ^= h >> 29
    return h & 0x7FFFFFFFFFFFFFFF


def torch_dtype(cfg):
    return torch.float32 if cfg["dtype"] == "f32" else torch.bfloat16


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def sequence_bias(cfg, b, device="cpu", instance=0):
    """Zipf-shaped bias over a per-sequence permutation of the token ids, fp32 [V]."""
    V = cfg["V"]
    g = _gen(device, _mix(BASE_SEED, cfg["idx"], instance, b, 0xB1A5))
    perm = torch.randperm(V, generator=g, device=device)
    return -cfg["zipf_s"] * torch.log((perm + 1).to(torch.float32))


def logits_layer(cfg, layer, device="cpu", seqs=None, instance=0, rows=None):
    """Logits for every frontier slot of `layer`: tensor [len(seqs)][rows][V] in the config's dtype.

    seqs: which sequences (default all B); rows: slots per sequence (default F).
    Row contents depend only on (config, instance, sequence, layer, slot).
    """
    B, V, F = cfg["B"], cfg["V"], cfg["F"]
    seqs = list(range(B)) if seqs is None else list(seqs)
    rows = F if rows is None else rows
    out = torch.empty((len(seqs), rows, V), dtype=torch_dtype(cfg), device=device)
    lo, hi = cfg["sigma"]
    for i, b in enumerate(seqs):
        bias = sequence_bias(cfg, b, device, instance)
        g = _gen(device, _mix(BASE_SEED, cfg["idx"], instance, b, layer + 1))
        sigma = lo + (hi - lo) * torch.rand((F, 1), generator=g, device=device)
        x = torch.randn((F, V), generator=g, device=device) * sigma + bias
        if cfg["spike_frac"] > 0:
            u = torch.rand((F,), generator=g, device=device)
            tok = torch.randint(0, V, (F,), generator=g, device=device)
            sel = torch.nonzero(u < cfg["spike_frac"]).flatten()
            x[sel, tok[sel]] += 20.0
        out[i] = x[:rows].to(out.dtype)
    return out


def as_numpy_bits(t):
    """torch logits (fp32 or bf16, CPU) -> numpy array the oracle binding accepts."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def classifier(cfg, seed):
    """3 -> h -> 1 MLP parameters, all drawn N(0, 0.5) in fp32: W1[h][3] (P,H,d), b1[h], w2[h], b2."""
    h = cfg["h"]
    rng = np.random.Generator(np.random.Philox(key=_mix(BASE_SEED, cfg["idx"], 0xC1A5, seed)))
    W1 = (0.5 * rng.standard_normal((h, 3))).astype(np.float32)
    b1 = (0.5 * rng.standard_normal(h)).astype(np.float32)
    w2 = (0.5 * rng.standard_normal(h)).astype(np.float32)
    b2 = np.float32(0.5 * rng.standard_normal())
    return W1, b1, w2, float(b2)


_SEEDS_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tests", "golden", "classifier_seeds.json")


def classifier_seed(name):
    """Seed chosen for a config by the rule in tests/golden/make_classifier_seeds.py
    (an oracle-only script); a random 3->h->1 MLP can be degenerate (keeps all or nothing)."""
    with open(_SEEDS_FILE) as f:
        return int(json.load(f)[name]["seed"])
