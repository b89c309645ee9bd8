"""The allocation-free reranking entry point (its scratch in the library's static device array)
against the workspace-backed one: same outputs, bit for bit, on two calls in a row, the second on a
smaller input; and its size limit."""
import numpy as np
import pytest
import torch

import workloads as W
from _harness import make_gpu, to_np

pytestmark = pytest.mark.gpu


def _phase(cfg, cls, instance):
    g = make_gpu(cfg, cls)
    g.reset()
    for l in range(cfg["D"]):
        g.expand_layer(W.logits_layer(cfg, l, device="cuda", instance=instance))
    torch.cuda.synchronize()
    return g


def _same(a, b, tag):
    for k in a:
        if a[k].dtype.kind == "f":
            np.testing.assert_array_equal(a[k].view(np.uint32), b[k].view(np.uint32), err_msg="%s %s" % (tag, k))
        else:
            np.testing.assert_array_equal(a[k], b[k], err_msg="%s %s" % (tag, k))


def test_static_scratch_reranking_matches_the_workspace_one():
    big = dict(idx=96, B=24, V=4104, dtype="bf16", D=5, F=16, K=8, h=8, beta=0.3, N=60, rerank=1,
               zipf_s=1.0, sigma=(1.0, 4.0), spike_frac=0.0, desc="static scratch, first call")
    small = dict(big, B=5, D=3, F=4, K=4, N=10, desc="static scratch, second call on a smaller input")
    total = 0
    for cfg, n_outs in ((big, (60, 200)), (small, (10, 7)), (big, (33,))):
        for seed in range(40):                     # a classifier that does not prune everything at the root
            cls = W.classifier(cfg, seed)
            g = _phase(cfg, cls, 0)
            if int(to_np(g.finalize_tree())["n_nodes"].min()) >= 2:
                break
        for n_out in n_outs:
            print("static scratch:", cfg["desc"], "B", cfg["B"], "n_out", n_out, flush=True)
            want = to_np(g.finalize_tree_reranked(n_out))
            torch.cuda.synchronize()
            got = to_np(g.finalize_tree_reranked_static(n_out))
            torch.cuda.synchronize()
            _same(want, got, "%s n_out=%d" % (cfg["desc"], n_out))
            assert int(got["n_nodes"].sum()) > 0
            total += int(got["n_nodes"].sum())
    assert total > 0


def test_static_scratch_reranking_rejects_sizes_beyond_its_array():
    from paper_2502_13652_amd.binding import C2TError
    # batch * max_depth * max_frontier * top_k = 2^22 + 2^15 history entries: one step over the limit
    cfg = dict(idx=95, B=129, V=2048, dtype="bf16", D=16, F=64, K=32, h=4, beta=0.3, N=64, rerank=1)
    g = make_gpu(cfg, W.classifier(cfg, 0))
    g.reset()
    with pytest.raises(C2TError) as e:
        g.finalize_tree_reranked_static(16)
    assert e.value.code == -2                       # C2T_ERR_UNSUPPORTED
    plain = dict(cfg, B=2, rerank=0)
    g = make_gpu(plain, W.classifier(plain, 0))
    g.reset()
    with pytest.raises(C2TError) as e:
        g.finalize_tree_reranked_static(16)
    assert e.value.code == -4                       # C2T_ERR_STATE: the context keeps no history
