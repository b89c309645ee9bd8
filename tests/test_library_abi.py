"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host-side argument / state checks answer without touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2502_13652_amd import load_library
    return load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "c2t.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(c2t_[a-z_]+)\s*\(", text)))


def test_exports_every_declared_symbol(lib):
    syms = declared_symbols()
    assert "c2t_expand_layer" in syms and "c2t_finalize_tree" in syms and len(syms) >= 14
    for s in syms:
        assert hasattr(lib, s), s


def cfg(**kw):
    from paper_2502_13652_amd import C2TConfig
    base = dict(batch=2, vocab=1000, max_frontier=4, top_k=4, max_depth=3, budget=10, hidden=8, logits_dtype=1,
                beta=0.5, entropy_top_m=0, rerank=0)
    base.update(kw)
    return C2TConfig(**base)


def test_config_validation(lib):
    need = ctypes.c_size_t()
    assert lib.c2t_workspace_bytes(ctypes.byref(cfg()), ctypes.byref(need)) == 0 and need.value > 0
    assert lib.c2t_workspace_bytes(ctypes.byref(cfg()), None) == -1
    for bad in (dict(batch=0), dict(vocab=0), dict(top_k=0), dict(beta=1.0), dict(beta=-0.1), dict(logits_dtype=7),
                dict(top_k=5, vocab=4), dict(budget=0), dict(hidden=0)):
        assert lib.c2t_workspace_bytes(ctypes.byref(cfg(**bad)), ctypes.byref(need)) == -1, bad
    for big in (dict(top_k=65, max_frontier=1), dict(max_frontier=65, top_k=1), dict(hidden=257), dict(budget=1025),
                dict(max_frontier=64, top_k=64)):
        assert lib.c2t_workspace_bytes(ctypes.byref(cfg(**big)), ctypes.byref(need)) == -2, big
    assert lib.c2t_workspace_bytes(ctypes.byref(cfg(entropy_top_m=1000)), ctypes.byref(need)) == 0
    # rows long enough to be split over workgroups may also take the entropy over the M largest logits
    assert lib.c2t_workspace_bytes(ctypes.byref(cfg(entropy_top_m=1000, vocab=1 << 22)), ctypes.byref(need)) == 0
    assert lib.c2t_workspace_bytes(ctypes.byref(cfg(entropy_top_m=1000, vocab=152064, logits_dtype=0)), ctypes.byref(need)) == 0
    assert lib.c2t_workspace_bytes(ctypes.byref(cfg(entropy_top_m=-1)), ctypes.byref(need)) == -1
    # reranking keeps every scored candidate: more workspace, bounded history
    plain = ctypes.c_size_t(); lib.c2t_workspace_bytes(ctypes.byref(cfg()), ctypes.byref(plain))
    assert lib.c2t_workspace_bytes(ctypes.byref(cfg(rerank=1)), ctypes.byref(need)) == 0 and need.value > plain.value
    assert lib.c2t_workspace_bytes(ctypes.byref(cfg(rerank=2)), ctypes.byref(need)) == -1
    assert lib.c2t_workspace_bytes(ctypes.byref(cfg(rerank=1, max_depth=64, max_frontier=32, top_k=32)), ctypes.byref(need)) == -2


def test_workspace_and_state_errors(lib):
    c = cfg()
    need = ctypes.c_size_t()
    lib.c2t_workspace_bytes(ctypes.byref(c), ctypes.byref(need))
    ctx = ctypes.c_void_p()
    assert lib.c2t_create(ctypes.byref(c), None, need.value, ctypes.byref(ctx)) == -3
    assert lib.c2t_create(ctypes.byref(c), ctypes.c_void_p(0x1001), need.value, ctypes.byref(ctx)) == -3      # misaligned
    assert lib.c2t_create(ctypes.byref(c), ctypes.c_void_p(0x10000), need.value - 1, ctypes.byref(ctx)) == -3  # too small
    # a context over a fake (never dereferenced) workspace address: host-side checks only
    assert lib.c2t_create(ctypes.byref(c), ctypes.c_void_p(0x10000), need.value, ctypes.byref(ctx)) == 0
    assert lib.c2t_reset(ctx, None) == -4                       # classifier not set
    assert lib.c2t_expand_layer(ctx, ctypes.c_void_p(0x20000), 1000, None) == -4   # before reset
    assert lib.c2t_expand_layer(ctx, None, 1000, None) == -1
    assert lib.c2t_finalize_tree(ctx, None, None) == -1
    assert lib.c2t_set_row_splits(ctx, -1, 0) == -1
    assert lib.c2t_set_row_splits(ctx, 1 << 20, 0) in (-2, -3)
    assert lib.c2t_set_row_splits(ctx, 2, 3) == 0
    p = ctypes.c_void_p()
    assert lib.c2t_get_frontier(ctx, ctypes.byref(p), None, None) == 0 and p.value
    assert lib.c2t_get_layer_rows(ctx, None) == -1
    assert lib.c2t_profile_sample(ctx, 0, 0) == -1 and lib.c2t_profile_sample(ctx, 4, 4) == -1
    assert lib.c2t_profile_sample(ctx, 4, 2) == 0 and lib.c2t_profile_sample(None, 1, 0) == -1
    # the allocation-free reranking: argument and state checks come before anything touches the device
    from paper_2502_13652_amd.binding import _TreeOut
    outs = ctypes.byref(_TreeOut(*[0x30000] * 9))
    assert lib.c2t_finalize_tree_reranked_static(ctx, None, 4, None) == -1
    assert lib.c2t_finalize_tree_reranked_static(ctx, outs, 0, None) == -1
    assert lib.c2t_finalize_tree_reranked_static(ctx, outs, 1025, None) == -2
    assert lib.c2t_finalize_tree_reranked_static(ctx, outs, 4, None) == -4    # not a rerank context, nothing expanded
    # the phase-time read-out exists only in the profiling build of the library
    buf = (ctypes.c_uint64 * 16)()
    assert lib.c2t_phase_times_read(buf, 1) == -2
    lib.c2t_destroy(ctx)
    lib.c2t_destroy(None)
    assert lib.c2t_strerror(0) == b"ok" and b"workspace" in lib.c2t_strerror(-3) and b"memory" in lib.c2t_strerror(-6)


def test_rows_shared_by_workgroups_launch_shape(lib):
    """Host logic only (no device: 256 CUs assumed): which launches let several workgroups count one row."""
    def per_row(c, splits=None):
        need = ctypes.c_size_t()
        assert lib.c2t_workspace_bytes(ctypes.byref(c), ctypes.byref(need)) == 0
        ctx = ctypes.c_void_p()
        assert lib.c2t_create(ctypes.byref(c), ctypes.c_void_p(0x10000), need.value, ctypes.byref(ctx)) == 0
        if splits:
            assert lib.c2t_set_row_splits(ctx, *splits) == 0
        a, b = ctypes.c_int32(-1), ctypes.c_int32(-1)
        assert lib.c2t_get_row_workgroups(ctx, ctypes.byref(a), ctypes.byref(b)) == 0
        assert lib.c2t_get_row_workgroups(ctx, None, None) == 0 and lib.c2t_get_row_workgroups(None, None, None) == -1
        lib.c2t_destroy(ctx)
        return a.value, b.value
    one_seq = dict(batch=1, vocab=152064, max_frontier=16, top_k=16, max_depth=8, budget=96, hidden=32)
    assert per_row(cfg(**one_seq)) == (5, 5)                      # ten groups of 32 KB: five workgroups with two each
    assert per_row(cfg(**one_seq), (1, 0)) == (1, 5) and per_row(cfg(**one_seq), (0, 2)) == (5, 2)   # a count that is set is taken literally
    assert per_row(cfg(**dict(one_seq, batch=64, vocab=128256))) == (4, 1)    # 64 root rows on 256 CUs; 1024 rows are not shared
    assert per_row(cfg(**dict(one_seq, batch=128, vocab=128256))) == (2, 1)
    assert per_row(cfg(**dict(one_seq, batch=129, vocab=128256))) == (1, 1)
    assert per_row(cfg(**dict(one_seq, vocab=49152))) == (1, 1)   # under four groups: the hand-over costs more than it saves
    assert per_row(cfg(**dict(one_seq, vocab=49160))) == (4, 4)   # 6145 chunks, four groups: the last workgroup gets the last chunk alone
    assert per_row(cfg(**dict(one_seq, vocab=65544))) == (5, 5)   # 8193 chunks: five groups, one each
    assert per_row(cfg(**dict(one_seq, vocab=32000, logits_dtype=0))) == (4, 4)   # fp32 rows are split, not shared


def test_no_cpu_fallback_and_no_oracle_in_the_product():
    """Without a GPU the binding raises instead of computing anything on the host, and nothing
    under the package imports, links or names the oracle."""
    import torch
    from paper_2502_13652_amd import C2TContext
    if not torch.cuda.is_available():
        with pytest.raises(RuntimeError, match="no CPU fallback"):
            C2TContext(1, 100, 2, 2, 2, 4, 4, 1, 0.5)
    pkg = os.path.join(ROOT, "paper_2502_13652_amd")
    for base, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(base, f)).read()
                assert "oracle" not in text.lower(), os.path.join(base, f)
