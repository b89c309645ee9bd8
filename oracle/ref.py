"""ctypes binding of the C++ oracle (oracle/c2t_oracle.cpp).  Test infrastructure only.

Arrays cross the boundary as numpy arrays; bf16 logits are passed as uint16 bit
patterns (numpy has no bf16 type).
"""
import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "c2t_oracle.cpp")
_LIB = os.path.join(_HERE, "libc2t_oracle.so")
_lib = None
_lock = threading.Lock()

F32, BF16 = 0, 1


def build_oracle(force=False):
    """Compile the oracle with the host compiler (plain -O2, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is not None:
            return _lib
        build_oracle()
        L = ctypes.CDLL(_LIB)
        vp, i32, i64, f32, f64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_double
        L.c2t_ref_row.argtypes = [vp, i32, i32, i32] + [vp] * 7
        L.c2t_ref_row.restype = i32
        L.c2t_ref_entropy_top_m.argtypes = [vp, i32, i32, i32]
        L.c2t_ref_entropy_top_m.restype = f64
        L.c2t_ref_mlp_logit.argtypes = [i32, vp, vp, vp, f32, f32, f32, f32]
        L.c2t_ref_mlp_logit.restype = f32
        L.c2t_ref_logit_of_beta.argtypes = [f32]
        L.c2t_ref_logit_of_beta.restype = f32
        L.c2t_ref_create.argtypes = [i32] * 8 + [f32]
        L.c2t_ref_create.restype = vp
        L.c2t_ref_destroy.argtypes = [vp]
        L.c2t_ref_set_entropy_top_m.argtypes = [vp, i32]
        L.c2t_ref_set_classifier.argtypes = [vp, vp, vp, vp, f32]
        L.c2t_ref_reset.argtypes = [vp]
        L.c2t_ref_expand_layer_range.argtypes = [vp, vp, i64, i32, i32]
        L.c2t_ref_expand_layer_range.restype = i32
        L.c2t_ref_end_layer.argtypes = [vp]
        L.c2t_ref_expand_layer.argtypes = [vp, vp, i64]
        L.c2t_ref_expand_layer.restype = i32
        L.c2t_ref_layer.argtypes = [vp]
        L.c2t_ref_layer.restype = i32
        L.c2t_ref_get_frontier.argtypes = [vp] * 4
        L.c2t_ref_get_candidates.argtypes = [vp] * 9
        L.c2t_ref_get_audit.argtypes = [vp] * 4
        L.c2t_ref_finalize.argtypes = [vp] * 10
        L.c2t_ref_finalize_rerank.argtypes = [vp, i32] + [vp] * 10
        L.c2t_ref_get_node_extras.argtypes = [vp] * 3
        _lib = L
        return L


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _row_array(row):
    """-> (contiguous numpy array, dtype code).  float32 stays; uint16 means bf16 bits."""
    row = np.ascontiguousarray(row)
    if row.dtype == np.float32:
        return row, F32
    if row.dtype == np.uint16:
        return row, BF16
    raise TypeError("logits must be float32 or uint16 (bf16 bit patterns), got %s" % row.dtype)


def ref_row(row, top_k):
    """One logits row -> dict(bad, m, Z, S, H, ids, logits, p)."""
    L = _load()
    row, dt = _row_array(row)
    V = row.shape[0]
    k = min(top_k, V)
    m, Z, S, H = (ctypes.c_double() for _ in range(4))
    ids = np.full(k, -1, np.int32)
    xs = np.zeros(k, np.float64)
    ps = np.zeros(k, np.float64)
    rc = L.c2t_ref_row(_ptr(row), dt, V, top_k, ctypes.byref(m), ctypes.byref(Z), ctypes.byref(S),
                       ctypes.byref(H), _ptr(ids), _ptr(xs), _ptr(ps))
    return dict(bad=bool(rc), m=m.value, Z=Z.value, S=S.value, H=H.value, ids=ids, logits=xs, p=ps)


def ref_entropy_top_m(row, M):
    L = _load()
    row, dt = _row_array(row)
    return L.c2t_ref_entropy_top_m(_ptr(row), dt, row.shape[0], M)


def ref_mlp_logit(W1, b1, w2, b2, P, H, d):
    L = _load()
    W1 = np.ascontiguousarray(W1, np.float32)
    b1 = np.ascontiguousarray(b1, np.float32)
    w2 = np.ascontiguousarray(w2, np.float32)
    return L.c2t_ref_mlp_logit(b1.shape[0], _ptr(W1), _ptr(b1), _ptr(w2), float(b2), float(P), float(H), float(d))


def ref_logit_of_beta(beta):
    return _load().c2t_ref_logit_of_beta(float(beta))


class RefTree:
    """reset -> expand_layer x D -> finalize on host memory."""

    def __init__(self, batch, vocab, max_frontier, top_k, max_depth, budget, hidden, dtype, beta):
        self.L = _load()
        self.B, self.V, self.F, self.K, self.D, self.N, self.h = batch, vocab, max_frontier, top_k, max_depth, budget, hidden
        self.dtype = dtype
        self.h_ = self.L.c2t_ref_create(batch, vocab, max_frontier, top_k, max_depth, budget, hidden, dtype, float(beta))
        if not self.h_:
            raise ValueError("invalid oracle configuration")

    def close(self):
        if self.h_:
            self.L.c2t_ref_destroy(self.h_)
            self.h_ = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_entropy_top_m(self, M):
        self.L.c2t_ref_set_entropy_top_m(self.h_, int(M))

    def set_classifier(self, W1, b1, w2, b2):
        W1 = np.ascontiguousarray(W1, np.float32).reshape(self.h, 3)
        b1 = np.ascontiguousarray(b1, np.float32).reshape(self.h)
        w2 = np.ascontiguousarray(w2, np.float32).reshape(self.h)
        self.L.c2t_ref_set_classifier(self.h_, _ptr(W1), _ptr(b1), _ptr(w2), float(b2))

    def reset(self):
        self.L.c2t_ref_reset(self.h_)

    def expand_layer(self, logits, threads=1):
        """logits: numpy [B][F][stride>=V], float32 or uint16 (bf16 bits)."""
        logits, dt = _row_array(logits)
        assert dt == self.dtype and logits.ndim == 3 and logits.shape[0] == self.B and logits.shape[1] == self.F
        stride = logits.shape[2]
        if threads <= 1 or self.B == 1:
            rc = self.L.c2t_ref_expand_layer(self.h_, _ptr(logits), stride)
            if rc:
                raise RuntimeError("oracle expand_layer refused (state or stride)")
            return
        # sequences are independent: shard them over threads (ctypes releases the GIL)
        bounds = np.linspace(0, self.B, min(threads, self.B) + 1).astype(int)
        rcs = []

        def work(b0, b1):
            rcs.append(self.L.c2t_ref_expand_layer_range(self.h_, _ptr(logits), stride, int(b0), int(b1)))

        ths = [threading.Thread(target=work, args=(bounds[i], bounds[i + 1])) for i in range(len(bounds) - 1)]
        for t in ths:
            t.start()
        for t in ths:
            t.join()
        if any(rcs):
            raise RuntimeError("oracle expand_layer refused (state or stride)")
        self.L.c2t_ref_end_layer(self.h_)

    @property
    def layer(self):
        return self.L.c2t_ref_layer(self.h_)

    def frontier(self):
        tok = np.zeros((self.B, self.F), np.int32)
        slot = np.zeros((self.B, self.F), np.int32)
        n = np.zeros(self.B, np.int32)
        self.L.c2t_ref_get_frontier(self.h_, _ptr(tok), _ptr(slot), _ptr(n))
        return dict(tokens=tok, parent_slot=slot, n_frontier=n)

    def candidates(self):
        FK = self.F * self.K
        n = np.zeros(self.B, np.int32)
        token = np.full((self.B, FK), -1, np.int32)
        slot = np.full((self.B, FK), -1, np.int32)
        kept = np.zeros((self.B, FK), np.int32)
        p, P, H, z = (np.zeros((self.B, FK), np.float32) for _ in range(4))
        self.L.c2t_ref_get_candidates(self.h_, _ptr(n), _ptr(token), _ptr(slot), _ptr(p), _ptr(P), _ptr(H), _ptr(z), _ptr(kept))
        return dict(n_cand=n, token=token, slot=slot, p=p, P=P, H=H, z=z, kept=kept)

    def audit(self):
        a = np.zeros(self.B, np.float64)
        g = np.zeros(self.B, np.float64)
        s = np.zeros(self.B, np.int64)
        self.L.c2t_ref_get_audit(self.h_, _ptr(a), _ptr(g), _ptr(s))
        return dict(min_thr_margin=a, min_rank_gap=g, scored=s)

    def finalize(self):
        B, N = self.B, self.N
        out = dict(tokens=np.zeros((B, N), np.int32), parent=np.zeros((B, N), np.int32),
                   position=np.zeros((B, N), np.int32), conf=np.zeros((B, N), np.float32),
                   joint_prob=np.zeros((B, N), np.float32), entropy=np.zeros((B, N), np.float32),
                   n_nodes=np.zeros(B, np.int32), mask=np.zeros((B, N, N), np.uint8),
                   status=np.zeros(B, np.uint32))
        self.L.c2t_ref_finalize(self.h_, *[_ptr(out[k]) for k in
                                           ("tokens", "parent", "position", "conf", "joint_prob", "entropy", "n_nodes", "mask", "status")])
        p = np.zeros((B, N), np.float32)
        z = np.zeros((B, N), np.float32)
        self.L.c2t_ref_get_node_extras(self.h_, _ptr(p), _ptr(z))
        out["p"] = p
        out["z"] = z
        return out

    def finalize_rerank(self, n_out):
        """Global top-n_out over every scored candidate by the path minimum of the classifier logit."""
        B, N = self.B, int(n_out)
        out = dict(tokens=np.zeros((B, N), np.int32), parent=np.zeros((B, N), np.int32),
                   position=np.zeros((B, N), np.int32), conf=np.zeros((B, N), np.float32),
                   joint_prob=np.zeros((B, N), np.float32), entropy=np.zeros((B, N), np.float32),
                   path_min_z=np.zeros((B, N), np.float32),
                   n_nodes=np.zeros(B, np.int32), mask=np.zeros((B, N, N), np.uint8),
                   status=np.zeros(B, np.uint32))
        self.L.c2t_ref_finalize_rerank(self.h_, N, *[_ptr(out[k]) for k in
                                       ("tokens", "parent", "position", "conf", "joint_prob", "entropy", "path_min_z",
                                        "n_nodes", "mask", "status")])
        return out
