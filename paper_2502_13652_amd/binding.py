"""ctypes binding of libc2t_hip.so.  Argument marshalling only: names and order follow
include/c2t.h.  There is no CPU fallback: a missing library or device is an error."""
import ctypes
import os
import subprocess

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_SRC_DIR = os.path.join(_HERE, "csrc")
_LIB_DIR = os.path.join(_HERE, "lib")
_LIB = os.path.join(_LIB_DIR, "libc2t_hip.so")
_lib = None

F32, BF16 = 0, 1
_ERR = {-1: "invalid argument", -2: "unsupported", -3: "workspace", -4: "state", -5: "hip", -6: "out of host memory"}

HIPCC_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


class C2TError(RuntimeError):
    def __init__(self, code, what):
        super().__init__("%s failed: %d (%s)" % (what, code, _ERR.get(code, "?")))
        self.code = code


class C2TConfig(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("vocab", ctypes.c_int32), ("max_frontier", ctypes.c_int32),
                ("top_k", ctypes.c_int32), ("max_depth", ctypes.c_int32), ("budget", ctypes.c_int32),
                ("hidden", ctypes.c_int32), ("logits_dtype", ctypes.c_int32), ("beta", ctypes.c_float),
                ("entropy_top_m", ctypes.c_int32), ("rerank", ctypes.c_int32)]


class _TreeOut(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("tokens", "parent", "position", "conf", "joint_prob", "entropy", "n_nodes", "mask", "status")]


def lib_path():
    return _LIB


def build(verbose=False):
    """Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
    os.makedirs(_LIB_DIR, exist_ok=True)
    cmd = ["hipcc"] + HIPCC_FLAGS + ["-I", os.path.join(_ROOT, "include"), "-o", _LIB,
                                      os.path.join(_SRC_DIR, "c2t_lib.hip")]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if verbose or r.returncode:
        print(r.stdout)
    if r.returncode:
        raise RuntimeError("hipcc failed")
    return _LIB


def load_library(path=None):
    """Load the built library (once per process).  `path`: another build of it, e.g. the profiling build of
    phase_times.py; only honoured by the first call."""
    global _lib
    if _lib is not None:
        return _lib
    if path is None and not os.path.exists(_LIB):
        build()
    L = ctypes.CDLL(path or _LIB)
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    P = ctypes.POINTER
    L.c2t_workspace_bytes.argtypes = [P(C2TConfig), P(sz)]
    L.c2t_create.argtypes = [P(C2TConfig), vp, sz, P(vp)]
    L.c2t_destroy.argtypes = [vp]
    L.c2t_destroy.restype = None
    L.c2t_set_classifier.argtypes = [vp, vp, vp, vp, f32, vp]
    L.c2t_reset.argtypes = [vp, vp]
    L.c2t_expand_layer.argtypes = [vp, vp, i64, vp]
    L.c2t_get_frontier.argtypes = [vp, P(vp), P(vp), P(vp)]
    L.c2t_get_candidates.argtypes = [vp] + [P(vp)] * 7
    L.c2t_finalize_tree.argtypes = [vp, P(_TreeOut), vp]
    L.c2t_finalize_tree_reranked.argtypes = [vp, P(_TreeOut), i32, vp]
    L.c2t_finalize_tree_reranked_static.argtypes = [vp, P(_TreeOut), i32, vp]
    L.c2t_get_layer_rows.argtypes = [vp, P(vp)]
    L.c2t_set_row_splits.argtypes = [vp, i32, i32]
    L.c2t_get_row_workgroups.argtypes = [vp, P(i32), P(i32)]
    L.c2t_profile_enable.argtypes = [vp, i32]
    L.c2t_profile_read.argtypes = [vp, vp, P(i32)]
    L.c2t_profile_sample.argtypes = [vp, i32, i32]
    L.c2t_stream_read.argtypes = [vp, sz, vp, vp]
    L.c2t_stream_read_rows.argtypes = [vp, i32, sz, sz, vp, vp]
    L.c2t_phase_times_read.argtypes = [vp, i32]
    L.c2t_strerror.argtypes = [ctypes.c_int]
    L.c2t_strerror.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(rc, what):
    if rc != 0:
        raise C2TError(rc, what)


def _stream_ptr(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _view(ptr, shape, dtype, device, keep):
    """Wrap a device pointer that lives in the workspace tensor `keep` as a torch tensor."""
    n = 1
    for d in shape:
        n *= d
    off = ptr - keep.data_ptr()
    nbytes = n * torch.empty((), dtype=dtype).element_size()
    return keep[off:off + nbytes].view(dtype).view(*shape)


class C2TContext:
    """reset -> expand_layer x D -> finalize_tree on device memory (see include/c2t.h)."""

    def __init__(self, batch, vocab, max_frontier, top_k, max_depth, budget, hidden, dtype, beta,
                 entropy_top_m=0, rerank=0, device="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("the C2T HIP path needs a GPU; there is no CPU fallback")
        self.L = load_library()
        self.device = torch.device(device)
        self.cfg = C2TConfig(batch, vocab, max_frontier, top_k, max_depth, budget, hidden,
                             BF16 if dtype in (BF16, torch.bfloat16, "bf16") else F32, beta, entropy_top_m, int(rerank))
        self.B, self.V, self.F, self.K, self.D, self.N, self.h = batch, vocab, max_frontier, top_k, max_depth, budget, hidden
        need = ctypes.c_size_t()
        _check(self.L.c2t_workspace_bytes(ctypes.byref(self.cfg), ctypes.byref(need)), "c2t_workspace_bytes")
        self.workspace = torch.zeros(need.value + 256, dtype=torch.uint8, device=self.device)
        pad = (-self.workspace.data_ptr()) % 256
        self._ws = self.workspace[pad:pad + need.value]
        self.ctx = ctypes.c_void_p()
        _check(self.L.c2t_create(ctypes.byref(self.cfg), ctypes.c_void_p(self._ws.data_ptr()), need.value,
                                 ctypes.byref(self.ctx)), "c2t_create")

    def close(self):
        if getattr(self, "ctx", None):
            self.L.c2t_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_classifier(self, W1, b1, w2, b2, stream=None):
        import numpy as np
        W1 = np.ascontiguousarray(W1, np.float32).reshape(self.h, 3)
        b1 = np.ascontiguousarray(b1, np.float32).reshape(self.h)
        w2 = np.ascontiguousarray(w2, np.float32).reshape(self.h)
        _check(self.L.c2t_set_classifier(self.ctx, W1.ctypes.data, b1.ctypes.data, w2.ctypes.data, float(b2),
                                         _stream_ptr(stream)), "c2t_set_classifier")

    def reset(self, stream=None):
        _check(self.L.c2t_reset(self.ctx, _stream_ptr(stream)), "c2t_reset")

    def expand_layer(self, logits, stream=None):
        """logits: device tensor [B][F][stride >= V] of the configured dtype (last dim contiguous)."""
        assert logits.is_cuda and logits.dim() == 3 and logits.stride(2) == 1
        assert logits.shape[0] == self.B and logits.shape[1] == self.F and logits.stride(0) == self.F * logits.stride(1)
        assert logits.dtype == (torch.bfloat16 if self.cfg.logits_dtype == BF16 else torch.float32)
        _check(self.L.c2t_expand_layer(self.ctx, ctypes.c_void_p(logits.data_ptr()), logits.stride(1),
                                       _stream_ptr(stream)), "c2t_expand_layer")

    def frontier(self):
        t, s, n = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
        _check(self.L.c2t_get_frontier(self.ctx, ctypes.byref(t), ctypes.byref(s), ctypes.byref(n)), "c2t_get_frontier")
        return dict(tokens=_view(t.value, (self.B, self.F), torch.int32, self.device, self._ws),
                    parent_slot=_view(s.value, (self.B, self.F), torch.int32, self.device, self._ws),
                    n_frontier=_view(n.value, (self.B,), torch.int32, self.device, self._ws))

    def candidates(self):
        ps = [ctypes.c_void_p() for _ in range(7)]
        _check(self.L.c2t_get_candidates(self.ctx, *[ctypes.byref(p) for p in ps]), "c2t_get_candidates")
        FK = self.F * self.K
        names = ("n_cand", "token", "p", "P", "H", "z", "kept")
        dts = (torch.int32, torch.int32, torch.float32, torch.float32, torch.float32, torch.float32, torch.int32)
        out = {}
        for nm, p, dt in zip(names, ps, dts):
            shape = (self.B,) if nm == "n_cand" else (self.B, FK)
            out[nm] = _view(p.value, shape, dt, self.device, self._ws)
        return out

    def new_tree_out(self, N=None):
        B, N, dev = self.B, (self.N if N is None else int(N)), self.device
        i32 = dict(dtype=torch.int32, device=dev)
        f32 = dict(dtype=torch.float32, device=dev)
        return dict(tokens=torch.empty((B, N), **i32), parent=torch.empty((B, N), **i32),
                    position=torch.empty((B, N), **i32), conf=torch.empty((B, N), **f32),
                    joint_prob=torch.empty((B, N), **f32), entropy=torch.empty((B, N), **f32),
                    n_nodes=torch.empty((B,), **i32), mask=torch.empty((B, N, N), dtype=torch.uint8, device=dev),
                    status=torch.empty((B,), **i32).view(torch.uint32))        # a bit field: uint32 as in the header

    def finalize_tree(self, out=None, stream=None):
        out = self.new_tree_out() if out is None else out
        o = _TreeOut(*[out[k].data_ptr() for k in
                       ("tokens", "parent", "position", "conf", "joint_prob", "entropy", "n_nodes", "mask", "status")])
        _check(self.L.c2t_finalize_tree(self.ctx, ctypes.byref(o), _stream_ptr(stream)), "c2t_finalize_tree")
        return out

    def finalize_tree_reranked(self, n_out, out=None, stream=None):
        out = self.new_tree_out(n_out) if out is None else out
        o = _TreeOut(*[out[k].data_ptr() for k in
                       ("tokens", "parent", "position", "conf", "joint_prob", "entropy", "n_nodes", "mask", "status")])
        _check(self.L.c2t_finalize_tree_reranked(self.ctx, ctypes.byref(o), int(n_out), _stream_ptr(stream)),
               "c2t_finalize_tree_reranked")
        return out

    def finalize_tree_reranked_static(self, n_out, out=None, stream=None):
        """The same reranking with the kernel's scratch in the library's static device array (no allocation)."""
        out = self.new_tree_out(n_out) if out is None else out
        o = _TreeOut(*[out[k].data_ptr() for k in
                       ("tokens", "parent", "position", "conf", "joint_prob", "entropy", "n_nodes", "mask", "status")])
        _check(self.L.c2t_finalize_tree_reranked_static(self.ctx, ctypes.byref(o), int(n_out), _stream_ptr(stream)),
               "c2t_finalize_tree_reranked_static")
        return out

    def layer_rows(self):
        p = ctypes.c_void_p()
        _check(self.L.c2t_get_layer_rows(self.ctx, ctypes.byref(p)), "c2t_get_layer_rows")
        return _view(p.value, (self.D + 1,), torch.int32, self.device, self._ws)

    def set_row_splits(self, first_layer=0, other_layers=0):
        _check(self.L.c2t_set_row_splits(self.ctx, first_layer, other_layers), "c2t_set_row_splits")

    def row_workgroups(self):
        """(first layer, later layers): workgroups per logits row as the context stands."""
        a, b = ctypes.c_int32(0), ctypes.c_int32(0)
        _check(self.L.c2t_get_row_workgroups(self.ctx, ctypes.byref(a), ctypes.byref(b)), "c2t_get_row_workgroups")
        return a.value, b.value

    def profile_enable(self, capacity):
        _check(self.L.c2t_profile_enable(self.ctx, capacity), "c2t_profile_enable")

    def profile_sample(self, every, first=0):
        """Attach the timing events only to the launches of draft phases first, first + every, ..."""
        _check(self.L.c2t_profile_sample(self.ctx, every, first), "c2t_profile_sample")

    def profile_read(self, capacity):
        buf = (ctypes.c_float * capacity)()
        n = ctypes.c_int32(capacity)
        _check(self.L.c2t_profile_read(self.ctx, buf, ctypes.byref(n)), "c2t_profile_read")
        return list(buf[:n.value])


def stream_read(tensor, out, stream=None):
    """Plain streaming read of a device tensor (the practical HBM ceiling)."""
    L = load_library()
    nbytes = tensor.numel() * tensor.element_size()
    _check(L.c2t_stream_read(ctypes.c_void_p(tensor.data_ptr()), nbytes - nbytes % 16,
                             ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream)), "c2t_stream_read")


def stream_read_rows(tensor, rows, row_bytes, out, stream=None):
    """Plain read of `rows` rows of `row_bytes` each (contiguous in `tensor`) with the logits pass's access pattern."""
    L = load_library()
    _check(L.c2t_stream_read_rows(ctypes.c_void_p(tensor.data_ptr()), int(rows), int(row_bytes), int(row_bytes),
                                  ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream)), "c2t_stream_read_rows")
