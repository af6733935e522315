"""Thin Python binding of the C-ABI library (include/vp.h): argument marshalling
only.  PyTorch supplies device memory and the current stream; every step of
the projection path runs in the library's HIP kernels.  There is no fallback:
if libvp.so is missing or fails to load, importing succeeds but the first use
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvp.so")

VP_OK, VP_ERR_INVALID_ARG, VP_ERR_UNSUPPORTED, VP_ERR_WORKSPACE, VP_ERR_HIP = range(5)
STATUS_NAMES = {0: "VP_OK", 1: "VP_ERR_INVALID_ARG", 2: "VP_ERR_UNSUPPORTED", 3: "VP_ERR_WORKSPACE",
                4: "VP_ERR_HIP"}

EXPORTS = ("vp_build_bytes", "vp_build", "vp_get_info", "vp_set_option", "vp_workspace_bytes",
           "vp_project", "vp_project_static", "vp_project_full", "vp_union_workspace_bytes", "vp_project_union",
           "vp_project_debug_logits", "vp_get_profile", "vp_destroy", "vp_last_error",
           "vp_kmeans_workspace_bytes", "vp_kmeans", "vp_active_sets_workspace_bytes", "vp_active_sets",
           "vp_round_to_half", "vp_beam_step", "vp_measure_ceilings")


class VpError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("%s: %s" % (STATUS_NAMES.get(status, status), message))
        self.status = status


class BuildDesc(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int32), ("V", ctypes.c_int32), ("K", ctypes.c_int32),
                ("W", ctypes.c_void_p), ("bias", ctypes.c_void_p), ("centroids", ctypes.c_void_p),
                ("cand_offsets", ctypes.c_void_p), ("cand_ids", ctypes.c_void_p),
                ("arena", ctypes.c_void_p), ("arena_bytes", ctypes.c_size_t),
                ("k_max", ctypes.c_int32), ("flags", ctypes.c_uint32)]


class IndexInfo(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int32), ("V", ctypes.c_int32), ("K", ctypes.c_int32),
                ("k_max", ctypes.c_int32), ("d_pad", ctypes.c_int32), ("n_min", ctypes.c_int32),
                ("n_max", ctypes.c_int32), ("n_total", ctypes.c_int64), ("slab_bytes", ctypes.c_int64),
                ("full_bytes", ctypes.c_int64), ("arena_bytes_used", ctypes.c_int64)]


_lib = None


def lib():
    """Loads libvp.so (built in-tree by paper_2208_06874_amd/build.py); fails loudly."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: run `python -m paper_2208_06874_amd.build` "
                               "(there is no non-HIP fallback)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        L.vp_last_error.restype = ctypes.c_char_p
        L.vp_build_bytes.restype = ctypes.c_size_t
        L.vp_build_bytes.argtypes = [ctypes.POINTER(BuildDesc)]
        L.vp_build.restype = ctypes.c_int
        L.vp_build.argtypes = [ctypes.POINTER(BuildDesc), vp, ctypes.POINTER(vp)]
        L.vp_get_info.restype = ctypes.c_int
        L.vp_get_info.argtypes = [vp, ctypes.POINTER(IndexInfo)]
        L.vp_set_option.restype = ctypes.c_int
        L.vp_set_option.argtypes = [vp, ctypes.c_char_p, ctypes.c_int64]
        L.vp_workspace_bytes.restype = ctypes.c_size_t
        L.vp_workspace_bytes.argtypes = [vp, ctypes.c_int32]
        L.vp_project.restype = ctypes.c_int
        L.vp_project.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.vp_project_static.restype = ctypes.c_int
        L.vp_project_static.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp]
        L.vp_project_full.restype = ctypes.c_int
        L.vp_project_full.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, ctypes.c_size_t, vp]
        L.vp_union_workspace_bytes.restype = ctypes.c_size_t
        L.vp_union_workspace_bytes.argtypes = [vp, ctypes.c_int32]
        L.vp_project_union.restype = ctypes.c_int
        L.vp_project_union.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.vp_project_debug_logits.restype = ctypes.c_int
        L.vp_project_debug_logits.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp,
                                              ctypes.c_size_t, vp, ctypes.c_size_t, vp]
        L.vp_get_profile.restype = ctypes.c_int
        L.vp_get_profile.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
        L.vp_destroy.restype = None
        L.vp_destroy.argtypes = [vp]
        L.vp_kmeans_workspace_bytes.restype = ctypes.c_size_t
        L.vp_kmeans_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
        L.vp_kmeans.restype = ctypes.c_int
        L.vp_kmeans.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_uint32, vp, vp,
                                vp, vp, ctypes.c_size_t, vp]
        L.vp_active_sets_workspace_bytes.restype = ctypes.c_size_t
        L.vp_active_sets_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32]
        L.vp_active_sets.restype = ctypes.c_int
        L.vp_active_sets.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp,
                                     ctypes.c_int64, ctypes.POINTER(ctypes.c_int64), vp, ctypes.c_size_t, vp]
        L.vp_beam_step.restype = ctypes.c_int
        L.vp_beam_step.argtypes = [vp, vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp]
        L.vp_measure_ceilings.restype = ctypes.c_int
        L.vp_measure_ceilings.argtypes = [vp, ctypes.c_size_t, ctypes.c_int32, ctypes.POINTER(ctypes.c_double),
                                          ctypes.POINTER(ctypes.c_double), vp]
        L.vp_round_to_half.restype = ctypes.c_uint16
        L.vp_round_to_half.argtypes = [ctypes.c_double]
        _lib = L
    return _lib


def last_error() -> str:
    return lib().vp_last_error().decode()


def _check(status: int):
    if status != VP_OK:
        raise VpError(status, last_error())


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _want(t, name: str, dtype, shape=None, device=None, optional: bool = False):
    """Checks a tensor argument before its address crosses the C ABI: a host pointer, a view with
    strides or a buffer of the wrong size would make the kernels read or write out of bounds."""
    import torch
    if t is None:
        if optional:
            return None
        raise ValueError("%s is required" % name)
    if not isinstance(t, torch.Tensor):
        raise TypeError("%s must be a torch.Tensor, got %s" % (name, type(t).__name__))
    if t.dtype != dtype:
        raise ValueError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    if not t.is_cuda:
        raise ValueError("%s must live in GPU memory (got a %s tensor)" % (name, t.device))
    if device is not None and t.device != device:
        raise ValueError("%s is on %s, the index on %s" % (name, t.device, device))
    return t


def _want_bytes(t, name: str, need: int, device=None):
    """A workspace: flat uint8, contiguous, on the GPU.  (Its size is checked by the library itself, on the
    host and before anything is launched: a short one gives VP_ERR_WORKSPACE.)"""
    import torch
    _want(t, name, torch.uint8, None, device)
    if t.dim() != 1:
        raise ValueError("%s must be a flat uint8 tensor, got shape %s" % (name, tuple(t.shape)))
    return t


def _stream(stream=None) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def make_desc(d, V, K, W, bias, centroids, cand_off: np.ndarray, cand_ids: np.ndarray, arena, arena_bytes,
              k_max, flags=0) -> BuildDesc:
    return BuildDesc(d, V, K, W, bias, centroids, cand_off.ctypes.data, cand_ids.ctypes.data, arena,
                     arena_bytes, k_max, flags)


class Index:
    """A packed index living in a torch uint8 arena on the GPU."""

    def __init__(self, W, bias, centroids, cand_off, cand_ids, k_max: int = 8, stream=None, flags: int = 0):
        import torch
        if not isinstance(W, torch.Tensor) or W.dim() != 2:
            raise ValueError("W must be a [d, V] tensor")
        d, V = W.shape
        if not isinstance(centroids, torch.Tensor) or centroids.dim() != 2 or centroids.shape[1] != d:
            raise ValueError("centroids must be a [K, d] tensor")
        K = centroids.shape[0]
        _want(W, "W", torch.float16)
        _want(bias, "bias", torch.float16, (V,), W.device)
        # (contiguous copies, if any were needed, must stay alive until vp_build has read them)
        self._C = _want(centroids.contiguous(), "centroids", torch.float16, (K, d), W.device)
        self._off = np.ascontiguousarray(cand_off, np.int64)
        self._ids = np.ascontiguousarray(cand_ids, np.int32)
        if self._off.shape != (K + 1,):
            raise ValueError("cand_off must have K + 1 = %d entries, got %s" % (K + 1, self._off.shape))
        if self._ids.ndim != 1 or (len(self._off) and self._ids.shape[0] != int(self._off[-1])):
            raise ValueError("cand_ids must hold cand_off[K] = %d entries, got %s" % (int(self._off[-1]), self._ids.shape))
        desc = make_desc(d, V, K, W.data_ptr(), bias.data_ptr(), self._C.data_ptr(), self._off,
                         self._ids, None, 0, k_max, flags)
        need = lib().vp_build_bytes(ctypes.byref(desc))
        if need == 0:
            # let vp_build report the precise status
            h = ctypes.c_void_p()
            _check(lib().vp_build(ctypes.byref(desc), _stream(stream), ctypes.byref(h)))
            raise VpError(VP_ERR_INVALID_ARG, last_error())
        self.arena = torch.empty(need, dtype=torch.uint8, device=W.device)
        desc.arena = self.arena.data_ptr()
        desc.arena_bytes = need
        h = ctypes.c_void_p()
        _check(lib().vp_build(ctypes.byref(desc), _stream(stream), ctypes.byref(h)))
        self.handle = h
        self._C = None    # vp_build has synchronised: the index holds its own packed copy
        self.device = W.device
        self.d, self.V, self.K, self.k_max = d, V, K, k_max
        self._ws = {}     # cached scratch buffers, one per stream: calls that share one must not overlap
        self._uws = {}

    def close(self):
        # (also runs from __del__ at interpreter shutdown, when module globals may already be gone)
        if getattr(self, "handle", None) and callable(lib):
            lib().vp_destroy(self.handle)
            self.handle = None

    __del__ = close

    def info(self) -> dict:
        i = IndexInfo()
        _check(lib().vp_get_info(self.handle, ctypes.byref(i)))
        return {f: getattr(i, f) for f, _ in IndexInfo._fields_}

    def set_option(self, name: str, value: int):
        _check(lib().vp_set_option(self.handle, name.encode(), int(value)))
        self._ws = {}     # the workspace size depends on the options
        self._uws = {}

    def get_profile(self):
        """(summed projection-kernel milliseconds, launches) since the last call."""
        ms, n = ctypes.c_double(), ctypes.c_int64()
        _check(lib().vp_get_profile(self.handle, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    def workspace_bytes(self, N: int) -> int:
        return lib().vp_workspace_bytes(self.handle, N)

    def workspace(self, N: int, stream=None):
        """The index's cached scratch buffer for calls on this stream (default: torch's current stream), grown
        on demand; the calls below use it when no workspace is passed.  Calls that share a workspace must not
        overlap, which calls on one stream never do; callers that want a workspace of their own allocate
        workspace_bytes(N) bytes and pass it."""
        import torch
        need = self.workspace_bytes(N)
        key = _stream(stream)
        ws = self._ws.get(key)
        if ws is None or ws.numel() < need:
            ws = self._ws[key] = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
        return ws

    def project(self, hidden, k: int, out_ids=None, out_logp=None, out_cluster=None, want_cluster=True,
                workspace=None, stream=None):
        """vp_project: hidden[N, d] fp16 -> (ids[N, k] int32, logp[N, k] fp32, cluster[N] int32)."""
        import torch
        N = self._rows(hidden)
        out_ids, out_logp = self._outputs(N, k, out_ids, out_logp)
        if out_cluster is None and want_cluster:
            out_cluster = torch.empty((N,), dtype=torch.int32, device=self.device)
        _want(out_cluster, "out_cluster", torch.int32, (N,), self.device, optional=True)
        ws = self.workspace(N, stream) if workspace is None else _want_bytes(workspace, "workspace",
                                                                           self.workspace_bytes(N), self.device)
        _check(lib().vp_project(self.handle, hidden.data_ptr(), N, k, out_ids.data_ptr(), out_logp.data_ptr(),
                                _ptr(out_cluster), ws.data_ptr(), ws.numel(), _stream(stream)))
        return out_ids, out_logp, out_cluster

    def _rows(self, hidden) -> int:
        import torch
        if not isinstance(hidden, torch.Tensor) or hidden.dim() != 2:
            raise ValueError("hidden must be an [N, d] tensor")
        _want(hidden, "hidden", torch.float16, (hidden.shape[0], self.d), self.device)
        return hidden.shape[0]

    def _outputs(self, N: int, k: int, out_ids, out_logp):
        import torch
        if out_ids is None:
            out_ids = torch.empty((N, k), dtype=torch.int32, device=self.device)
        if out_logp is None:
            out_logp = torch.empty((N, k), dtype=torch.float32, device=self.device)
        _want(out_ids, "out_ids", torch.int32, (N, k), self.device)
        _want(out_logp, "out_logp", torch.float32, (N, k), self.device)
        return out_ids, out_logp

    def project_static(self, hidden, k: int, out_ids, out_logp, out_cluster=None, stream=None):
        """vp_project_static: vp_project on the library's own scratch array; the caller passes every output
        (nothing is allocated here either)."""
        import torch
        N = self._rows(hidden)
        _want(out_ids, "out_ids", torch.int32, (N, k), self.device)
        _want(out_logp, "out_logp", torch.float32, (N, k), self.device)
        _want(out_cluster, "out_cluster", torch.int32, (N,), self.device, optional=True)
        _check(lib().vp_project_static(self.handle, hidden.data_ptr(), N, k, out_ids.data_ptr(), out_logp.data_ptr(),
                                       _ptr(out_cluster), _stream(stream)))
        return out_ids, out_logp, out_cluster

    def project_full(self, hidden, k: int, out_ids=None, out_logp=None, workspace=None, stream=None):
        """vp_project_full: the default projection over all V tokens."""
        N = self._rows(hidden)
        out_ids, out_logp = self._outputs(N, k, out_ids, out_logp)
        ws = self.workspace(N, stream) if workspace is None else _want_bytes(workspace, "workspace",
                                                                           self.workspace_bytes(N), self.device)
        _check(lib().vp_project_full(self.handle, hidden.data_ptr(), N, k, out_ids.data_ptr(),
                                     out_logp.data_ptr(), ws.data_ptr(), ws.numel(), _stream(stream)))
        return out_ids, out_logp

    def union_workspace_bytes(self, N: int) -> int:
        return lib().vp_union_workspace_bytes(self.handle, N)

    def project_union(self, hidden, k: int, out_ids=None, out_logp=None, out_cluster=None, out_union_size=None,
                      workspace=None, stream=None):
        """vp_project_union: the paper's batched form -> (ids, logp, cluster, union_size[1])."""
        import torch
        N = self._rows(hidden)
        out_ids, out_logp = self._outputs(N, k, out_ids, out_logp)
        if out_cluster is None:
            out_cluster = torch.empty((N,), dtype=torch.int32, device=self.device)
        if out_union_size is None:
            out_union_size = torch.zeros((1,), dtype=torch.int32, device=self.device)
        _want(out_cluster, "out_cluster", torch.int32, (N,), self.device)
        _want(out_union_size, "out_union_size", torch.int32, (1,), self.device)
        need = self.union_workspace_bytes(N)
        if workspace is None:
            key = _stream(stream)
            workspace = self._uws.get(key)
            if workspace is None or workspace.numel() < need:
                workspace = self._uws[key] = torch.empty(max(need, 256), dtype=torch.uint8, device=self.device)
        else:
            _want_bytes(workspace, "workspace", need, self.device)
        _check(lib().vp_project_union(self.handle, hidden.data_ptr(), N, k, out_ids.data_ptr(), out_logp.data_ptr(),
                                      out_cluster.data_ptr(), out_union_size.data_ptr(), workspace.data_ptr(),
                                      workspace.numel(), _stream(stream)))
        return out_ids, out_logp, out_cluster, out_union_size

    def debug_logits(self, hidden, full: bool = False, stream=None):
        """vp_project_debug_logits -> (cluster[N], row_offsets[N+1] int64, logits fp32)."""
        import torch
        N = self._rows(hidden)
        cap = N * (self.V if full else self.info()["n_max"])
        cluster = torch.empty((N,), dtype=torch.int32, device=self.device)
        offs = torch.empty((N + 1,), dtype=torch.int64, device=self.device)
        logits = torch.full((max(cap, 1),), float("nan"), dtype=torch.float32, device=self.device)
        ws = self.workspace(N, stream)
        _check(lib().vp_project_debug_logits(self.handle, hidden.data_ptr(), N, int(full), cluster.data_ptr(),
                                             offs.data_ptr(), logits.data_ptr(), cap, ws.data_ptr(), ws.numel(),
                                             _stream(stream)))
        return cluster, offs, logits


# ---- the C-ABI entry points under their own names --------------------------------------------
BUILD_NO_UNION = 1


def vp_build(W, bias, centroids, cand_off, cand_ids, k_max: int = 8, stream=None, flags: int = 0) -> Index:
    return Index(W, bias, centroids, cand_off, cand_ids, k_max=k_max, stream=stream, flags=flags)


def vp_project(index: Index, hidden, k: int, **kw):
    return index.project(hidden, k, **kw)


def vp_project_static(index: Index, hidden, k: int, out_ids, out_logp, out_cluster=None, stream=None):
    return index.project_static(hidden, k, out_ids, out_logp, out_cluster, stream=stream)


STATIC_SCRATCH_BYTES = 16 << 20


def vp_project_full(index: Index, hidden, k: int, **kw):
    return index.project_full(hidden, k, **kw)


def vp_project_union(index: Index, hidden, k: int, **kw):
    return index.project_union(hidden, k, **kw)


def vp_union_workspace_bytes(index: Index, N_max: int) -> int:
    return index.union_workspace_bytes(N_max)


def vp_project_debug_logits(index: Index, hidden, full: bool = False, **kw):
    return index.debug_logits(hidden, full=full, **kw)


def vp_workspace_bytes(index: Index, N_max: int) -> int:
    return index.workspace_bytes(N_max)


def vp_set_option(index: Index, name: str, value: int):
    index.set_option(name, value)


def vp_get_info(index: Index) -> dict:
    return index.info()


def vp_get_profile(index: Index):
    return index.get_profile()


def vp_destroy(index: Index):
    index.close()


def vp_last_error() -> str:
    return last_error()


def vp_measure_ceilings(buf, repeats: int = 5, stream=None):
    """vp_measure_ceilings on a uint8 GPU buffer -> (streaming-read GB/s, dense fp16 MFMA TFLOP/s)."""
    import torch
    _want(buf, "buf", torch.uint8)
    r, m = ctypes.c_double(), ctypes.c_double()
    _check(lib().vp_measure_ceilings(buf.data_ptr(), buf.numel(), int(repeats), ctypes.byref(r), ctypes.byref(m),
                                     _stream(stream)))
    return r.value, m.value


# ---------------------------------------------------------------- offline training of the clusters
def vp_round_to_half(v: float) -> int:
    return int(lib().vp_round_to_half(float(v)))


KMEANS_SPLIT_EMPTY = 1


def vp_kmeans(X, centroids, iters: int = 20, workspace=None, stream=None, split_empty: bool = False):
    """vp_kmeans: trains `centroids` (fp16 [K, d], updated in place) on X (fp16 [n, d]).
    Returns (assign int32 [n], counts int32 [K]) under the final centroids."""
    import torch
    if not isinstance(X, torch.Tensor) or X.dim() != 2 or not isinstance(centroids, torch.Tensor) or centroids.dim() != 2:
        raise ValueError("X must be an [n, d] and centroids a [K, d] tensor")
    n, d = X.shape
    K = centroids.shape[0]
    _want(X, "X", torch.float16)
    _want(centroids, "centroids", torch.float16, (K, d), X.device)
    need = lib().vp_kmeans_workspace_bytes(n, d, K)
    if need == 0:
        raise VpError(VP_ERR_UNSUPPORTED, last_error())
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    else:
        _want_bytes(workspace, "workspace", need, X.device)
    assign = torch.empty(n, dtype=torch.int32, device=X.device)
    counts = torch.empty(K, dtype=torch.int32, device=X.device)
    _check(lib().vp_kmeans(X.data_ptr(), n, d, K, iters, KMEANS_SPLIT_EMPTY if split_empty else 0, centroids.data_ptr(),
                           assign.data_ptr(), counts.data_ptr(),
                           workspace.data_ptr(), workspace.numel(), _stream(stream)))
    return assign, counts


def vp_active_sets(top_ids, assign, K: int, V: int, capacity: Optional[int] = None, stream=None):
    """vp_active_sets: returns (cand_offsets int64 [K+1], cand_ids int32 [total]) on the device."""
    import torch
    if not isinstance(top_ids, torch.Tensor) or top_ids.dim() != 2:
        raise ValueError("top_ids must be an [n, T] tensor")
    n, T = top_ids.shape
    _want(top_ids, "top_ids", torch.int32)
    _want(assign, "assign", torch.int32, (n,), top_ids.device)
    need = lib().vp_active_sets_workspace_bytes(K, V)
    if need == 0:
        raise VpError(VP_ERR_UNSUPPORTED, last_error())
    ws = torch.empty(need, dtype=torch.uint8, device=top_ids.device)
    if capacity is None:
        capacity = n * T   # a union cannot hold more entries than were recorded
    off = torch.empty(K + 1, dtype=torch.int64, device=top_ids.device)
    ids = torch.empty(max(capacity, 1), dtype=torch.int32, device=top_ids.device)
    total = ctypes.c_int64(0)
    _check(lib().vp_active_sets(top_ids.data_ptr(), assign.data_ptr(), n, T, K, V, off.data_ptr(), ids.data_ptr(),
                                capacity, ctypes.byref(total), ws.data_ptr(), ws.numel(), _stream(stream)))
    return off, ids[: total.value]


def vp_kmeans_workspace_bytes(n: int, d: int, K: int) -> int:
    return lib().vp_kmeans_workspace_bytes(n, d, K)


def vp_active_sets_workspace_bytes(K: int, V: int) -> int:
    return lib().vp_active_sets_workspace_bytes(K, V)


def vp_beam_step(cand_ids, cand_logp, scores, B: int, out=None, stream=None):
    """vp_beam_step: returns (out_scores fp32 [S*B], out_parent int32 [S*B], out_token int32 [S*B])."""
    import torch
    if not isinstance(cand_ids, torch.Tensor) or cand_ids.dim() != 2:
        raise ValueError("cand_ids must be an [S * B, k] tensor")
    n, k = cand_ids.shape
    _want(cand_ids, "cand_ids", torch.int32)
    _want(cand_logp, "cand_logp", torch.float32, (n, k), cand_ids.device)
    _want(scores, "scores", torch.float32, (n,), cand_ids.device)
    if B < 1 or n % B != 0:
        raise ValueError("the %d rows are not a whole number of sentences of %d hypotheses" % (n, B))
    if out is not None:
        _want(out[0], "out_scores", torch.float32, (n,), cand_ids.device)
        _want(out[1], "out_parent", torch.int32, (n,), cand_ids.device)
        _want(out[2], "out_token", torch.int32, (n,), cand_ids.device)
    if out is None:
        out = (torch.empty(n, dtype=torch.float32, device=cand_ids.device),
               torch.empty(n, dtype=torch.int32, device=cand_ids.device),
               torch.empty(n, dtype=torch.int32, device=cand_ids.device))
    _check(lib().vp_beam_step(cand_ids.data_ptr(), cand_logp.data_ptr(), scores.data_ptr(), n // B, B, k,
                              out[0].data_ptr(), out[1].data_ptr(), out[2].data_ptr(), _stream(stream)))
    return out
