"""ctypes front end of the CPU oracle (``vp_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg, never by the product package.  It shares no
code with the HIP library and does not import it.

All array arguments are numpy arrays; fp16 data is passed as its raw bits.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, f) for f in ("vp_oracle.c", "vp_train_oracle.c", "vp_search_oracle.c")]
_SO = os.path.join(_HERE, "libvp_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle's C files with gcc (plain -O2 loops, OpenMP over rows only)."""
    stale = (not os.path.exists(_SO)) or os.path.getmtime(_SO) < max(os.path.getmtime(f) for f in _SRCS)
    if force or stale:
        tmp = _SO + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", tmp] + _SRCS + ["-lm"]
        )
        os.replace(tmp, _SO)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_SO)
        lib.vpo_half_to_double.restype = ctypes.c_double
        lib.vpo_half_to_double.argtypes = [ctypes.c_uint16]
        lib.vpo_log_softmax.restype = ctypes.c_double
        lib.vpo_double_to_half.restype = ctypes.c_uint16
        lib.vpo_double_to_half.argtypes = [ctypes.c_double]
        lib.vpo_active_sets.restype = ctypes.c_int64
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _bits(a) -> np.ndarray:
    """fp16 array (or raw uint16 bits) -> contiguous uint16 bit patterns."""
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("oracle inputs must be float16 or uint16 bit patterns, got %s" % a.dtype)
    return np.ascontiguousarray(a)


def half_to_double(bits: int) -> float:
    return float(_load().vpo_half_to_double(ctypes.c_uint16(int(bits))))


def cnorm(C) -> np.ndarray:
    C = _bits(C)
    K, d = C.shape
    out = np.empty(K, np.float64)
    _load().vpo_cnorm(_p(C), ctypes.c_int(K), ctypes.c_int(d), _p(out))
    return out


def assign(H, C, return_scores: bool = False):
    """Eq. 2: cluster id of every row (and optionally all N*K scores)."""
    H, C = _bits(H), _bits(C)
    N, d = H.shape
    K = C.shape[0]
    assert C.shape[1] == d
    cn = cnorm(C)
    g = np.empty(N, np.int32)
    scores = np.empty((N, K), np.float64) if return_scores else None
    _load().vpo_assign(_p(H), ctypes.c_int(N), ctypes.c_int(d), _p(C), ctypes.c_int(K),
                       _p(cn), _p(g), _p(scores))
    return (g, scores) if return_scores else g


def logits_row(W, b, h, ids=None) -> np.ndarray:
    """Eq. 1 for one row over the listed token ids (all V when ids is None)."""
    W, b, h = _bits(W), _bits(b), _bits(h)
    d, V = W.shape
    if ids is not None:
        ids = np.ascontiguousarray(ids, np.int32)
        n = ids.shape[0]
    else:
        n = V
    z = np.empty(n, np.float64)
    _load().vpo_logits_row(_p(W), _p(b), ctypes.c_int(d), ctypes.c_int(V), _p(h), _p(ids),
                           ctypes.c_int(n), _p(z))
    return z


def log_softmax(z):
    z = np.ascontiguousarray(z, np.float64)
    logp = np.empty_like(z)
    lse = _load().vpo_log_softmax(_p(z), ctypes.c_int(z.shape[0]), _p(logp))
    return logp, float(lse)


def topk(z, k: int) -> np.ndarray:
    z = np.ascontiguousarray(z, np.float64)
    pos = np.empty(k, np.int32)
    _load().vpo_topk(_p(z), ctypes.c_int(z.shape[0]), ctypes.c_int(k), _p(pos))
    return pos


def project(W, b, C, cand_off, cand_ids, H, k: int, forced_g=None, want_all: bool = False):
    """Clustered projection.  Returns a dict with g, ids, logp, z, lse and, if
    want_all, all_off / all_z (every candidate logit of every row)."""
    W, b, C, H = _bits(W), _bits(b), _bits(C), _bits(H)
    d, V = W.shape
    K = C.shape[0]
    N = H.shape[0]
    cand_off = np.ascontiguousarray(cand_off, np.int64)
    cand_ids = np.ascontiguousarray(cand_ids, np.int32)
    assert cand_off.shape[0] == K + 1
    g = np.empty(N, np.int32)
    ids = np.empty((N, k), np.int32)
    logp = np.empty((N, k), np.float64)
    z = np.empty((N, k), np.float64)
    lse = np.empty(N, np.float64)
    fg = None if forced_g is None else np.ascontiguousarray(forced_g, np.int32)
    all_off = all_z = None
    if want_all:
        # the row's cluster is needed to size the buffer: run Eq. 2 first
        g0 = assign(H, C)
        if fg is not None:
            g0 = np.where(fg >= 0, fg, g0).astype(np.int32)
        sizes = (cand_off[1:] - cand_off[:-1])[g0]
        all_off = np.zeros(N + 1, np.int64)
        np.cumsum(sizes, out=all_off[1:])
        all_z = np.empty(int(all_off[-1]), np.float64)
    _load().vpo_project(_p(W), _p(b), ctypes.c_int(d), ctypes.c_int(V), _p(C), ctypes.c_int(K),
                        _p(cand_off), _p(cand_ids), _p(H), ctypes.c_int(N), ctypes.c_int(k),
                        _p(fg), _p(g), _p(ids), _p(logp), _p(z), _p(lse), _p(all_off), _p(all_z))
    out = dict(g=g, ids=ids, logp=logp, z=z, lse=lse)
    if want_all:
        out["all_off"] = all_off
        out["all_z"] = all_z
    return out


def project_union(W, b, C, cand_off, cand_ids, H, k: int, forced_g=None, want_all: bool = False):
    """The paper's batched form: every row is projected onto the union U of the
    active sets of all predicted clusters and normalised over U.  Returns g, flags
    (the boolean list over V), U, ids, logp, z, lse and, if want_all, all_z[N, |U|]."""
    W, b, C, H = _bits(W), _bits(b), _bits(C), _bits(H)
    d, V = W.shape
    K = C.shape[0]
    N = H.shape[0]
    cand_off = np.ascontiguousarray(cand_off, np.int64)
    cand_ids = np.ascontiguousarray(cand_ids, np.int32)
    fg = None if forced_g is None else np.ascontiguousarray(forced_g, np.int32)
    g = np.empty(N, np.int32)
    flags = np.zeros(V, np.uint8)
    U = np.empty(V, np.int32)
    nU = ctypes.c_int32(0)
    ids = np.empty((N, k), np.int32)
    logp = np.empty((N, k), np.float64)
    z = np.empty((N, k), np.float64)
    lse = np.empty(N, np.float64)
    all_z = np.empty((N, V), np.float64) if want_all else None   # upper bound; trimmed below
    _load().vpo_project_union(_p(W), _p(b), ctypes.c_int(d), ctypes.c_int(V), _p(C), ctypes.c_int(K),
                              _p(cand_off), _p(cand_ids), _p(H), ctypes.c_int(N), ctypes.c_int(k), _p(fg),
                              _p(g), _p(flags), _p(U), ctypes.byref(nU), _p(ids), _p(logp), _p(z), _p(lse),
                              _p(all_z))
    n = nU.value
    out = dict(g=g, flags=flags, U=U[:n].copy(), ids=ids, logp=logp, z=z, lse=lse)
    if want_all:
        out["all_z"] = all_z.reshape(-1)[: N * n].reshape(N, n).copy()
    return out


def project_full(W, b, H, k: int, want_all: bool = False):
    """Full-vocabulary projection, log-softmax over V and top-k."""
    W, b, H = _bits(W), _bits(b), _bits(H)
    d, V = W.shape
    N = H.shape[0]
    ids = np.empty((N, k), np.int32)
    logp = np.empty((N, k), np.float64)
    z = np.empty((N, k), np.float64)
    lse = np.empty(N, np.float64)
    all_z = np.empty((N, V), np.float64) if want_all else None
    _load().vpo_project_full(_p(W), _p(b), ctypes.c_int(d), ctypes.c_int(V), _p(H),
                             ctypes.c_int(N), ctypes.c_int(k), _p(ids), _p(logp), _p(z), _p(lse),
                             _p(all_z))
    out = dict(ids=ids, logp=logp, z=z, lse=lse)
    if want_all:
        out["all_z"] = all_z
    return out


def logit_points(W, b, H, rows, toks) -> np.ndarray:
    """Eq. 1 for single (row, token) pairs."""
    W, b, H = _bits(W), _bits(b), _bits(H)
    d, V = W.shape
    rows = np.ascontiguousarray(rows, np.int32)
    toks = np.ascontiguousarray(toks, np.int32)
    z = np.empty(rows.shape[0], np.float64)
    _load().vpo_logit_points(_p(W), _p(b), ctypes.c_int(d), ctypes.c_int(V), _p(H), _p(rows),
                             _p(toks), ctypes.c_int(rows.shape[0]), _p(z))
    return z


# ------------------------------------------------------------------ offline training of the clusters
def double_to_half(v: float) -> int:
    """binary16 bit pattern of v, round to nearest even."""
    return int(_load().vpo_double_to_half(ctypes.c_double(float(v))))


def kmeans_step(X, C, forced=None):
    """One Lloyd iteration from the centroids C (float64 [K, d]).  Returns assign, counts, the new
    centroids (float64, not rounded) and the objective of the assignment."""
    X = _bits(X)
    n, d = X.shape
    C = np.ascontiguousarray(C, np.float64)
    K = C.shape[0]
    assert C.shape[1] == d
    fg = None if forced is None else np.ascontiguousarray(forced, np.int32)
    assign = np.empty(n, np.int32)
    counts = np.empty(K, np.int32)
    Cn = np.empty((K, d), np.float64)
    obj = ctypes.c_double(0.0)
    _load().vpo_kmeans_step(_p(X), ctypes.c_int(n), ctypes.c_int(d), _p(C), ctypes.c_int(K), _p(fg), _p(assign),
                            _p(counts), _p(Cn), ctypes.byref(obj))
    return dict(assign=assign, counts=counts, C=Cn, objective=obj.value)


def split_empty(C, counts, round_half: bool = True):
    """The optional remedy for clusters without members, applied to float64 centroids C [K, d] and the
    member counts.  Returns the new (C, counts)."""
    C = np.array(C, np.float64, order="C")
    counts = np.array(counts, np.int32)
    K, d = C.shape
    _load().vpo_split_empty(_p(C), _p(counts), ctypes.c_int(K), ctypes.c_int(d), ctypes.c_int(1 if round_half else 0))
    return C, counts


def kmeans(X, C0, iters: int, round_half: bool = True, split_empty: bool = False):
    """iters Lloyd iterations from the binary16 centroids C0, then the membership against the final
    centroids.  Returns C (float64), C_bits (uint16), assign, counts, objective[iters + 1]."""
    X, C0 = _bits(X), _bits(C0)
    n, d = X.shape
    K = C0.shape[0]
    assert C0.shape[1] == d
    C = np.empty((K, d), np.float64)
    Cb = np.empty((K, d), np.uint16)
    assign = np.empty(n, np.int32)
    counts = np.empty(K, np.int32)
    obj = np.empty(iters + 1, np.float64)
    _load().vpo_kmeans(_p(X), ctypes.c_int(n), ctypes.c_int(d), _p(C0), ctypes.c_int(K), ctypes.c_int(iters),
                       ctypes.c_int(1 if round_half else 0), ctypes.c_int(1 if split_empty else 0), _p(C), _p(Cb),
                       _p(assign), _p(counts), _p(obj))
    return dict(C=C, C_bits=Cb, assign=assign, counts=counts, objective=obj)


def active_sets(top, assign, K: int, V: int):
    """Section 2.2: per cluster, the ascending union of the recorded tokens of its members.
    top is int32 [n, T] (entries < 0 mean none).  Returns cand_off (int64 [K+1]) and cand_ids."""
    top = np.ascontiguousarray(top, np.int32)
    n, T = top.shape
    assign = np.ascontiguousarray(assign, np.int32)
    off = np.empty(K + 1, np.int64)
    args = (_p(top), ctypes.c_int(n), ctypes.c_int(T), _p(assign), ctypes.c_int(K), ctypes.c_int(V), _p(off))
    total = _load().vpo_active_sets(*args, None)
    ids = np.empty(int(total), np.int32)
    _load().vpo_active_sets(*args, _p(ids))
    return off, ids


# ------------------------------------------------------------------ toy search consumer
def beam_step(cand_ids, cand_logp, scores, B: int):
    """One beam-search step.  cand_ids int32 [S*B, k], cand_logp float32 [S*B, k], scores float32 [S*B].
    Returns (out_scores float32 [S*B], out_parent int32 [S*B], out_token int32 [S*B])."""
    cand_ids = np.ascontiguousarray(cand_ids, np.int32)
    cand_logp = np.ascontiguousarray(cand_logp, np.float32)
    scores = np.ascontiguousarray(scores, np.float32)
    n, k = cand_ids.shape
    assert n % B == 0 and cand_logp.shape == (n, k) and scores.shape == (n,)
    S = n // B
    out_s = np.empty(n, np.float32)
    out_p = np.empty(n, np.int32)
    out_t = np.empty(n, np.int32)
    _load().vpo_beam_step(_p(cand_ids), _p(cand_logp), _p(scores), ctypes.c_int(S), ctypes.c_int(B), ctypes.c_int(k),
                          _p(out_s), _p(out_p), _p(out_t))
    return out_s, out_p, out_t
