"""Seeded synthetic workloads shaped like the paper's (section 3.1: d = 1024,
V = 250,000 / 128,000, rows = batch x beam, hundreds to thousands of clusters).

This module only *generates inputs*: weights, centroids, hidden rows and the
per-cluster active-token lists.  It holds none of the projection path's own
arithmetic and is imported by the tests, the smoke check and the benchmark;
neither the CPU oracle nor the HIP library depends on it.  Everything it
returns is an input handed to both sides.

The active-token lists follow the paper's construction (section 2.2): the
set of a cluster is the union of the top-T predicted tokens of the cluster's
member vectors.  Members are seeded samples around the centroid; their
predictions come from a library matmul + top-k (torch), optionally on the
GPU for large vocabularies.  The union alone yields far fewer ids than the
configured list sizes, so each list is topped up with seeded random distinct
token ids to its target size.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Iterable, Optional, Sequence

import numpy as np

BASE_SEED = 220806874


@dataclass(frozen=True)
class Config:
    name: str
    index: int                 # position in the list of workloads (seeds derive from it)
    d: int
    V: int
    K: int
    N: int
    k: int
    top_t: int                 # tokens recorded per member vector
    n_samples: int             # member vectors per cluster
    n_global: int              # token ids shared by every cluster
    size_lo: int               # target list size range
    size_hi: int
    size_dist: str = "uniform"  # "uniform" | "loguniform"
    row_dist: str = "uniform"   # "uniform" | "zipf"
    zipf_s: float = 1.1
    noise: float = 0.3
    sweep_N: Sequence[int] = field(default_factory=tuple)


CONFIGS = {
    "tiny": Config("tiny", 0, d=512, V=32000, K=32, N=16, k=4, top_t=50, n_samples=256,
                   n_global=500, size_lo=1800, size_hi=2200),
    "mid": Config("mid", 1, d=1024, V=128000, K=200, N=64, k=8, top_t=100, n_samples=256,
                  n_global=1000, size_lo=5000, size_hi=8000),
    "large": Config("large", 2, d=1024, V=250000, K=1000, N=256, k=8, top_t=100,
                    n_samples=256, n_global=1000, size_lo=10000, size_hi=20000),
    "sweep": Config("sweep", 3, d=1024, V=250000, K=1000, N=1024, k=1, top_t=100,
                    n_samples=256, n_global=1000, size_lo=10000, size_hi=20000,
                    sweep_N=(1, 4, 16, 64, 256, 1024)),
    "skewed": Config("skewed", 4, d=1536, V=250000, K=500, N=4096, k=8, top_t=100,
                     n_samples=256, n_global=1000, size_lo=2000, size_hi=40000,
                     size_dist="loguniform", row_dist="zipf"),
}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of a workload with some fields replaced (used for reduced test sizes)."""
    d = dict(cfg.__dict__)
    d.update(kw)
    return Config(**d)


def _rng(cfg: Config, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * cfg.index + stream))


def make_model(cfg: Config):
    """W[d,V] ~ N(0, 1/d), b[V] ~ N(0, 0.1) (variance), C[K,d] ~ N(0, 1); fp16."""
    r = _rng(cfg, 0)
    W = (r.standard_normal((cfg.d, cfg.V), dtype=np.float32) / np.sqrt(cfg.d)).astype(np.float16)
    b = (r.standard_normal(cfg.V, dtype=np.float32) * np.sqrt(0.1)).astype(np.float16)
    C = r.standard_normal((cfg.K, cfg.d), dtype=np.float32).astype(np.float16)
    return W, b, C


def row_clusters(cfg: Config, N: int, stream: int = 1) -> np.ndarray:
    """Intended cluster of each row: uniform over clusters, or Zipf(s) over a
    seeded permutation of the clusters."""
    r = _rng(cfg, stream)
    if cfg.row_dist == "uniform":
        return r.integers(0, cfg.K, size=N).astype(np.int32)
    ranks = np.arange(1, cfg.K + 1, dtype=np.float64)
    p = ranks ** (-cfg.zipf_s)
    p /= p.sum()
    order = r.permutation(cfg.K)
    return order[r.choice(cfg.K, size=N, p=p)].astype(np.int32)


def make_rows(cfg: Config, C: np.ndarray, N: Optional[int] = None, stream: int = 1,
              clusters: Optional[np.ndarray] = None):
    """h_r = C[q_r] + noise * eps, eps ~ N(0, I); fp16.  Returns (H, q)."""
    N = cfg.N if N is None else N
    q = row_clusters(cfg, N, stream) if clusters is None else np.asarray(clusters, np.int32)
    r = _rng(cfg, 100 + stream)
    eps = r.standard_normal((N, cfg.d), dtype=np.float32)
    H = (C[q].astype(np.float32) + cfg.noise * eps).astype(np.float16)
    return H, q


def training_set(cfg: Config, C: np.ndarray, n: int, stream: int = 7):
    """Recorded hidden vectors for the offline training of the clusters: n draws from the same
    mixture as the decode rows (a centroid of C plus noise), and K of them, picked without
    replacement, as starting centroids.  Returns (X fp16 [n, d], q int32 [n], C0 fp16 [K, d])."""
    X, q = make_rows(cfg, C, N=n, stream=stream, clusters=_rng(cfg, 300 + stream).integers(0, C.shape[0], n))
    pick = _rng(cfg, 400 + stream).choice(n, size=C.shape[0], replace=False)
    return X, q.astype(np.int32), X[np.sort(pick)].copy()


def union_sorted(token_lists: Iterable[Iterable[int]]) -> np.ndarray:
    """Active set of a cluster: the union of its members' recorded tokens
    (section 2.2), as an ascending list without duplicates."""
    parts = [np.asarray(list(t), dtype=np.int64).ravel() for t in token_lists]
    if not parts:
        return np.zeros(0, np.int32)
    return np.unique(np.concatenate(parts)).astype(np.int32)


def list_sizes(cfg: Config) -> np.ndarray:
    r = _rng(cfg, 2)
    if cfg.size_dist == "loguniform":
        s = np.exp(r.uniform(np.log(cfg.size_lo), np.log(cfg.size_hi), size=cfg.K))
    else:
        s = r.uniform(cfg.size_lo, cfg.size_hi, size=cfg.K)
    return np.minimum(np.round(s).astype(np.int64), cfg.V)


def make_candidates(cfg: Config, W: np.ndarray, b: np.ndarray, C: np.ndarray,
                    device: str = "cpu", predicted: bool = True):
    """Per-cluster ascending token-id lists as CSR (cand_off[K+1] int64,
    cand_ids int32).

    predicted=True follows the construction above (member samples -> top-T
    tokens -> union, plus the shared global ids, plus the random top-up);
    predicted=False skips the member predictions and uses global ids +
    top-up only (same sizes, no matmul; for shapes where only list sizes
    matter).
    """
    import torch

    sizes = list_sizes(cfg)
    rg = _rng(cfg, 3)
    global_ids = np.sort(rg.choice(cfg.V, size=min(cfg.n_global, cfg.V), replace=False))
    dev = torch.device(device)
    if predicted:
        cdtype = torch.float16 if dev.type == "cuda" else torch.float32
        Wt = torch.from_numpy(W).to(dev).to(cdtype)
        bt = torch.from_numpy(b).to(dev).to(cdtype)
        Ct = torch.from_numpy(C).to(dev).to(cdtype)
        gen = torch.Generator(device="cpu")
        gen.manual_seed(BASE_SEED + 1000 * cfg.index + 4)
    lists = []
    rt = _rng(cfg, 5)
    for j in range(cfg.K):
        parts = [global_ids]
        if predicted:
            eps = torch.randn((cfg.n_samples, cfg.d), generator=gen, dtype=torch.float32)
            members = (Ct[j].float() + cfg.noise * eps.to(dev)).to(cdtype)
            scores = members @ Wt + bt
            top = torch.topk(scores, min(cfg.top_t, cfg.V), dim=1).indices
            parts.append(top.reshape(-1).cpu().numpy())
        base = union_sorted(parts)
        target = int(sizes[j])
        if base.shape[0] < target:
            # top-up: seeded random token ids not yet in the set
            need = target - base.shape[0]
            draw = rt.choice(cfg.V, size=min(cfg.V, need + base.shape[0] + 64), replace=False)
            extra = draw[~np.isin(draw, base, assume_unique=True)][:need]
            base = union_sorted([base, extra])
        lists.append(base)
    cand_off = np.zeros(cfg.K + 1, np.int64)
    np.cumsum([len(x) for x in lists], out=cand_off[1:])
    cand_ids = np.concatenate(lists).astype(np.int32)
    return cand_off, cand_ids


def full_lists(K: int, V: int):
    """Every cluster lists the whole vocabulary (the case in which the
    clustered path must reproduce the full projection)."""
    cand_off = np.arange(K + 1, dtype=np.int64) * V
    cand_ids = np.tile(np.arange(V, dtype=np.int32), K)
    return cand_off, cand_ids
