"""Acceptance rule for GPU results against the CPU oracle.

fp16 inputs with fp32 accumulation against an fp64 oracle:
  * cluster ids equal, except where the oracle's own Eq. 2 scores of the two
    competing centroids differ by less than tau_c (the row is then re-evaluated
    by the oracle with the GPU's cluster forced);
  * top-k token ids equal position by position, except where the oracle's
    logits of the two competing tokens differ by less than TAU; the GPU ids
    must be distinct members of the row's active set;
  * logits and log-probs within TAU = 2e-2 absolute.
A second, much tighter bound (SANITY) is what fp32 accumulation over d <= 1536
products of magnitude <= ~1 should really achieve; it is asserted as well so
that a systematic error hiding inside the tolerance is still caught.
"""
import numpy as np

TAU = 2e-2
SANITY = 2e-3


def to_np(t):
    return t.detach().cpu().numpy()


def check_clusters(oracle, H, C, g_gpu):
    g_or, s = oracle.assign(H, C, return_scores=True)
    g_gpu = np.asarray(g_gpu)
    bad = np.nonzero(g_gpu != g_or)[0]
    excused = 0
    if bad.size:
        Hd = H.astype(np.float64)
        cn = (C.astype(np.float64) ** 2).sum(1).max()
        for r in bad:
            assert 0 <= g_gpu[r] < C.shape[0]
            tau_c = 1e-5 * ((Hd[r] ** 2).sum() + cn)
            gap = s[r, g_gpu[r]] - s[r, g_or[r]]
            assert gap < tau_c, "row %d: GPU cluster %d vs oracle %d, score gap %g" % (r, g_gpu[r], g_or[r], gap)
            excused += 1
    return g_or, excused


def check_projection(oracle, W, b, C, cand_off, cand_ids, H, k, ids_gpu, logp_gpu, g_gpu, logits_gpu=None,
                     offs_gpu=None):
    """Full element-by-element comparison of a clustered projection."""
    N = H.shape[0]
    _, excused_c = check_clusters(oracle, H, C, g_gpu)
    ref = oracle.project(W, b, C, cand_off, cand_ids, H, k, forced_g=np.asarray(g_gpu, np.int32), want_all=True)
    stats = _compare_topk(ref, cand_off, cand_ids, np.asarray(g_gpu), k, ids_gpu, logp_gpu)
    stats["excused_clusters"] = excused_c
    if logits_gpu is not None:
        offs_gpu = np.asarray(offs_gpu)
        assert np.array_equal(offs_gpu, ref["all_off"])
        zg = np.asarray(logits_gpu)[: ref["all_off"][-1]].astype(np.float64)
        assert not np.isnan(zg).any(), "debug logits left unwritten"
        err = np.abs(zg - ref["all_z"]).max() if zg.size else 0.0
        assert err <= TAU and err <= SANITY, "candidate logits off by %g" % err
        stats["max_logit_err"] = float(err)
    assert N == ids_gpu.shape[0]
    return stats


def _compare_topk(ref, cand_off, cand_ids, g, k, ids_gpu, logp_gpu):
    ids_gpu = np.asarray(ids_gpu)
    logp_gpu = np.asarray(logp_gpu).astype(np.float64)
    N = ids_gpu.shape[0]
    max_err = 0.0
    excused = 0
    for r in range(N):
        if cand_off is None:
            n = ref["V"]
            lo = 0
            zrow = ref["all_z"][r]
            members = None
        else:
            lo, hi = int(cand_off[g[r]]), int(cand_off[g[r] + 1])
            n = hi - lo
            members = cand_ids[lo:hi]
            zrow = ref["all_z"][ref["all_off"][r]: ref["all_off"][r + 1]]
        kk = min(k, n)
        got = ids_gpu[r]
        assert np.all(got[kk:] == -1) and np.all(np.isneginf(logp_gpu[r, kk:])), "row %d padding" % r
        assert len(set(got[:kk].tolist())) == kk, "row %d: duplicate ids %s" % (r, got)
        if members is None:
            assert np.all((got[:kk] >= 0) & (got[:kk] < n))
            pos = got[:kk]
        else:
            pos = np.searchsorted(members, got[:kk])
            assert np.all(pos < n) and np.array_equal(members[pos], got[:kk]), "row %d: id outside the active set" % r
        z_of_gpu = zrow[pos]
        want_ids = ref["ids"][r, :kk]
        want_z = ref["z"][r, :kk]
        diff = got[:kk] != want_ids
        if diff.any():
            gap = np.abs(z_of_gpu[diff] - want_z[diff])
            assert np.all(gap < TAU), "row %d: ids %s vs %s, logit gaps %s" % (r, got[:kk], want_ids, gap)
            excused += int(diff.sum())
        err = np.abs(logp_gpu[r, :kk] - (z_of_gpu - ref["lse"][r]))
        assert np.all(err <= TAU) and np.all(err <= SANITY), "row %d: logp off by %g" % (r, err.max())
        max_err = max(max_err, float(err.max()) if kk else 0.0)
    return dict(max_logp_err=max_err, excused_ids=excused)


def check_union(oracle, W, b, C, cand_off, cand_ids, H, k, ids_gpu, logp_gpu, g_gpu, union_size_gpu):
    """The batch-union form: every row against the union of the predicted clusters' active sets."""
    _, excused_c = check_clusters(oracle, H, C, g_gpu)
    ref = oracle.project_union(W, b, C, cand_off, cand_ids, H, k, forced_g=np.asarray(g_gpu, np.int32),
                               want_all=True)
    U = ref["U"]
    assert int(union_size_gpu) == len(U), "union size %d vs %d" % (int(union_size_gpu), len(U))
    N = H.shape[0]
    view = dict(ref)
    view["all_off"] = np.arange(N + 1, dtype=np.int64) * len(U)
    view["all_z"] = ref["all_z"].reshape(-1)
    one_off = np.array([0, len(U)], np.int64)
    stats = _compare_topk(view, one_off, U, np.zeros(N, np.int64), k, ids_gpu, logp_gpu)
    stats["excused_clusters"] = excused_c
    stats["union_size"] = len(U)
    return stats


def check_full(oracle, W, b, H, k, ids_gpu, logp_gpu, logits_gpu=None):
    ref = oracle.project_full(W, b, H, k, want_all=True)
    ref["V"] = W.shape[1]
    stats = _compare_topk(ref, None, None, None, k, ids_gpu, logp_gpu)
    if logits_gpu is not None:
        zg = np.asarray(logits_gpu).astype(np.float64).reshape(H.shape[0], W.shape[1])
        err = np.abs(zg - ref["all_z"]).max()
        assert err <= TAU and err <= SANITY, "full logits off by %g" % err
        stats["max_logit_err"] = float(err)
    return stats
