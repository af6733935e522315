"""GPU parity of the offline cluster training (paper, section 2.2): vp_kmeans and
vp_active_sets, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Centroids and active sets are compared bit for bit; memberships are equal
except where the oracle's own distances of the two competing centroids differ by less
than the tolerance of the fp32 scores."""
import ctypes

import numpy as np
import pytest

from paper_2208_06874_amd import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def _dev(a):
    torch = _torch()
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _gpu_kmeans(X, C0, iters, split_empty=False):
    """Returns (centroid bits uint16 [K, d], assign, counts) of vp_kmeans."""
    torch = _torch()
    from paper_2208_06874_amd import vp
    Xt, Ct = _dev(X), _dev(C0.copy())
    assign, counts = vp.vp_kmeans(Xt, Ct, iters, split_empty=split_empty)
    torch.cuda.synchronize()
    return pu.to_np(Ct).view(np.uint16), pu.to_np(assign), pu.to_np(counts)


def _check_membership(oracle, X, Cbits, assign_gpu):
    """GPU membership against the oracle's nearest centroid; returns the number of excused rows."""
    C = Cbits.view(np.float16)
    _, excused = pu.check_clusters(oracle, X, C, assign_gpu)
    return excused


def _mixture(cfg_name, n, **scale):
    cfg = wl.scaled(wl.CONFIGS[cfg_name], **scale) if scale else wl.CONFIGS[cfg_name]
    _W, _b, C = wl.make_model(cfg)
    X, q, C0 = wl.training_set(cfg, C, n)
    return cfg, X, q, C0


@pytest.mark.parametrize("name,n,scale", [("tiny", 4096, {}), ("tiny", 1000, dict(d=72, K=5)),
                                          ("mid", 3000, dict(d=264, K=77)), ("mid", 5000, dict(K=77)),
                                          ("skewed", 4500, dict(K=50)), ("tiny", 6000, dict(K=300)),
                                          ("mid", 6000, dict(K=260, d=264)), ("mid", 5000, dict(K=256, d=2056))])
def test_lloyd_steps_match_the_oracle(oracle, name, n, scale):
    cfg, X, _q, C0 = _mixture(name, n, **scale)
    Cb = C0.view(np.uint16).copy()
    excused = 0
    for step in range(3):
        # membership under the current centroids (no update) ...
        same, assign, counts = _gpu_kmeans(X, Cb.view(np.float16), 0)
        assert np.array_equal(same, Cb), "iters = 0 must leave the centroids alone"
        excused += _check_membership(oracle, X, Cb, assign)
        assert np.array_equal(counts, np.bincount(assign, minlength=Cb.shape[0]))
        # ... and one iteration from them: the means of exactly those members, rounded once
        new, _a2, _c2 = _gpu_kmeans(X, Cb.view(np.float16), 1)
        st = oracle.kmeans_step(X, Cb.view(np.float16).astype(np.float64), forced=assign)
        want = st["C"].astype(np.float16).view(np.uint16)
        assert np.array_equal(new, want), "step %d: %d centroid coordinates differ" % (step, (new != want).sum())
        Cb = new
    print("lloyd steps", name, n, scale, "excused memberships", excused)


def test_twenty_iterations_and_determinism(oracle):
    cfg, X, q, C0 = _mixture("tiny", 8192)
    Cb, assign, counts = _gpu_kmeans(X, C0, 20)
    Cb2, assign2, counts2 = _gpu_kmeans(X, C0, 20)
    assert np.array_equal(Cb, Cb2) and np.array_equal(assign, assign2) and np.array_equal(counts, counts2)
    ref = oracle.kmeans(X, C0, 20, round_half=True)
    excused = _check_membership(oracle, X, Cb, assign)
    assert counts.sum() == X.shape[0] and np.array_equal(counts, np.bincount(assign, minlength=cfg.K))
    if np.array_equal(Cb, ref["C_bits"]):
        assert excused > 0 or np.array_equal(assign, ref["assign"])
        outcome = "bit-identical centroids"
    else:
        # a membership decided differently inside the fp32 tolerance sends the two runs down
        # different paths; both must end at the same quality
        mine = oracle.kmeans_step(X, Cb.view(np.float16).astype(np.float64))["objective"]
        assert abs(mine - ref["objective"][-1]) <= 1e-3 * ref["objective"][-1]
        outcome = "objective %.6g vs %.6g" % (mine, ref["objective"][-1])
    # the training must have improved on the start
    assert ref["objective"][-1] < ref["objective"][0]
    print("twenty iterations:", outcome, "excused", excused)


@pytest.mark.parametrize("name,n,scale,lost", [("tiny", 3000, dict(d=72, K=9), 3), ("mid", 6000, dict(K=300, d=264), 40),
                                               ("tiny", 5000, dict(K=1100, d=64), 500), ("tiny", 40, dict(K=30, d=32), 25)])
def test_split_of_clusters_without_members(oracle, name, n, scale, lost):
    """Centroids that nobody is near lose their members in the first step; with the option set every
    iteration ends with the oracle's split of the largest clusters, bit for bit."""
    cfg, X, _q, C0 = _mixture(name, n, **scale)
    C0 = C0.copy()
    far = np.random.default_rng(lost).choice(C0.shape[0], lost, replace=False)
    C0[far] = np.float16(200.0)
    Cb = C0.view(np.uint16).copy()
    K = Cb.shape[0]
    for step in range(6):
        print("split", name, n, scale, "step", step, flush=True)
        _same, assign, counts = _gpu_kmeans(X, Cb.view(np.float16), 0)
        _check_membership(oracle, X, Cb, assign)
        new, _a2, _c2 = _gpu_kmeans(X, Cb.view(np.float16), 1, split_empty=True)
        st = oracle.kmeans_step(X, Cb.view(np.float16).astype(np.float64), forced=assign)
        rounded = st["C"].astype(np.float16).astype(np.float64)
        want, cn = oracle.split_empty(rounded, st["counts"], round_half=True)
        if step == 0:
            assert (st["counts"] == 0).sum() >= lost
            plain, _a3, _c3 = _gpu_kmeans(X, Cb.view(np.float16), 1)
            assert np.array_equal(plain, rounded.astype(np.float16).view(np.uint16)), "flag off: centroids stay"
        assert cn.sum() == n
        want = want.astype(np.float16).view(np.uint16)
        assert np.array_equal(new, want), "step %d: %d coordinates differ" % (step, (new != want).sum())
        Cb = new
    _same, assign, counts = _gpu_kmeans(X, Cb.view(np.float16), 0)
    empty_now = int((counts == 0).sum())
    print("split", name, "clusters without members after 6 iterations:", empty_now, "of", K)
    if n >= 2 * K:
        assert empty_now < lost


def test_ties_round_to_even_for_every_pair_of_neighbours(oracle):
    """One cluster of two members whose coordinates are neighbouring fp16 values: every mean is a tie."""
    pos = np.arange(0, 0x7bff, dtype=np.uint16)   # neighbour pairs (p, p + 1), all finite
    d = 4096
    for lo in range(0, len(pos), d):
        a = pos[lo:lo + d]
        if len(a) < d:
            a = np.concatenate([a, np.zeros(d - len(a), np.uint16)])
        sign = np.uint16(0x8000) if (lo // d) % 2 else np.uint16(0)
        X = np.stack([a | sign, (a + 1) | sign]).view(np.float16)
        C0 = X[:1].copy()
        got, assign, counts = _gpu_kmeans(X, C0, 1)
        assert counts.tolist() == [2] and assign.tolist() == [0, 0]
        mean = 0.5 * (X[0].astype(np.float64) + X[1].astype(np.float64))
        want = mean.astype(np.float16).view(np.uint16)
        assert np.array_equal(got[0], want)
        assert np.array_equal(got[0], np.array([oracle.double_to_half(v) for v in mean], np.uint16))


def test_edge_cases(oracle):
    torch = _torch()
    from paper_2208_06874_amd import vp
    # a centroid nobody is near keeps its value; K = 1; a single vector; more vectors than one launch takes
    cfg, X, _q, C0 = _mixture("tiny", 777, d=64, K=6)
    C0 = np.concatenate([C0, np.full((1, 64), 90.0, np.float16)])
    Cb, assign, counts = _gpu_kmeans(X, C0, 2)
    assert counts[-1] == 0 and np.all(Cb[-1].view(np.float16) == 90.0)
    ref = oracle.kmeans(X, C0, 2, round_half=True)
    if _check_membership(oracle, X, Cb, assign) == 0:
        assert np.array_equal(Cb, ref["C_bits"]) and np.array_equal(assign, ref["assign"])

    Cb, assign, counts = _gpu_kmeans(X, X[:1].copy(), 1)
    assert counts.tolist() == [777] and not assign.any()
    assert np.array_equal(Cb[0], X.astype(np.float64).mean(0).astype(np.float16).view(np.uint16))

    Cb, assign, counts = _gpu_kmeans(X[:1], C0[:3], 1)
    assert counts.sum() == 1 and np.array_equal(Cb[assign[0]], X[0].view(np.uint16))

    cfg, X, _q, C0 = _mixture("tiny", 70001, d=32, K=9)
    Cb, assign, counts = _gpu_kmeans(X, C0, 1)
    _s, a0, _c = _gpu_kmeans(X, C0, 0)
    st = oracle.kmeans_step(X, C0.astype(np.float64), forced=a0)
    assert np.array_equal(Cb, st["C"].astype(np.float16).view(np.uint16))
    assert _check_membership(oracle, X, Cb, assign) >= 0 and counts.sum() == 70001

    # argument errors leave the outputs alone
    Xt, Ct = _dev(X[:100]), _dev(C0)
    ws = torch.empty(16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(vp.VpError) as e:
        vp.vp_kmeans(Xt, Ct, 1, workspace=ws)
    assert e.value.status == vp.VP_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert np.array_equal(pu.to_np(Ct).view(np.uint16), C0.view(np.uint16))


def test_active_sets_match_the_oracle(oracle):
    torch = _torch()
    from paper_2208_06874_amd import vp
    r = np.random.default_rng(21)
    for n, T, K, V in ((5000, 5, 37, 1000), (300, 1, 4, 33), (20000, 3, 200, 128000), (0, 3, 5, 100)):
        top = r.integers(0, V, (n, T)).astype(np.int32)
        top[r.random((n, T)) < 0.05] = -1
        assign = r.integers(0, max(K - 1, 1), n).astype(np.int32)   # the last cluster stays empty
        if n:
            off, ids = vp.vp_active_sets(_dev(top), _dev(assign), K, V)
        else:
            off, ids = vp.vp_active_sets(torch.empty((0, T), dtype=torch.int32, device="cuda:0"),
                                         torch.empty(0, dtype=torch.int32, device="cuda:0"), K, V)
        torch.cuda.synchronize()
        want_off, want_ids = oracle.active_sets(top, assign, K, V)
        assert np.array_equal(pu.to_np(off), want_off)
        assert np.array_equal(pu.to_np(ids), want_ids)
    # too small an output: the total is reported, nothing is written
    top = r.integers(0, 50, (64, 2)).astype(np.int32)
    assign = np.zeros(64, np.int32)
    with pytest.raises(vp.VpError) as e:
        vp.vp_active_sets(_dev(top), _dev(assign), 2, 50, capacity=3)
    assert e.value.status == vp.VP_ERR_WORKSPACE and "needed" in str(e.value)


def test_worked_example_of_the_active_set(oracle):
    """Section 2.2: members with recorded tokens {2,4,6} and {2,8,9} give {2,4,6,8,9}."""
    torch = _torch()
    from paper_2208_06874_amd import vp
    top = np.array([[2, 4, 6], [2, 8, 9]], np.int32)
    off, ids = vp.vp_active_sets(_dev(top), _dev(np.zeros(2, np.int32)), 1, 10)
    torch.cuda.synchronize()
    assert pu.to_np(off).tolist() == [0, 5] and pu.to_np(ids).tolist() == [2, 4, 6, 8, 9]


def test_trained_index_end_to_end(oracle):
    """Record top-T tokens with the full projection, train the clusters, build the active sets, build
    the index from them and check a decode batch against the oracle with the same lists."""
    torch = _torch()
    from paper_2208_06874_amd import vp
    cfg = wl.CONFIGS["tiny"]
    W, b, C_true = wl.make_model(cfg)
    X, _q, C0 = wl.training_set(cfg, C_true, 6000)
    T = 3
    Wt, bt = _dev(W), _dev(b)
    boot = vp.vp_build(Wt, bt, _dev(C0[:1]), np.array([0, 1], np.int64), np.array([0], np.int32), k_max=T)
    Xt = _dev(X)
    top, _lp = boot.project_full(Xt, T)
    Ct = _dev(C0.copy())
    assign, counts = vp.vp_kmeans(Xt, Ct, 20)
    off, ids = vp.vp_active_sets(top, assign, cfg.K, cfg.V)
    torch.cuda.synchronize()
    counts = pu.to_np(counts)
    off_h, ids_h = pu.to_np(off), pu.to_np(ids)
    # the sets are the oracle's union of what was recorded, for the GPU's memberships
    want_off, want_ids = oracle.active_sets(pu.to_np(top), pu.to_np(assign), cfg.K, cfg.V)
    assert np.array_equal(off_h, want_off) and np.array_equal(ids_h, want_ids)
    # the recorded tokens are the oracle's top-T of the full projection
    sf = pu.check_full(oracle, W, b, X[:64], T, pu.to_np(top)[:64], pu.to_np(_lp)[:64])
    # a cluster that lost all its members has an empty active set; the index takes it as it is
    keep = np.nonzero(counts > 0)[0]
    sizes = np.diff(off_h)
    assert np.all(sizes[keep] > 0) and np.all(sizes[counts == 0] == 0)
    C_new = pu.to_np(Ct)
    index = vp.vp_build(Wt, bt, Ct, off_h, ids_h, k_max=8)
    H, _ = wl.make_rows(cfg, C_true, N=64, stream=9)
    out_ids, out_logp, g = index.project(_dev(H), 4)
    torch.cuda.synchronize()
    st = pu.check_projection(oracle, W, b, C_new, off_h, ids_h, H, 4, pu.to_np(out_ids), pu.to_np(out_logp),
                             pu.to_np(g))
    # the trained clusters do their job: the full projection's best token is in the row's active set
    f_ids, _ = boot.project_full(_dev(H), 1)
    torch.cuda.synchronize()
    hit = np.mean(pu.to_np(f_ids)[:, 0] == pu.to_np(out_ids)[:, 0])
    print("trained index:", st, sf, "top-1 agreement with the full projection %.3f" % hit,
          "clusters kept %d of %d," % (len(keep), cfg.K), "mean active set %.0f of %d" % (len(ids_h) / len(keep), cfg.V))
    assert hit >= 0.6


def test_cluster_sweep_of_the_benchmark_runs():
    """bench.py --cluster-sweep (synthetic analogue of the paper's section 3.5) on the tiny workload."""
    torch = _torch()
    import argparse
    import bench
    out = bench.cluster_sweep(argparse.Namespace(workload="tiny", train_vectors=8192), torch.device("cuda:0"))
    rows = out["rows"]
    assert len(rows) == 18 and all(r["ms_per_step"] > 0 and 0 < r["mean_active_fraction"] <= 1 for r in rows)
    # more recorded tokens per vector can only enlarge the active sets and the chance to hold the best token
    for a, b, c in zip(rows[0::3], rows[1::3], rows[2::3]):
        assert a["mean_active_fraction"] <= b["mean_active_fraction"] <= c["mean_active_fraction"]
        assert a["top1_in_active_set"] <= b["top1_in_active_set"] + 1e-9 <= c["top1_in_active_set"] + 2e-9


def test_random_training_shapes(oracle):
    """Seeded random (n, d, K): one Lloyd step from the same start must give the oracle's centroids bit for
    bit for the GPU's memberships, and the active sets of random recordings must match."""
    torch = _torch()
    from paper_2208_06874_amd import vp
    rs = np.random.default_rng(806874)
    for case in range(12):
        d = 8 * int(rs.integers(1, 200))
        K = int(rs.choice([1, 3, 40, 255, 256, 300, 700]))
        n = int(rs.integers(max(K, 2), 9000))
        print("random training: case %d  n %d d %d K %d" % (case, n, d, K), flush=True)
        centres = rs.standard_normal((K, d))
        q = rs.integers(0, K, n)
        X = (centres[q] + 0.4 * rs.standard_normal((n, d))).astype(np.float16)
        C0 = X[np.sort(rs.choice(n, K, replace=False))].copy()
        _same, a0, c0 = _gpu_kmeans(X, C0, 0)
        _check_membership(oracle, X, C0.view(np.uint16), a0)
        new, _a, _c = _gpu_kmeans(X, C0, 1)
        st = oracle.kmeans_step(X, C0.astype(np.float64), forced=a0)
        assert np.array_equal(new, st["C"].astype(np.float16).view(np.uint16))
        T, V = int(rs.integers(1, 6)), int(rs.integers(40, 3000))
        top = rs.integers(-1, V, (n, T)).astype(np.int32)
        off, ids = vp.vp_active_sets(_dev(top), _dev(a0), K, V)
        torch.cuda.synchronize()
        want_off, want_ids = oracle.active_sets(top, a0, K, V)
        assert np.array_equal(pu.to_np(off), want_off) and np.array_equal(pu.to_np(ids), want_ids)


def test_train_build_decode_joined_at_the_mid_shape(oracle):
    """The rows of the scope end to end at the mid shape (d = 1,024, V = 128,000, K = 200), every stage
    against its own oracle: clusters trained by vp_kmeans (Lloyd steps bit for bit, final memberships
    against brute force), active sets from recorded top-3 tokens (section 2.2), the index packed from them,
    and a beam search of 8 sentences x beam 8 that decodes on it with vp_project (section 2.3) and
    vp_beam_step (section 2.1), with the library's default options."""
    torch = _torch()
    from paper_2208_06874_amd import vp
    cfg = wl.CONFIGS["mid"]
    W, b, C_true = wl.make_model(cfg)
    n, T = 12000, 3
    X, _q, C0 = wl.training_set(cfg, C_true, n)
    Wt, bt, Xt = _dev(W), _dev(b), _dev(X)
    # recording: the full projection's top-T of every vector (sampled rows against the oracle)
    boot = vp.vp_build(Wt, bt, _dev(C0[:1]), np.array([0, 1], np.int64), np.array([0], np.int32), k_max=T)
    top, top_lp = boot.project_full(Xt, T)
    torch.cuda.synchronize()
    sample = np.array([0, 1, n // 2, n - 1])
    pu.check_full(oracle, W, b, X[sample], T, pu.to_np(top)[sample], pu.to_np(top_lp)[sample])
    # training: every Lloyd step the oracle's, given the GPU's memberships
    Cb = C0.view(np.uint16).copy()
    for step in range(3):
        _same, a, _c = _gpu_kmeans(X, Cb.view(np.float16), 0)
        _check_membership(oracle, X, Cb, a)
        new, _a2, _c2 = _gpu_kmeans(X, Cb.view(np.float16), 1)
        want = oracle.kmeans_step(X, Cb.view(np.float16).astype(np.float64), forced=a)["C"].astype(np.float16)
        assert np.array_equal(new, want.view(np.uint16)), "Lloyd step %d" % step
        Cb = new
    Ct = _dev(C0.copy())
    assign, counts = vp.vp_kmeans(Xt, Ct, 20)
    torch.cuda.synchronize()
    C_new = pu.to_np(Ct)
    excused = _check_membership(oracle, X, C_new.view(np.uint16), pu.to_np(assign))
    # active sets: the oracle's union of the recorded tokens of every cluster's members
    off, ids = vp.vp_active_sets(top, assign, cfg.K, cfg.V)
    torch.cuda.synchronize()
    off_h, ids_h = pu.to_np(off), pu.to_np(ids)
    want_off, want_ids = oracle.active_sets(pu.to_np(top), pu.to_np(assign), cfg.K, cfg.V)
    assert np.array_equal(off_h, want_off) and np.array_equal(ids_h, want_ids)
    # the index from the learned clusters, and a search that decodes on it
    index = vp.vp_build(Wt, bt, Ct, off_h, ids_h, k_max=8)
    S, B, k = 8, 8, 8
    scores = np.tile(np.array([0.0] + [-np.inf] * (B - 1), np.float32), S)
    parent = np.tile(np.arange(B, dtype=np.int32), S)
    for step in range(3):
        fresh, _ = wl.make_rows(cfg, C_true, N=S * B, stream=300 + step)
        gather = (np.arange(S * B) // B) * B + np.maximum(parent, 0)
        H = np.ascontiguousarray(fresh[gather])
        out_ids, out_logp, g = index.project(_dev(H), k)
        torch.cuda.synchronize()
        st = pu.check_projection(oracle, W, b, C_new, off_h, ids_h, H, k, pu.to_np(out_ids), pu.to_np(out_logp),
                                 pu.to_np(g))
        new = vp.vp_beam_step(out_ids, out_logp, _dev(scores), B)
        torch.cuda.synchronize()
        got = tuple(pu.to_np(o) for o in new)
        want = oracle.beam_step(pu.to_np(out_ids), pu.to_np(out_logp), scores, B)
        for a, w in zip(got, want):
            assert np.array_equal(a, w)
        scores, parent = got[0], got[1]
    sizes = np.diff(off_h)
    print("joined: clusters with members %d of %d, mean active set %.0f tokens, excused memberships %d, last step %s"
          % (int((pu.to_np(counts) > 0).sum()), cfg.K, sizes[sizes > 0].mean(), excused, st))
    assert np.isfinite(scores).sum() == S * B
