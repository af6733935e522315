"""Pins of the cluster-training oracle (paper, section 2.2 and the training settings of
section 3.1) against things other than itself: every binary16 value and a library cast for the
rounding, a hand-computed Lloyd step, two library k-means routines started from the same
centroids, brute-force membership, the monotone objective, and the worked example of the
active-set union.  No GPU, no HIP library."""
import os
import warnings

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _mixture(seed, n=600, d=12, K=7, spread=0.35):
    r = np.random.default_rng(seed)
    centres = r.standard_normal((K, d))
    q = r.integers(0, K, n)
    X = (centres[q] + spread * r.standard_normal((n, d))).astype(np.float16)
    C0 = X[r.choice(n, K, replace=False)].copy()
    return X, C0


# ------------------------------------------------------------------ rounding to binary16
def test_rounding_is_the_identity_on_every_binary16_value(oracle):
    for bits in range(0x10000):
        expo = (bits >> 10) & 0x1f
        if expo == 31 and (bits & 0x3ff):
            continue   # NaN payloads are not preserved
        v = oracle.half_to_double(bits)
        assert oracle.double_to_half(v) == bits, hex(bits)


def test_rounding_of_midpoints_goes_to_the_even_neighbour(oracle):
    pos = np.arange(0, 0x7c00, dtype=np.uint16)          # 0 .. largest finite, ascending in value
    vals = pos.view(np.float16).astype(np.float64)
    for i in range(0, len(pos) - 1, 7):
        mid = 0.5 * (vals[i] + vals[i + 1])               # exact in double
        want = int(pos[i]) if (pos[i] & 1) == 0 else int(pos[i + 1])
        assert oracle.double_to_half(mid) == want
        assert oracle.double_to_half(-mid) == (want | 0x8000)
        assert oracle.double_to_half(np.nextafter(mid, np.inf)) == int(pos[i + 1])
        assert oracle.double_to_half(np.nextafter(mid, -np.inf)) == int(pos[i])
    assert oracle.double_to_half(65519.99) == 0x7bff and oracle.double_to_half(65520.0) == 0x7c00


def test_rounding_matches_the_library_cast(oracle):
    r = np.random.default_rng(3)
    v = np.concatenate([r.standard_normal(20000), r.standard_normal(5000) * 1e-6, r.standard_normal(5000) * 3e4,
                        r.standard_normal(2000) * 1e-9, r.standard_normal(2000) * 1e6])
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half(x) for x in v], np.uint16)
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ Lloyd iteration
def test_lloyd_step_hand_case(oracle):
    # 1-D: {0, 2, 10, 12} from centroids {1, 12}: members {0,2,10 | 12}?  |10-1| = 9 > |10-12| = 2,
    # so {0,2} and {10,12}; means 1 and 11; objective 1 + 1 + 4 + 0 = 6.
    X = np.array([[0.0], [2.0], [10.0], [12.0]], np.float16)
    st = oracle.kmeans_step(X, np.array([[1.0], [12.0]]))
    assert st["assign"].tolist() == [0, 0, 1, 1] and st["counts"].tolist() == [2, 2]
    assert st["C"].ravel().tolist() == [1.0, 11.0] and st["objective"] == 6.0
    # 2-D, a tie: (1,0) is equally far from (0,0) and (2,0) -> lowest index; a third centroid far
    # away has no members and stays where it is.
    X = np.array([[1, 0], [0, 1], [3, 0], [3, 2]], np.float16)
    st = oracle.kmeans_step(X, np.array([[0.0, 0.0], [2.0, 0.0], [50.0, 50.0]]))
    assert st["assign"].tolist() == [0, 0, 1, 1] and st["counts"].tolist() == [2, 2, 0]
    assert st["C"].tolist() == [[0.5, 0.5], [3.0, 1.0], [50.0, 50.0]]
    assert st["objective"] == 1 + 1 + 1 + 5


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_membership_is_the_brute_force_nearest_centroid(oracle, seed):
    X, C0 = _mixture(seed)
    C = C0.astype(np.float64)
    st = oracle.kmeans_step(X, C)
    Xd = X.astype(np.float64)
    dist = ((Xd[:, None, :] - C[None, :, :]) ** 2).sum(-1)
    assert np.array_equal(st["assign"], dist.argmin(1))
    assert st["counts"].sum() == X.shape[0]
    assert np.isclose(st["objective"], dist.min(1).sum(), rtol=1e-12)
    for j in range(C.shape[0]):
        mem = Xd[st["assign"] == j]
        want = mem.mean(0) if len(mem) else C[j]
        assert np.allclose(st["C"][j], want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("iters", [1, 3, 20])
def test_iterations_match_library_kmeans(oracle, iters):
    from scipy.cluster.vq import kmeans2, vq
    from sklearn.cluster import KMeans

    X, C0 = _mixture(10 + iters, n=900, d=8, K=6)
    got = oracle.kmeans(X, C0, iters, round_half=False)
    Xd = X.astype(np.float64)
    with warnings.catch_warnings():
        warnings.simplefilter("ignore")
        book, _ = kmeans2(Xd, C0.astype(np.float64), iter=iters, minit="matrix", missing="warn")
        km = KMeans(n_clusters=C0.shape[0], init=C0.astype(np.float64), n_init=1, max_iter=iters, tol=0.0,
                    algorithm="lloyd").fit(Xd)
    assert np.allclose(got["C"], book, rtol=0, atol=1e-10)
    assert np.array_equal(got["assign"], vq(Xd, book)[0])
    assert np.allclose(got["C"], km.cluster_centers_, rtol=0, atol=1e-8)
    assert np.isclose(got["objective"][-1], ((Xd - got["C"][got["assign"]]) ** 2).sum(), rtol=1e-12)


def test_objective_never_increases_and_empty_cluster_keeps_its_centroid(oracle):
    X, C0 = _mixture(5, n=500, d=10, K=6)
    C0 = np.concatenate([C0, np.full((1, 10), 40.0, np.float16)])   # nobody is near this one
    got = oracle.kmeans(X, C0, 12, round_half=False)
    obj = got["objective"]
    assert np.all(np.diff(obj) <= 1e-9 * obj[0])
    assert got["counts"][-1] == 0 and np.all(got["C"][-1] == 40.0)
    assert got["counts"].sum() == 500


def test_rounded_iteration_is_the_step_followed_by_the_library_cast(oracle):
    X, C0 = _mixture(8, n=700, d=16, K=9)
    C = C0.astype(np.float64)
    for _ in range(3):
        st = oracle.kmeans_step(X, C)
        C = st["C"].astype(np.float16).astype(np.float64)
    got = oracle.kmeans(X, C0, 3, round_half=True)
    assert np.array_equal(got["C"], C)
    assert np.array_equal(got["C_bits"], C.astype(np.float16).view(np.uint16))
    # its objective may rise by rounding only: far less than one part in 10^3 per step
    assert np.all(np.diff(got["objective"]) <= 1e-3 * got["objective"][0])


def test_forced_membership(oracle):
    X, C0 = _mixture(4, n=50, d=6, K=4)
    C = C0.astype(np.float64)
    free = oracle.kmeans_step(X, C)
    forced = np.full(50, -1, np.int32)
    forced[7] = (free["assign"][7] + 1) % 4
    st = oracle.kmeans_step(X, C, forced=forced)
    want = free["assign"].copy()
    want[7] = forced[7]
    assert np.array_equal(st["assign"], want)
    mem = X[want == forced[7]].astype(np.float64)
    assert np.allclose(st["C"][forced[7]], mem.mean(0), atol=1e-12)
    assert st["objective"] > free["objective"]


def test_split_of_empty_clusters(oracle):
    # hand case: clusters 1 and 3 are empty; 0 has 7 members, 2 has 4.  Cluster 1 splits cluster 0 (7 -> 4 + 3),
    # then the sizes are 4, 3, 4, 0: cluster 3 splits the lowest of the largest, cluster 0 again (4 -> 2 + 2).
    C = np.array([[1.0, -2.0], [9.0, 9.0], [0.5, 0.25], [7.0, 7.0]])
    counts = np.array([7, 0, 4, 0], np.int32)
    eps = 2.0 ** -10
    Cn, cn = oracle.split_empty(C, counts, round_half=False)
    assert cn.tolist() == [2, 3, 4, 2]
    once = C[0] * (1 - eps)
    assert np.array_equal(Cn[1], C[0] * (1 + eps)) and np.array_equal(Cn[3], once * (1 + eps))
    assert np.array_equal(Cn[0], once * (1 - eps)) and np.array_equal(Cn[2], C[2])
    # rounded form: each product goes through the library cast
    Ch, _ = oracle.split_empty(C, counts, round_half=True)
    h = lambda v: v.astype(np.float16).astype(np.float64)
    assert np.array_equal(Ch[1], h(C[0] * (1 + eps)))
    assert np.array_equal(Ch[3], h(h(C[0] * (1 - eps)) * (1 + eps)))
    # nothing to split from: a single member cannot be shared
    Cs, cs = oracle.split_empty(np.ones((3, 2)), np.array([1, 0, 0], np.int32))
    assert cs.tolist() == [1, 0, 0] and np.all(Cs == 1.0)


def test_training_with_the_split_leaves_no_empty_cluster(oracle):
    X, C0 = _mixture(9, n=800, d=10, K=8)
    C0 = np.concatenate([C0, np.full((2, 10), 30.0, np.float16)])        # two centroids nobody is near
    plain = oracle.kmeans(X, C0, 15, round_half=True, split_empty=False)
    split = oracle.kmeans(X, C0, 15, round_half=True, split_empty=True)
    assert (plain["counts"] == 0).sum() == 2 and (split["counts"] == 0).sum() == 0
    assert split["objective"][-1] < plain["objective"][-1]
    assert split["counts"].sum() == 800


# ------------------------------------------------------------------ active sets
def test_active_set_worked_example(oracle):
    members, rows = [], {}
    with open(os.path.join(GOLD, "active_set_union.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            (members.append([int(v) for v in vals]) if key == "member" else rows.__setitem__(key, [int(v) for v in vals]))
    top = np.array(members, np.int32)
    off, ids = oracle.active_sets(top, np.zeros(len(members), np.int32), K=1, V=10)
    assert off.tolist() == [0, len(rows["union"])] and ids.tolist() == rows["union"]


def test_active_sets_match_python_sets(oracle):
    r = np.random.default_rng(11)
    n, T, K, V = 400, 5, 9, 300
    top = r.integers(0, V, (n, T)).astype(np.int32)
    top[r.random((n, T)) < 0.1] = -1
    assign = r.integers(0, K - 1, n).astype(np.int32)      # cluster K-1 stays empty
    off, ids = oracle.active_sets(top, assign, K, V)
    assert off[0] == 0 and off[-1] == len(ids) and off[K] == off[K - 1]
    for j in range(K):
        want = sorted({int(v) for v in top[assign == j].ravel() if v >= 0})
        assert ids[off[j]:off[j + 1]].tolist() == want
