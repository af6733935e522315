"""Pins of the CPU oracle against things other than itself: closed forms,
brute force, a library routine on the special case that reduces to it, a
hand-computed case and the invariants the method fixes (paper sections
2.1 and 2.3).  No GPU, no HIP library."""
import os

import numpy as np
import pytest

from paper_2208_06874_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _small(seed, d=24, V=57, K=5, N=9):
    r = np.random.default_rng(seed)
    W = (r.standard_normal((d, V)) / np.sqrt(d)).astype(np.float16)
    b = (r.standard_normal(V) * 0.3).astype(np.float16)
    C = r.standard_normal((K, d)).astype(np.float16)
    q = r.integers(0, K, N)
    H = (C[q].astype(np.float32) + 0.3 * r.standard_normal((N, d))).astype(np.float16)
    return W, b, C, H


def _random_lists(r, K, V, lo, hi):
    lists = [np.sort(r.choice(V, size=int(r.integers(lo, hi + 1)), replace=False)) for _ in range(K)]
    off = np.zeros(K + 1, np.int64)
    np.cumsum([len(x) for x in lists], out=off[1:])
    return off, np.concatenate(lists).astype(np.int32)


# ---------------------------------------------------------------- fp16 decode
def test_half_decode_all_bit_patterns(oracle):
    """Every binary16 bit pattern widens to the value numpy assigns to it."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(x)) for x in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ------------------------------------------------------------- Eq. 2 (argmin)
def test_cnorm_closed_form(oracle):
    C = np.array([[3, 4, 0, 0], [1, 1, 1, 1], [0, 0, 0, 0], [-2, 0.5, 0, 1]], np.float16)
    assert np.array_equal(oracle.cnorm(C), np.array([25.0, 4.0, 0.0, 5.25]))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_assign_matches_brute_force_euclid(oracle, seed):
    """Eq. 2 picks the centroid nearest in Euclidean distance."""
    W, b, C, H = _small(seed, d=40, K=17, N=64)
    g, s = oracle.assign(H, C, return_scores=True)
    Hd, Cd = H.astype(np.float64), C.astype(np.float64)
    dist2 = ((Hd[:, None, :] - Cd[None, :, :]) ** 2).sum(-1)
    # scores differ from the squared distance by the row constant ||h||^2
    assert np.allclose(s + (Hd ** 2).sum(1)[:, None], dist2, rtol=0, atol=1e-9)
    srt = np.sort(dist2, axis=1)
    clear = (srt[:, 1] - srt[:, 0]) > 1e-9
    assert clear.all()
    assert np.array_equal(g, dist2.argmin(1))


def test_assign_signed_not_absolute(oracle):
    """Reading Eq. 2 with an absolute value would pick a far centroid whose
    score is near zero over the true nearest one whose score is negative."""
    C = np.array([[2.0, 0.0], [0.25, 0.0]], np.float16)
    H = np.array([[2.0, 0.0]], np.float16)       # h == C_0; score_0 = 4 - 8 = -4, score_1 = 1/16 - 1
    g, s = oracle.assign(H, C, return_scores=True)
    assert np.array_equal(s, [[-4.0, 0.0625 - 1.0]])
    assert g[0] == 0
    assert np.abs(s[0]).argmin() == 1             # the rejected reading disagrees


def test_assign_special_cases(oracle):
    r = np.random.default_rng(5)
    C = r.standard_normal((6, 16)).astype(np.float16)
    # a row equal to a centroid belongs to it
    assert np.array_equal(oracle.assign(C.copy(), C), np.arange(6))
    # duplicated centroid rows: the lower index wins
    C2 = np.concatenate([C, C[[3]], C[[1]]], 0)
    assert np.array_equal(oracle.assign(C.copy(), C2), np.arange(6))
    C3 = np.concatenate([C[[4]], C], 0)
    assert oracle.assign(C[[4]], C3)[0] == 0
    # one cluster
    assert np.array_equal(oracle.assign(C.copy(), C[:1]), np.zeros(6, np.int32))


# ----------------------------------------------------------- Eq. 1 + softmax
def test_full_matches_library_log_softmax(oracle):
    """The default projection is log_softmax(h W + b) and a descending sort."""
    W, b, C, H = _small(11, d=32, V=101, N=7)
    k = 6
    out = oracle.project_full(W, b, H, k, want_all=True)
    z = H.astype(np.float64) @ W.astype(np.float64) + b.astype(np.float64)
    assert np.allclose(out["all_z"], z, rtol=0, atol=1e-12)
    import torch
    lp = torch.log_softmax(torch.from_numpy(z), dim=1).numpy()
    order = np.argsort(-z, axis=1, kind="stable")[:, :k]
    assert np.array_equal(out["ids"], order)
    assert np.allclose(out["logp"], np.take_along_axis(lp, order, 1), rtol=0, atol=1e-12)
    assert np.allclose(out["z"], np.take_along_axis(z, order, 1), rtol=0, atol=1e-12)


def test_hand_case_integers(oracle):
    """d = 4, V = 6, K = 2 with small integers: logits written out by hand."""
    # columns of W are the tokens
    W = np.array([[1, 0, -1, 2, 0, 1],
                  [0, 1, 1, -1, 2, 1],
                  [2, -2, 0, 1, 1, 1],
                  [1, 1, -1, 0, -2, 1]], np.float16)
    b = np.array([0, 1, -1, 2, 0, -3], np.float16)
    C = np.array([[1, 1, 1, 1], [-1, 2, 0, -2]], np.float16)
    H = np.array([[1, 2, 1, 0],      # nearest C_0 (dist^2 2 vs 9)
                  [-1, 2, 0, -1]], np.float16)  # nearest C_1 (dist^2 10 vs 1)
    # full logits: row0 = [1+0+2+0, 0+2-2+0, -1+2+0+0, 2-2+1+0, 0+4+1+0, 1+2+1+0] + b
    z0 = np.array([3, 0, 1, 1, 5, 4]) + np.array([0, 1, -1, 2, 0, -3])     # [3,1,0,3,5,1]
    # row1 = [-1+0+0-1, 0+2+0-1, 1+2+0+1, -2-2+0+0, 0+4+0+2, -1+2+0-1] + b
    z1 = np.array([-2, 1, 4, -4, 6, 0]) + np.array([0, 1, -1, 2, 0, -3])   # [-2,2,3,-2,6,-3]
    cand_off = np.array([0, 4, 7], np.int64)
    cand_ids = np.array([0, 1, 3, 5,   2, 3, 4], np.int32)
    out = oracle.project(W, b, C, cand_off, cand_ids, H, k=3, want_all=True)
    assert np.array_equal(out["g"], [0, 1])
    assert np.array_equal(out["all_z"], np.concatenate([z0[[0, 1, 3, 5]], z1[[2, 3, 4]]]).astype(float))
    # row 0 candidates {0,1,3,5} -> logits [3,1,3,1]: ties go to the smaller token id
    assert np.array_equal(out["ids"][0], [0, 3, 1])
    # row 1 candidates {2,3,4} -> logits [3,-2,6]
    assert np.array_equal(out["ids"][1], [4, 2, 3])
    lse0 = np.log(2 * np.exp(3.0) + 2 * np.exp(1.0))
    lse1 = np.log(np.exp(3.0) + np.exp(-2.0) + np.exp(6.0))
    assert np.allclose(out["logp"][0], np.array([3, 3, 1]) - lse0, atol=1e-12)
    assert np.allclose(out["logp"][1], np.array([6, 3, -2]) - lse1, atol=1e-12)
    full = oracle.project_full(W, b, H, k=2)
    assert np.array_equal(full["ids"], [[4, 0], [4, 2]])
    assert np.allclose(full["z"], [[5, 3], [6, 3]])


def test_full_lists_reproduce_full_projection_exactly(oracle):
    """If every cluster lists the whole vocabulary, clustered == full, bit for bit."""
    W, b, C, H = _small(21, d=48, V=130, K=4, N=11)
    cand_off, cand_ids = wl.full_lists(4, 130)
    a = oracle.project(W, b, C, cand_off, cand_ids, H, k=5, want_all=True)
    f = oracle.project_full(W, b, H, k=5, want_all=True)
    assert np.array_equal(a["ids"], f["ids"])
    assert np.array_equal(a["logp"], f["logp"])
    assert np.array_equal(a["z"], f["z"])
    assert np.array_equal(a["all_z"].reshape(11, 130), f["all_z"])


def test_candidate_logits_are_a_subselection_of_full(oracle):
    W, b, C, H = _small(31, d=32, V=90, K=6, N=13)
    r = np.random.default_rng(31)
    cand_off, cand_ids = _random_lists(r, 6, 90, 5, 40)
    a = oracle.project(W, b, C, cand_off, cand_ids, H, k=3, want_all=True)
    f = oracle.project_full(W, b, H, k=1, want_all=True)
    for row in range(13):
        j = a["g"][row]
        ids = cand_ids[cand_off[j]:cand_off[j + 1]]
        assert np.array_equal(a["all_z"][a["all_off"][row]:a["all_off"][row + 1]], f["all_z"][row, ids])


def test_log_softmax_normalises_over_candidates(oracle):
    """Tokens outside the active set sit at -inf: probabilities of the listed
    tokens sum to one, and relate to the full softmax by renormalisation."""
    W, b, C, H = _small(41, d=32, V=80, K=5, N=10)
    r = np.random.default_rng(41)
    cand_off, cand_ids = _random_lists(r, 5, 80, 3, 50)
    n_all = cand_off[1:] - cand_off[:-1]
    g = oracle.assign(H, C)
    kmax = int(n_all.max())
    a = oracle.project(W, b, C, cand_off, cand_ids, H, k=kmax)
    f = oracle.project_full(W, b, H, k=1, want_all=True)
    zf = f["all_z"]
    logp_full = zf - f["lse"][:, None]
    for row in range(10):
        n = int(n_all[g[row]])
        lp = a["logp"][row, :n]
        assert abs(np.exp(lp).sum() - 1.0) < 1e-12
        assert np.all(np.isneginf(a["logp"][row, n:])) and np.all(a["ids"][row, n:] == -1)
        ids = a["ids"][row, :n]
        assert np.array_equal(np.sort(ids), cand_ids[cand_off[g[row]]:cand_off[g[row] + 1]])
        mass = np.log(np.exp(logp_full[row, ids]).sum())
        assert np.allclose(lp, logp_full[row, ids] - mass, rtol=0, atol=1e-12)
        # k = n returns the whole list in descending order of the logit
        assert np.all(np.diff(a["z"][row, :n]) <= 0)


def test_log_softmax_invariants(oracle):
    r = np.random.default_rng(3)
    z = r.standard_normal(37) * 4
    lp, lse = oracle.log_softmax(z)
    assert abs(np.exp(lp).sum() - 1) < 1e-12
    lp2, lse2 = oracle.log_softmax(z + 123.25)
    assert np.allclose(lp, lp2, atol=1e-12) and abs(lse2 - lse - 123.25) < 1e-12
    lp1, lse1 = oracle.log_softmax(np.array([-7.5]))
    assert lp1[0] == 0.0 and lse1 == -7.5
    # a superset can only lower each log-probability
    lp_sub, _ = oracle.log_softmax(z[:20])
    assert np.all(lp[:20] <= lp_sub + 1e-15)
    # large logits do not overflow
    lpb, _ = oracle.log_softmax(np.array([1000.0, 1000.0]))
    assert np.allclose(lpb, np.log(0.5))


def test_bias_shift_leaves_logp_unchanged(oracle):
    W, b, C, H = _small(51, d=16, V=40, K=3, N=6)
    cand_off, cand_ids = wl.full_lists(3, 40)
    a = oracle.project(W, b, C, cand_off, cand_ids, H, k=4)
    b2 = (b.astype(np.float32) * 0 + 2.0).astype(np.float16)  # constant bias
    b0 = np.zeros_like(b)
    x = oracle.project(W, b2, C, cand_off, cand_ids, H, k=4)
    y = oracle.project(W, b0, C, cand_off, cand_ids, H, k=4)
    assert np.array_equal(x["ids"], y["ids"])
    assert np.allclose(x["logp"], y["logp"], atol=1e-12)
    assert np.allclose(x["z"], y["z"] + 2.0, atol=1e-12)
    assert a["ids"].shape == (6, 4)


# --------------------------------------------------------------------- top-k
def test_topk_matches_stable_sort_and_ties(oracle):
    r = np.random.default_rng(8)
    z = np.round(r.standard_normal(200) * 2) / 2      # many exact ties
    for k in (1, 3, 17, 200):
        want = np.argsort(-z, kind="stable")[:k]
        assert np.array_equal(oracle.topk(z, k), want)
    assert np.array_equal(oracle.topk(np.array([1.0, 2.0]), 4), [1, 0, -1, -1])


def test_duplicate_columns_tie_goes_to_smaller_token(oracle):
    W, b, C, H = _small(61, d=16, V=30, K=2, N=5)
    W[:, 17] = W[:, 4]
    b[17] = b[4]
    W[:, 4] *= 8                                     # make the pair dominate
    W[:, 17] = W[:, 4]
    f = oracle.project_full(W, b, H, k=30, want_all=True)
    for row in range(5):
        ids = list(f["ids"][row])
        assert f["all_z"][row, 4] == f["all_z"][row, 17]
        assert ids.index(4) + 1 == ids.index(17)


def test_empty_active_set_gives_no_candidates(oracle):
    W, b, C, H = _small(21, N=6)
    off = np.array([0, 4, 4, 9, 9, 12], np.int64)            # clusters 1 and 3 list nothing
    ids = np.array([1, 5, 9, 30, 2, 4, 6, 8, 50, 0, 7, 56], np.int32)
    forced = np.array([0, 1, 2, 3, 4, 1], np.int32)
    out = oracle.project(W, b, C, off, ids, H, 3, forced_g=forced, want_all=True)
    for r in (1, 3, 5):
        assert out["ids"][r].tolist() == [-1, -1, -1] and np.all(np.isneginf(out["logp"][r]))
    assert out["all_off"].tolist() == [0, 4, 4, 9, 9, 12, 12]
    free = oracle.project(W, b, C, off, ids, H[[0, 2, 4]], 3, forced_g=forced[[0, 2, 4]])
    assert np.array_equal(free["ids"], out["ids"][[0, 2, 4]]) and np.array_equal(free["logp"], out["logp"][[0, 2, 4]])


def test_rows_are_independent(oracle):
    W, b, C, H = _small(71, d=24, V=64, K=4, N=12)
    r = np.random.default_rng(71)
    cand_off, cand_ids = _random_lists(r, 4, 64, 8, 30)
    a = oracle.project(W, b, C, cand_off, cand_ids, H, k=4)
    p = r.permutation(12)
    c = oracle.project(W, b, C, cand_off, cand_ids, H[p], k=4)
    for key in ("g", "ids", "logp", "z", "lse"):
        assert np.array_equal(a[key][p], c[key])


def test_forced_cluster(oracle):
    W, b, C, H = _small(81, d=24, V=64, K=4, N=6)
    r = np.random.default_rng(81)
    cand_off, cand_ids = _random_lists(r, 4, 64, 8, 30)
    forced = np.array([-1, 2, -1, 0, 3, -1], np.int32)
    a = oracle.project(W, b, C, cand_off, cand_ids, H, k=2)
    c = oracle.project(W, b, C, cand_off, cand_ids, H, k=2, forced_g=forced)
    want_g = np.where(forced >= 0, forced, a["g"])
    assert np.array_equal(c["g"], want_g)
    for row in range(6):
        ids = cand_ids[cand_off[want_g[row]]:cand_off[want_g[row] + 1]]
        assert set(c["ids"][row]) <= set(ids)


def test_logit_points(oracle):
    W, b, C, H = _small(91, d=24, V=64, N=6)
    f = oracle.project_full(W, b, H, k=1, want_all=True)
    rows = np.array([0, 5, 3, 3], np.int32)
    toks = np.array([63, 0, 17, 18], np.int32)
    assert np.array_equal(oracle.logit_points(W, b, H, rows, toks), f["all_z"][rows, toks])


# ------------------------------------------------ the paper's batch-union form
def test_union_worked_example_of_the_boolean_list(oracle):
    """Section 2.3: predicted centroids {0,1,2} with active sets {2,4,6}, {2,8,9},
    {1,3} give the boolean list [0,1,1,1,1,0,1,0,1,1] and the columns {1,2,3,4,6,8,9}."""
    members, rows = _read_golden("batch_union.txt")
    V, d = len(rows["flags"]), 8
    r = np.random.default_rng(0)
    W = (r.standard_normal((d, V)) / 3).astype(np.float16)
    b = np.zeros(V, np.float16)
    C = np.eye(3, d).astype(np.float16) * 4
    H = C.copy()                                   # row i sits on centroid i
    off = np.zeros(4, np.int64)
    np.cumsum([len(m) for m in members], out=off[1:])
    ids = np.concatenate(members).astype(np.int32)
    u = oracle.project_union(W, b, C, off, ids, H, k=3, want_all=True)
    assert list(u["g"]) == [0, 1, 2]
    assert list(u["flags"]) == rows["flags"]
    assert list(u["U"]) == rows["union"]
    f = oracle.project_full(W, b, H, k=1, want_all=True)
    assert np.array_equal(u["all_z"], f["all_z"][:, rows["union"]])
    assert np.allclose(np.exp(u["all_z"] - u["lse"][:, None]).sum(1), 1.0, atol=1e-12)


def test_union_equals_per_cluster_form_when_rows_share_a_cluster(oracle):
    W, b, C, H = _small(101, d=24, V=70, K=4, N=9)
    r = np.random.default_rng(101)
    cand_off, cand_ids = _random_lists(r, 4, 70, 5, 30)
    forced = np.full(9, 2, np.int32)
    a = oracle.project(W, b, C, cand_off, cand_ids, H, k=4, forced_g=forced)
    u = oracle.project_union(W, b, C, cand_off, cand_ids, H, k=4, forced_g=forced)
    assert np.array_equal(u["U"], cand_ids[cand_off[2]:cand_off[3]])
    for key in ("g", "ids", "logp", "z", "lse"):
        assert np.array_equal(a[key], u[key])


def test_union_normalises_over_the_union_and_relates_to_the_other_forms(oracle):
    W, b, C, H = _small(111, d=24, V=90, K=5, N=12)
    r = np.random.default_rng(111)
    cand_off, cand_ids = _random_lists(r, 5, 90, 5, 25)
    kk = 90
    u = oracle.project_union(W, b, C, cand_off, cand_ids, H, k=kk, want_all=True)
    a = oracle.project(W, b, C, cand_off, cand_ids, H, k=kk)
    f = oracle.project_full(W, b, H, k=1, want_all=True)
    U = u["U"]
    want_U = np.unique(np.concatenate([cand_ids[cand_off[j]:cand_off[j + 1]] for j in set(u["g"])]))
    assert np.array_equal(U, want_U) and np.array_equal(np.nonzero(u["flags"])[0], U)
    n = len(U)
    for row in range(12):
        lp = u["logp"][row, :n]
        assert abs(np.exp(lp).sum() - 1.0) < 1e-12
        assert np.all(u["ids"][row, n:] == -1)
        assert np.array_equal(np.sort(u["ids"][row, :n]), U)
        # the union is a superset of the row's own active set: its normaliser is larger
        assert u["lse"][row] >= a["lse"][row] - 1e-12
        # and renormalising the full softmax over U gives the same numbers
        logp_full = f["all_z"][row] - f["lse"][row]
        mass = np.log(np.exp(logp_full[U]).sum())
        assert np.allclose(lp, logp_full[u["ids"][row, :n]] - mass, atol=1e-12)
    cand_off_f, cand_ids_f = wl.full_lists(5, 90)
    uf = oracle.project_union(W, b, C, cand_off_f, cand_ids_f, H, k=6)
    ff = oracle.project_full(W, b, H, k=6)
    for key in ("ids", "logp", "z", "lse"):
        assert np.array_equal(uf[key], ff[key])


# ------------------------------------------------- workload generator (inputs)
def _read_golden(name):
    members, rows = [], {}
    with open(os.path.join(GOLD, name)) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            if key == "member":
                members.append([int(v) for v in vals])
            else:
                rows[key] = [int(v) for v in vals]
    return members, rows


def test_active_set_union_worked_example():
    members, rows = _read_golden("active_set_union.txt")
    assert list(wl.union_sorted(members)) == rows["union"]


def test_batch_union_worked_example():
    members, rows = _read_golden("batch_union.txt")
    u = wl.union_sorted(members)
    assert list(u) == rows["union"]
    flags = np.zeros(len(rows["flags"]), int)
    flags[u] = 1
    assert list(flags) == rows["flags"]


def test_generator_shapes_and_determinism():
    cfg = wl.scaled(wl.CONFIGS["tiny"], V=4000, K=6, n_samples=32, size_lo=300, size_hi=400,
                    n_global=50)
    W, b, C = wl.make_model(cfg)
    W2, b2, C2 = wl.make_model(cfg)
    assert W.dtype == np.float16 and W.shape == (cfg.d, cfg.V) and np.array_equal(W, W2)
    assert abs(float(W.astype(np.float64).std()) - 1 / np.sqrt(cfg.d)) < 1e-3
    assert abs(float(b.astype(np.float64).var()) - 0.1) < 0.01
    off, ids = wl.make_candidates(cfg, W, b, C)
    off2, ids2 = wl.make_candidates(cfg, W, b, C)
    assert np.array_equal(off, off2) and np.array_equal(ids, ids2)
    sizes = off[1:] - off[:-1]
    assert np.array_equal(sizes, wl.list_sizes(cfg))
    for j in range(cfg.K):
        a = ids[off[j]:off[j + 1]]
        assert np.all(np.diff(a) > 0) and a[0] >= 0 and a[-1] < cfg.V
    H, q = wl.make_rows(cfg, C)
    assert H.shape == (cfg.N, cfg.d) and H.dtype == np.float16


def test_generated_rows_land_in_their_cluster_and_top1_is_listed(oracle):
    """With noise 0.3 a row stays nearest to its own centroid, and the lists
    built from member predictions contain the full projection's best token
    for most rows (this is what makes the method an approximation that works)."""
    cfg = wl.scaled(wl.CONFIGS["tiny"], V=4000, K=6, N=24, n_samples=64, size_lo=300,
                    size_hi=400, n_global=50)
    W, b, C = wl.make_model(cfg)
    off, ids = wl.make_candidates(cfg, W, b, C)
    H, q = wl.make_rows(cfg, C)
    a = oracle.project(W, b, C, off, ids, H, k=1)
    f = oracle.project_full(W, b, H, k=1)
    assert np.array_equal(a["g"], q)
    agree = (a["ids"][:, 0] == f["ids"][:, 0]).mean()
    assert agree >= 0.75
    # and a clustered log-prob can only exceed the full one (smaller normaliser)
    same = a["ids"][:, 0] == f["ids"][:, 0]
    assert np.all(a["logp"][same, 0] >= f["logp"][same, 0] - 1e-12)


def test_zipf_rows():
    cfg = wl.scaled(wl.CONFIGS["skewed"], K=50, N=2000)
    q = wl.row_clusters(cfg, 2000)
    counts = np.sort(np.bincount(q, minlength=50))[::-1]
    assert counts[0] > 4 * counts[10] > 0
