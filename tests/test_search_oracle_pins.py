"""Pins of the beam-step oracle (the toy search consumer; paper, section 2.1: the sorted probabilities
feed beam search / greedy search) against a hand-computed step, numpy's lexsort, the greedy special
case and the tie rule.  No GPU, no HIP library."""
import numpy as np


def _brute(cand_ids, cand_logp, scores, B):
    n, k = cand_ids.shape
    S = n // B
    out_s = np.full(n, -np.inf, np.float32)
    out_p = np.full(n, -1, np.int32)
    out_t = np.full(n, -1, np.int32)
    for s in range(S):
        rows = []
        for b in range(B):
            for j in range(k):
                if cand_ids[s * B + b, j] >= 0:
                    rows.append((np.float32(scores[s * B + b]) + np.float32(cand_logp[s * B + b, j]), b, j))
        if not rows:
            continue
        sums = np.array([r[0] for r in rows], np.float32)
        bs = np.array([r[1] for r in rows])
        js = np.array([r[2] for r in rows])
        order = np.lexsort((js, bs, -sums.astype(np.float64)))
        t = 0
        for i in order[:B]:
            if not np.isfinite(sums[i]) and sums[i] < 0:
                break
            out_s[s * B + t], out_p[s * B + t], out_t[s * B + t] = sums[i], bs[i], cand_ids[s * B + bs[i], js[i]]
            t += 1
    return out_s, out_p, out_t


def test_hand_computed_step(oracle):
    # one sentence, 2 hypotheses with scores -1 and -2, 3 candidates each
    ids = np.array([[7, 3, 9], [4, 7, -1]], np.int32)
    lp = np.array([[-0.5, -1.5, -3.0], [-0.25, -2.0, 0.0]], np.float32)
    sc = np.array([-1.0, -2.0], np.float32)
    s, p, t = oracle.beam_step(ids, lp, sc, B=2)
    # sums: (0,0) -1.5, (0,1) -2.5, (0,2) -4, (1,0) -2.25, (1,1) -4, (1,2) does not exist
    assert s.tolist() == [-1.5, -2.25] and p.tolist() == [0, 1] and t.tolist() == [7, 4]


def test_matches_lexsort_on_random_inputs(oracle):
    r = np.random.default_rng(5)
    for S, B, k in ((3, 4, 5), (1, 1, 8), (7, 8, 8), (2, 16, 3), (5, 2, 1)):
        n = S * B
        ids = r.integers(0, 1000, (n, k)).astype(np.int32)
        ids[r.random((n, k)) < 0.1] = -1
        lp = np.round(-r.random((n, k)).astype(np.float32) * 8, 2)   # rounding makes equal sums likely
        sc = np.round(-r.random(n).astype(np.float32) * 4, 2)
        sc[r.random(n) < 0.15] = -np.inf                               # dead hypotheses
        got = oracle.beam_step(ids, lp, sc, B)
        want = _brute(ids, lp, sc, B)
        for g, w in zip(got, want):
            assert np.array_equal(g, w)


def test_greedy_is_the_best_candidate(oracle):
    ids = np.array([[5, 2, 8], [1, 0, 3]], np.int32)
    lp = np.array([[-0.1, -0.1, -2.0], [-3.0, -1.0, -1.0]], np.float32)
    s, p, t = oracle.beam_step(ids, lp, np.zeros(2, np.float32), B=1)
    assert t.tolist() == [5, 0] and p.tolist() == [0, 0]           # ties go to the earlier candidate
    assert np.array_equal(s, np.array([-0.1, -1.0], np.float32))


def test_ties_and_missing_hypotheses(oracle):
    ids = np.array([[1, 2], [3, 4], [-1, -1]], np.int32)
    lp = np.zeros((3, 2), np.float32)
    sc = np.array([-1.0, -1.0, 0.0], np.float32)
    s, p, t = oracle.beam_step(ids, lp, sc, B=3)
    assert p.tolist() == [0, 0, 1] and t.tolist() == [1, 2, 3]       # equal sums: hypothesis, then rank
    sc2 = np.array([0.0, -np.inf, -np.inf], np.float32)               # first step of a search: one live hypothesis
    s, p, t = oracle.beam_step(ids, lp, sc2, B=3)
    assert p.tolist() == [0, 0, -1] and t.tolist() == [1, 2, -1] and s[2] == -np.inf
