"""GPU parity of the toy search consumer (vp_beam_step) against the CPU oracle, bit for bit, and a short
decode loop in which every step's projection and beam step are checked."""
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


def _gpu_step(ids, lp, sc, B):
    torch = _torch()
    from paper_2208_06874_amd import vp
    out = vp.vp_beam_step(_dev(ids), _dev(lp), _dev(sc), B)
    torch.cuda.synchronize()
    return tuple(pu.to_np(o) for o in out)


@pytest.mark.parametrize("S,B,k", [(3, 4, 5), (1, 1, 8), (64, 8, 8), (2, 64, 32), (5, 2, 1), (7, 33, 3), (1, 1, 1)])
def test_beam_step_matches_the_oracle(oracle, S, B, k):
    r = np.random.default_rng(100 * S + 10 * B + k)
    n = S * B
    ids = r.integers(0, 250000, (n, k)).astype(np.int32)
    ids[r.random((n, k)) < 0.1] = -1
    lp = np.round(-r.random((n, k)).astype(np.float32) * 8, 1)      # coarse values: many equal sums
    sc = np.round(-r.random(n).astype(np.float32) * 4, 1)
    sc[r.random(n) < 0.15] = -np.inf
    got = _gpu_step(ids, lp, sc, B)
    want = oracle.beam_step(ids, lp, sc, B)
    for g, w, name in zip(got, want, ("scores", "parents", "tokens")):
        assert np.array_equal(g, w), name


def test_beam_step_edge_cases(oracle):
    # first step of a search (one live hypothesis), nothing alive at all, fewer continuations than B
    ids = np.array([[1, 2], [3, 4], [5, 6]], np.int32)
    lp = np.array([[-1, -2], [-0.5, -0.6], [-0.1, -0.2]], np.float32)
    for sc in ([0, -np.inf, -np.inf], [-np.inf] * 3, [0, 0, 0]):
        sc = np.array(sc, np.float32)
        got = _gpu_step(ids, lp, sc, 3)
        want = oracle.beam_step(ids, lp, sc, 3)
        for g, w in zip(got, want):
            assert np.array_equal(g, w)
    none = np.full((3, 2), -1, np.int32)
    got = _gpu_step(none, lp, np.zeros(3, np.float32), 3)
    assert np.all(got[1] == -1) and np.all(got[2] == -1) and np.all(np.isneginf(got[0]))


def test_decode_loop(oracle):
    """Five decode steps of 4 sentences x beam 4 on the tiny workload: project the hypotheses' hidden rows,
    take a beam step, carry every surviving hypothesis' row slot on to the next step's rows."""
    torch = _torch()
    from paper_2208_06874_amd import vp
    cfg = wl.CONFIGS["tiny"]
    W, b, C = wl.make_model(cfg)
    off, ids = wl.make_candidates(cfg, W, b, C, device="cuda:0")
    index = vp.vp_build(_dev(W), _dev(b), _dev(C), off, ids, k_max=8)
    S, B, k = 4, 4, 4
    scores = np.tile(np.array([0.0] + [-np.inf] * (B - 1), np.float32), S)
    parent = np.tile(np.arange(B, dtype=np.int32), S)
    for step in range(5):
        # toy model: the next hidden row of a hypothesis is a fresh row of the mixture in its parent's slot
        fresh, _ = wl.make_rows(cfg, C, N=S * B, stream=200 + step)
        gather = (np.arange(S * B) // B) * B + np.maximum(parent, 0)
        H = np.ascontiguousarray(fresh[gather])
        out_ids, out_logp, g = index.project(_dev(H), k)
        torch.cuda.synchronize()
        pu.check_projection(oracle, W, b, C, off, ids, H, k, pu.to_np(out_ids), pu.to_np(out_logp), pu.to_np(g))
        new = vp.vp_beam_step(out_ids, out_logp, _dev(scores), B)
        torch.cuda.synchronize()
        got = tuple(pu.to_np(o) for o in new)
        want = oracle.beam_step(pu.to_np(out_ids), pu.to_np(out_logp), scores, B)
        for a, w in zip(got, want):
            assert np.array_equal(a, w)
        scores, parent = got[0], got[1]
        assert np.all(np.diff(scores.reshape(S, B), axis=1) <= 0)       # hypotheses stay sorted
        alive = int(np.isfinite(scores).sum())
        assert alive == S * min(B, k ** (step + 1))
    print("decode loop: final scores of sentence 0", scores[:B])
