"""vp_project_static (the entry point for callers that cannot allocate: its scratch is an array inside
the library's device code) against vp_project on the same inputs, through the C ABI: two calls in a
row, the second with a smaller batch, so that what the first left in the shared array must not matter."""
import ctypes

import numpy as np
import pytest

from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _case(seed, d, V, K):
    r = np.random.default_rng(seed)
    W = (r.standard_normal((d, V)) / np.sqrt(d)).astype(np.float16)
    b = (r.standard_normal(V) * 0.3).astype(np.float16)
    C = r.standard_normal((K, d)).astype(np.float16)
    lists = [np.sort(r.choice(V, size=int(n), replace=False)) for n in r.integers(40, 900, K)]
    off = np.zeros(K + 1, np.int64)
    np.cumsum([len(x) for x in lists], out=off[1:])
    ids = np.concatenate(lists).astype(np.int32)
    return r, W, b, C, off, ids


def test_static_scratch_entry_matches_vp_project(oracle):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2208_06874_amd import vp
    dev = torch.device("cuda:0")
    r, W, b, C, off, ids = _case(77, 264, 5000, 23)
    index = vp.vp_build(torch.from_numpy(W).to(dev), torch.from_numpy(b).to(dev), torch.from_numpy(C).to(dev),
                        off, ids, k_max=8)
    L = vp.lib()
    K = C.shape[0]
    for N, k in ((150, 8), (9, 3)):          # the second call is smaller and finds the first one's leftovers
        H = (C[r.integers(0, K, N)].astype(np.float32) + 0.3 * r.standard_normal((N, C.shape[1]))).astype(np.float16)
        Ht = torch.from_numpy(H).to(dev)
        ref_ids, ref_logp, ref_g = vp.vp_project(index, Ht, k)
        out_ids = torch.full((N, k), -7, dtype=torch.int32, device=dev)
        out_logp = torch.full((N, k), float("nan"), dtype=torch.float32, device=dev)
        out_g = torch.full((N,), -7, dtype=torch.int32, device=dev)
        print("vp_project_static N=%d k=%d" % (N, k), flush=True)
        st = L.vp_project_static(index.handle, Ht.data_ptr(), N, k, out_ids.data_ptr(), out_logp.data_ptr(),
                                 out_g.data_ptr(), torch.cuda.current_stream().cuda_stream)
        assert st == vp.VP_OK, vp.last_error()
        torch.cuda.synchronize()
        assert np.array_equal(pu.to_np(out_g), pu.to_np(ref_g))
        assert np.array_equal(pu.to_np(out_ids), pu.to_np(ref_ids))
        assert np.array_equal(pu.to_np(out_logp), pu.to_np(ref_logp))
        # and both against the oracle, to the bar of every other parity test
        pu.check_projection(oracle, W, b, C, off, ids, H, k, pu.to_np(out_ids), pu.to_np(out_logp), pu.to_np(out_g))
    # sizes beyond the array are refused before anything is launched
    big = 65536
    assert vp.vp_workspace_bytes(index, big) > vp.STATIC_SCRATCH_BYTES
    st = L.vp_project_static(index.handle, Ht.data_ptr(), big, 1, out_ids.data_ptr(), out_logp.data_ptr(), None, None)
    assert st == vp.VP_ERR_WORKSPACE and "scratch" in vp.last_error()
    vp.vp_destroy(index)


def test_static_scratch_entry_replayed_from_a_graph():
    """What the entry point is for: a call that allocates nothing can be captured into a HIP graph.  Every
    replay, with other rows in the input buffer and eager calls in between, must equal vp_project."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2208_06874_amd import vp
    dev = torch.device("cuda:0")
    r, W, b, C, off, ids = _case(78, 512, 6000, 17)
    index = vp.vp_build(torch.from_numpy(W).to(dev), torch.from_numpy(b).to(dev), torch.from_numpy(C).to(dev),
                        off, ids, k_max=4)
    L = vp.lib()
    K, N, k = C.shape[0], 40, 4
    rows = [(C[r.integers(0, K, N)].astype(np.float32) + 0.3 * r.standard_normal((N, C.shape[1]))).astype(np.float16)
            for _ in range(2)]
    want = []
    for H in rows:
        o = vp.vp_project(index, torch.from_numpy(H).to(dev), k)
        torch.cuda.synchronize()
        want.append(tuple(pu.to_np(t).copy() for t in o))
    hbuf = torch.from_numpy(rows[0]).to(dev)
    out_ids = torch.empty((N, k), dtype=torch.int32, device=dev)
    out_logp = torch.empty((N, k), dtype=torch.float32, device=dev)
    out_g = torch.empty((N,), dtype=torch.int32, device=dev)

    def call():
        st = L.vp_project_static(index.handle, hbuf.data_ptr(), N, k, out_ids.data_ptr(), out_logp.data_ptr(),
                                 out_g.data_ptr(), torch.cuda.current_stream().cuda_stream)
        assert st == vp.VP_OK, vp.last_error()

    call()                                   # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for rep in range(4):
        j = rep % 2
        hbuf.copy_(torch.from_numpy(rows[j]).to(dev))
        out_ids.fill_(-7)
        out_logp.zero_()
        print("replay", rep, flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(pu.to_np(out_g), want[j][2])
        assert np.array_equal(pu.to_np(out_ids), want[j][0])
        assert np.array_equal(pu.to_np(out_logp), want[j][1])
        vp.vp_project(index, torch.from_numpy(rows[1 - j]).to(dev), k)   # eager work between replays
        torch.cuda.synchronize()
    del graph
    vp.vp_destroy(index)
