"""The C ABI without Python in the way: examples/vp_cli (hipMalloc, vp_build, vp_project, vp_project_full,
built together with the library) runs as a program of its own; its output must match the CPU oracle."""
import os
import subprocess

import numpy as np
import pytest

from tests import parity_util as pu

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLI = os.path.join(ROOT, "examples", "vp_cli")


def test_stand_alone_caller_matches_the_oracle(oracle, tmp_path):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    assert os.path.exists(CLI), "examples/vp_cli is missing: run `python -m paper_2208_06874_amd.build`"
    r = np.random.default_rng(31)
    d, V, K, N, k = 264, 3001, 7, 45, 5
    W = (r.standard_normal((d, V)) / np.sqrt(d)).astype(np.float16)
    b = (r.standard_normal(V) * 0.3).astype(np.float16)
    C = r.standard_normal((K, d)).astype(np.float16)
    lists = [np.sort(r.choice(V, size=int(n), replace=False)) for n in r.integers(3, 700, K)]
    off = np.zeros(K + 1, np.int64)
    np.cumsum([len(x) for x in lists], out=off[1:])
    ids = np.concatenate(lists).astype(np.int32)
    H = (C[r.integers(0, K, N)].astype(np.float32) + 0.3 * r.standard_normal((N, d))).astype(np.float16)
    src, dst = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(src, "wb") as f:
        f.write(np.array([d, V, K, N, k], np.int32).tobytes())
        for a in (W, b, C, off, ids, H):
            f.write(np.ascontiguousarray(a).tobytes())
    run = subprocess.run([CLI, str(src), str(dst)], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    raw = np.fromfile(dst, np.uint8)
    nk = N * k * 4
    ids_g = raw[:nk].view(np.int32).reshape(N, k)
    logp_g = raw[nk:2 * nk].view(np.float32).reshape(N, k)
    g = raw[2 * nk:2 * nk + N * 4].view(np.int32)
    f_ids = raw[2 * nk + N * 4:3 * nk + N * 4].view(np.int32).reshape(N, k)
    f_logp = raw[3 * nk + N * 4:4 * nk + N * 4].view(np.float32).reshape(N, k)
    st = pu.check_projection(oracle, W, b, C, off, ids, H, k, ids_g, logp_g, g)
    sf = pu.check_full(oracle, W, b, H, k, f_ids, f_logp)
    print(run.stdout.strip(), st, sf)
