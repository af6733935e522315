"""CPU-side checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments on the host before touching a GPU.
No compute call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2208_06874_amd import vp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "vp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vp_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert set(names) == set(vp.EXPORTS)
    L = vp.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_python_binding_has_the_same_names():
    import paper_2208_06874_amd as P
    for n in ("vp_build", "vp_project", "vp_project_full", "vp_project_debug_logits", "vp_workspace_bytes",
              "vp_set_option", "vp_get_info", "vp_get_profile", "vp_destroy", "vp_last_error", "vp_project_union",
              "vp_union_workspace_bytes", "vp_kmeans", "vp_kmeans_workspace_bytes", "vp_active_sets",
              "vp_active_sets_workspace_bytes", "vp_round_to_half", "vp_beam_step", "vp_project_static", "vp_measure_ceilings"):
        assert callable(getattr(P, n))


def _desc(d=64, V=100, K=3, lists=None, k_max=4, flags=0):
    if lists is None:
        lists = [np.arange(0, 40, 2), np.arange(5, 60), np.array([99])]
    off = np.zeros(len(lists) + 1, np.int64)
    np.cumsum([len(x) for x in lists], out=off[1:])
    ids = (np.concatenate(lists) if len(lists) else np.zeros(0)).astype(np.int32)
    desc = vp.make_desc(d, V, K, 0x1000, 0x1000, 0x1000, off, ids, None, 0, k_max, flags)
    return desc, off, ids   # keep the arrays alive


def test_build_bytes_valid_and_monotone():
    L = vp.lib()
    d1, *_k1 = _desc()
    n1 = L.vp_build_bytes(ctypes.byref(d1))
    assert n1 > 0 and n1 % 256 == 0
    d2, *_k2 = _desc(lists=[np.arange(0, 80), np.arange(5, 60), np.array([99])])
    assert L.vp_build_bytes(ctypes.byref(d2)) > n1
    # slab bytes: candidate groups of 16, d padded to 256, 2 bytes each
    info_groups = sum((len(x) + 15) // 16 for x in [np.arange(0, 40, 2), np.arange(5, 60), np.array([99])])
    assert n1 >= info_groups * 16 * 256 * 2 + ((100 + 15) // 16) * 16 * 256 * 2


@pytest.mark.parametrize("kw,status", [
    (dict(d=60), vp.VP_ERR_UNSUPPORTED),          # d % 8 != 0
    (dict(d=0), vp.VP_ERR_UNSUPPORTED),
    (dict(d=8192), vp.VP_ERR_UNSUPPORTED),
    (dict(K=0, lists=[]), vp.VP_ERR_UNSUPPORTED),
    (dict(k_max=0), vp.VP_ERR_UNSUPPORTED),
    (dict(k_max=33), vp.VP_ERR_UNSUPPORTED),
    (dict(flags=2), vp.VP_ERR_INVALID_ARG),            # an unknown flag bit
    (dict(lists=[np.zeros(0, int), np.zeros(0, int), np.zeros(0, int)]), vp.VP_ERR_UNSUPPORTED),   # all sets empty
    (dict(lists=[np.array([3, 2]), np.arange(4), np.arange(3)]), vp.VP_ERR_INVALID_ARG),   # unsorted
    (dict(lists=[np.array([2, 2]), np.arange(4), np.arange(3)]), vp.VP_ERR_INVALID_ARG),   # duplicate
    (dict(lists=[np.array([2, 100]), np.arange(4), np.arange(3)]), vp.VP_ERR_INVALID_ARG),  # id >= V
    (dict(lists=[np.array([-1, 4]), np.arange(4), np.arange(3)]), vp.VP_ERR_INVALID_ARG),  # id < 0
])
def test_build_rejects_bad_descriptions_on_the_host(kw, status):
    L = vp.lib()
    desc, *_keep = _desc(**kw)
    h = ctypes.c_void_p()
    st = L.vp_build(ctypes.byref(desc), None, ctypes.byref(h))
    assert st == status, vp.last_error()
    assert h.value is None
    assert vp.last_error() != ""


def test_build_rejects_null_and_small_arena_before_any_gpu_work():
    L = vp.lib()
    desc, *_keep = _desc()
    h = ctypes.c_void_p()
    assert L.vp_build(ctypes.byref(desc), None, ctypes.byref(h)) == vp.VP_ERR_INVALID_ARG   # null arena
    desc.arena = 0x100000
    desc.arena_bytes = 1024
    assert L.vp_build(ctypes.byref(desc), None, ctypes.byref(h)) == vp.VP_ERR_WORKSPACE
    desc.arena = 0x100010                      # misaligned
    desc.arena_bytes = 1 << 30
    assert L.vp_build(ctypes.byref(desc), None, ctypes.byref(h)) == vp.VP_ERR_INVALID_ARG
    desc.W = None
    desc.arena = 0x100000
    assert L.vp_build(ctypes.byref(desc), None, ctypes.byref(h)) == vp.VP_ERR_INVALID_ARG
    assert L.vp_build(None, None, ctypes.byref(h)) == vp.VP_ERR_INVALID_ARG
    assert L.vp_build_bytes(None) == 0


def test_calls_reject_null_index():
    L = vp.lib()
    assert L.vp_project(None, None, 1, 1, None, None, None, None, 0, None) == vp.VP_ERR_INVALID_ARG
    assert L.vp_project_full(None, None, 1, 1, None, None, None, 0, None) == vp.VP_ERR_INVALID_ARG
    assert L.vp_project_debug_logits(None, None, 1, 0, None, None, None, 0, None, 0, None) == vp.VP_ERR_INVALID_ARG
    assert L.vp_project_union(None, None, 1, 1, None, None, None, None, None, 0, None) == vp.VP_ERR_INVALID_ARG
    assert L.vp_union_workspace_bytes(None, 4) == 0
    assert L.vp_workspace_bytes(None, 4) == 0
    assert L.vp_set_option(None, b"rstar", 1) == vp.VP_ERR_INVALID_ARG
    assert L.vp_get_info(None, None) == vp.VP_ERR_INVALID_ARG
    assert L.vp_get_profile(None, None, None) == vp.VP_ERR_INVALID_ARG
    L.vp_destroy(None)   # no-op


def test_training_calls_reject_bad_arguments_on_the_host():
    L = vp.lib()
    assert L.vp_kmeans_workspace_bytes(1000, 64, 10) > 0
    assert L.vp_kmeans_workspace_bytes(1000, 60, 10) == 0        # d % 8
    assert L.vp_kmeans_workspace_bytes(0, 64, 10) == 0
    assert L.vp_kmeans_workspace_bytes(1000, 64, 5000) == 0
    assert L.vp_kmeans_workspace_bytes(2000, 64, 10) >= L.vp_kmeans_workspace_bytes(1000, 64, 10)
    assert L.vp_kmeans(None, 10, 64, 4, 1, 0, None, None, None, None, 0, None) == vp.VP_ERR_INVALID_ARG
    assert L.vp_kmeans(0x1000, 10, 64, 4, 1, 2, 0x1000, 0x1000, 0x1000, 0x1000, 1 << 30, None) == vp.VP_ERR_INVALID_ARG
    assert L.vp_kmeans(0x1000, 10, 64, 4, -1, 0, 0x1000, 0x1000, 0x1000, 0x1000, 1 << 30, None) == vp.VP_ERR_INVALID_ARG
    assert L.vp_kmeans(0x1000, 10, 64, 4, 1, 0, 0x1000, 0x1000, 0x1000, 0x1000, 16, None) == vp.VP_ERR_WORKSPACE
    assert "needed" in vp.last_error()
    assert L.vp_kmeans(0x1008, 10, 64, 4, 1, 0, 0x1000, 0x1000, 0x1000, 0x1000, 1 << 30, None) == vp.VP_ERR_INVALID_ARG
    assert L.vp_active_sets_workspace_bytes(4, 100) > 0
    assert L.vp_active_sets_workspace_bytes(0, 100) == 0
    tot = ctypes.c_int64(0)
    assert L.vp_active_sets(None, None, 5, 3, 4, 100, None, None, 0, ctypes.byref(tot), None, 0, None) == \
        vp.VP_ERR_INVALID_ARG
    assert L.vp_active_sets(0x1000, 0x1000, 5, 0, 4, 100, 0x1000, 0x1000, 8, ctypes.byref(tot), 0x1000, 1 << 20,
                            None) == vp.VP_ERR_INVALID_ARG
    assert L.vp_active_sets(0x1000, 0x1000, 5, 3, 4, 100, 0x1000, 0x1000, 8, ctypes.byref(tot), 0x1000, 16,
                            None) == vp.VP_ERR_WORKSPACE


def test_beam_step_rejects_bad_arguments_on_the_host():
    L = vp.lib()
    assert L.vp_beam_step(None, None, None, 2, 4, 4, None, None, None, None) == vp.VP_ERR_INVALID_ARG
    assert L.vp_beam_step(0x1000, 0x1000, 0x1000, 2, 128, 32, 0x1000, 0x1000, 0x1000, None) == vp.VP_ERR_UNSUPPORTED
    assert L.vp_beam_step(0x1000, 0x1000, 0x1000, 2, 0, 4, 0x1000, 0x1000, 0x1000, None) == vp.VP_ERR_UNSUPPORTED
    assert L.vp_beam_step(None, None, None, 0, 4, 4, None, None, None, None) == vp.VP_OK   # no sentences: no-op


def test_round_to_half_is_the_library_cast():
    """The host copy of the rounding vp_kmeans applies to a mean: every fp16 value, midpoints, random doubles."""
    pos = np.arange(0, 0x7c00, dtype=np.uint16)
    vals = pos.view(np.float16).astype(np.float64)
    for i in range(len(pos)):
        assert vp.vp_round_to_half(vals[i]) == int(pos[i])
        assert vp.vp_round_to_half(-vals[i]) == int(pos[i]) | 0x8000
    mids = 0.5 * (vals[:-1] + vals[1:])
    r = np.random.default_rng(0)
    v = np.concatenate([mids, -mids, np.nextafter(mids, np.inf), np.nextafter(mids, -np.inf),
                        r.standard_normal(20000), r.standard_normal(5000) * 1e-6, r.standard_normal(5000) * 3e4,
                        r.standard_normal(1000) * 1e-9, r.standard_normal(1000) * 1e6, [65519.9, 65520.0, 1e300, 0.0]])
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    got = np.array([vp.vp_round_to_half(x) for x in v], np.uint16)
    assert np.array_equal(got, want)


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(vp, "_lib", None)
    monkeypatch.setattr(vp, "LIB_PATH", str(tmp_path / "libvp.so"))
    with pytest.raises(RuntimeError, match="missing"):
        vp.lib()


def test_product_path_does_not_reach_the_oracle():
    """Nothing under the package may import or name the oracle."""
    pkg = os.path.join(ROOT, "paper_2208_06874_amd")
    for base, _dirs, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(base, f)).read()
                assert "vp_oracle" not in text and "import oracle" not in text and "from oracle" not in text, f


# ------------------------------------------------------------------ host logic: how a projection is cut into work items
@pytest.fixture(scope="module")
def layout(tmp_path_factory):
    import subprocess
    out = tmp_path_factory.mktemp("layout") / "liblayout_shim.so"
    src = os.path.join(ROOT, "tests", "layout_shim.cpp")
    inc = os.path.join(ROOT, "paper_2208_06874_amd", "csrc")
    subprocess.run(["g++", "-O1", "-shared", "-fPIC", "-I", inc, src, "-o", str(out)], check=True)
    L = ctypes.CDLL(str(out))
    L.shim_tiles_per_wave.argtypes = [ctypes.c_longlong, ctypes.c_int, ctypes.c_int]
    L.shim_tiles_per_wave_units.argtypes = [ctypes.c_longlong, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    return L


def test_item_sizing_rules(layout):
    """Tiles per wavefront of a plan: at least 1; never more items than asked for; with little work at least
    one item per resident workgroup slot while items stay >= 4 tiles per wavefront; the clustered variant
    never shortens items and, when it lengthens them, the plan fits one round of workgroup slots."""
    r = np.random.default_rng(5)
    for target, min_items in ((8192, 1024), (2048, 1024), (512, 512), (8192, 768)):
        for total in [1, 3, 16, 4095, 4096, 4097, 8192, 15625, 16384, 16385, 60800, 250000, 10 ** 7] + \
                     [int(x) for x in r.integers(1, 400000, 60)]:
            tpw = layout.shim_tiles_per_wave(total, target, min_items)
            assert tpw >= 1
            items = -(-total // (4 * tpw))
            assert items <= max(target, min_items)
            if total >= 16 * max(target, min_items):          # plenty of work: about `target` items
                assert items > max(target, min_items) // 2
            if total <= 16 * min_items and min_items <= target:   # little work: one item per slot, or short items
                assert tpw <= max(1, -(-total // (4 * min_items)))
            for units in (1, 2, 17, 200, 600, 5000):
                t2 = layout.shim_tiles_per_wave_units(total, units, target, min_items)
                assert t2 >= tpw
                if t2 > tpw:
                    ub_before = -(-total // (4 * tpw)) + units
                    assert min_items < ub_before <= 2 * min_items and 2 * units < min_items
                    assert -(-total // (4 * t2)) + units <= min_items + 1


def test_round_filling_item_count_of_the_many_row_kernel(layout):
    """Items of the kernel that runs one workgroup per compute unit: a whole number of candidate ranges per
    row group, at least one; at most eight rounds of the slots (unless there are more row groups than that);
    the plan the planning kernels then make (tiles per wavefront from that count) has no more items than
    asked for; and no choice of fewer rounds would have filled its rounds better."""
    r = np.random.default_rng(9)
    cases = [(1, 256, 15625), (4, 256, 15625), (16, 256, 15625), (86, 256, 15625), (6, 256, 15625), (1024, 256, 15625),
             (3000, 256, 15625), (5, 256, 3), (86, 304, 8000)]
    cases += [(int(a), int(b), int(c)) for a, b, c in zip(r.integers(1, 1500, 200), r.choice([64, 104, 256, 304], 200),
                                                           r.integers(1, 40000, 200))]
    for rgs, slots, vtiles in cases:
        items = layout.shim_rounds_item_count(rgs, slots, vtiles)
        assert items >= rgs and items % rgs == 0
        ranges = items // rgs
        assert ranges <= max(1, vtiles)
        assert items <= 8 * slots or ranges == 1
        # what the planning kernels make of it: ranges of 4 * tpw tiles
        tpw = layout.shim_tiles_per_wave(rgs * vtiles, items, items)
        chunks = -(-vtiles // (4 * tpw))
        assert chunks * rgs <= items
        fill = items / (-(-items // slots) * slots)
        for rounds in range(1, 9):
            rg2 = min(rounds * slots // rgs, vtiles)
            if rg2 < 1:
                continue
            it2 = rgs * rg2
            f2 = it2 / (-(-it2 // slots) * slots)
            assert f2 <= fill + 1e-9 or fill > 0.97, (rgs, slots, vtiles, items, rounds)
            if f2 > 0.97:
                break


def test_short_items_bound_of_the_raw_logit_form(layout):
    """The host considers raw logits only for calls of at most 8,192 candidate tiles.  With the default
    sizing (8,192 items asked for, 1,024 workgroup slots) such a plan has at most VP_RAW_TILES tiles per
    wavefront unless its (bucket, row group) units push it just past one round of workgroups, in which case
    the items get longer and the kernel, which checks the plan's figure, keeps its lists."""
    raw = layout.shim_raw_tiles()
    longer = 0
    for total in list(range(1, 8193, 7)) + [8192]:
        for units in (1, 4, 16, 64):
            tpw = layout.shim_tiles_per_wave_units(total, units, 8192, 1024)
            if total + 8 * units <= 8192:
                assert tpw <= raw
            else:
                assert tpw <= raw + 1
                longer += tpw > raw
    assert longer > 0
    assert layout.shim_tiles_per_wave_units(8193 + 4096, 1, 8192, 1024) > raw
    assert layout.shim_partial_floats(8) == 18


def test_workgroup_to_item_maps_take_every_item_once(layout):
    """The two XCD-aware orders in which workgroups take work items: over a grid of the size the host
    launches, every item is taken by exactly one workgroup and no workgroup gets an item outside the list."""
    B = layout.shim_xcd_block_items()
    r = np.random.default_rng(11)
    # clustered plans with heavy buckets: blocks of B consecutive items dealt to the XCDs, rotated starts
    for total in [1, 2, 31, 32, 33, 255, 256, 257, 1000, 2047, 2048, 2049, 8466] + [int(x) for x in r.integers(1, 20000, 40)]:
        grid = total + 8 * B
        got = [layout.shim_item_of_workgroup(wg, total, -B, 0) for wg in range(grid)]
        taken = sorted(x for x in got if x >= 0)
        assert taken == list(range(total)), total
        assert all(x == -1 or 0 <= x < total for x in got)
    # single bucket, several row groups: candidate ranges dealt to the XCDs, a range's row groups together
    for rgs in (2, 3, 4, 16, 64):
        for chunks in (8, 9, 15, 16, 17, 100, 977):
            grid = -(-chunks // 8) * 8 * rgs
            got = [layout.shim_item_of_workgroup(wg, chunks * rgs, rgs, chunks) for wg in range(grid)]
            assert sorted(x for x in got if x >= 0) == list(range(chunks * rgs)), (rgs, chunks)
            # the row groups of one range run on one XCD
            for wg, it in enumerate(got):
                if it >= 0:
                    assert (it // rgs) % 8 == wg % 8
    # no swizzle
    assert [layout.shim_item_of_workgroup(wg, 10, 0, 0) for wg in range(10)] == list(range(10))


def _fake_index(d=64, k_max=4):
    """An Index object without a library handle: the binding's own checks run before any C call."""
    import torch
    idx = vp.Index.__new__(vp.Index)
    idx.handle = None
    idx.device = torch.device("cuda:0")
    idx.d, idx.V, idx.K, idx.k_max = d, 100, 3, k_max
    idx._ws, idx._uws = {}, {}
    return idx


def test_binding_rejects_host_tensors_and_wrong_shapes_before_any_c_call():
    """A CPU tensor, a strided view or an output of the wrong size would hand the kernels a host pointer or
    a short buffer: the binding raises first (handle is None here, so reaching the C call would fail differently)."""
    import torch
    idx = _fake_index()
    H = torch.zeros((5, 64), dtype=torch.float16)            # host memory
    for call in (lambda: idx.project(H, 2), lambda: idx.project_full(H, 2), lambda: idx.project_union(H, 2),
                 lambda: idx.debug_logits(H),
                 lambda: idx.project_static(H, 2, torch.zeros((5, 2), dtype=torch.int32),
                                            torch.zeros((5, 2), dtype=torch.float32))):
        with pytest.raises(ValueError, match="GPU memory"):
            call()
    with pytest.raises(ValueError, match="hidden must be"):
        idx.project(torch.zeros(64, dtype=torch.float16), 2)
    with pytest.raises(ValueError, match="shape"):
        idx.project(torch.zeros((5, 32), dtype=torch.float16), 2)
    # the checks themselves, on tensors that claim nothing about the GPU
    t = torch.zeros((4, 6), dtype=torch.float32)
    with pytest.raises(ValueError, match="GPU memory"):
        vp._want(t, "t", torch.float32)
    with pytest.raises(TypeError):
        vp._want([1, 2], "t", torch.float32)
    with pytest.raises(ValueError, match="required"):
        vp._want(None, "t", torch.float32)
    assert vp._want(None, "t", torch.float32, optional=True) is None
    with pytest.raises(ValueError, match="contiguous"):
        vp._want(t.t(), "t", torch.float32)
    with pytest.raises(ValueError, match="float16"):
        idx.project(torch.zeros((5, 64), dtype=torch.float32), 2)


def test_build_rejects_bad_tensors_before_any_c_call():
    import torch
    W = torch.zeros((64, 100), dtype=torch.float16)
    b = torch.zeros(100, dtype=torch.float16)
    C = torch.zeros((3, 64), dtype=torch.float16)
    off = np.array([0, 1, 2, 3], np.int64)
    ids = np.array([0, 1, 2], np.int32)
    with pytest.raises(ValueError, match="GPU memory"):
        vp.Index(W, b, C, off, ids)
    with pytest.raises(ValueError, match="W must be"):
        vp.Index(b, b, C, off, ids)
    with pytest.raises(ValueError, match="centroids must be"):
        vp.Index(W, b, torch.zeros((3, 32), dtype=torch.float16), off, ids)
    for fn in (lambda: vp.vp_kmeans(W, C), lambda: vp.vp_active_sets(torch.zeros((4, 2), dtype=torch.int32),
                                                                      torch.zeros(4, dtype=torch.int32), 3, 100),
               lambda: vp.vp_beam_step(torch.zeros((4, 2), dtype=torch.int32), torch.zeros((4, 2)), torch.zeros(4), 2)):
        with pytest.raises(ValueError, match="GPU memory"):
            fn()


def test_build_flag_drops_the_token_major_copy():
    """VP_BUILD_NO_UNION: the arena shrinks by V * d_pad * 2 bytes; other flag bits are refused."""
    L = vp.lib()
    d0, *_k0 = _desc()
    d1, *_k1 = _desc(flags=vp.BUILD_NO_UNION)
    n0, n1 = L.vp_build_bytes(ctypes.byref(d0)), L.vp_build_bytes(ctypes.byref(d1))
    assert n0 - n1 >= 100 * 256 * 2 and n1 > 0
    d2, *_k2 = _desc(flags=2)
    assert L.vp_build_bytes(ctypes.byref(d2)) == 0 and "flag" in vp.last_error()
