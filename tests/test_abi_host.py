"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects bad
arguments before touching a GPU.  CPU only."""
import ctypes as C
import os
import re

import pytest

from paper_2602_21780_amd import xsv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(xsv.LIB_PATH):
        from paper_2602_21780_amd.build import build
        build()
    return xsv.lib()


def test_every_declared_symbol_is_exported(lib):
    for header_name, exports in (("xsv.h", xsv.EXPORTS), ("xsv_tune.h", xsv.TUNE_EXPORTS)):
        header = open(os.path.join(ROOT, "include", header_name)).read()
        declared = set(re.findall(r"\b(xsv_[a-z_]+)\s*\(", header))
        assert declared == set(exports), header_name
        for name in declared:
            assert hasattr(lib, name), name


def test_strerror(lib):
    assert xsv.strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -5, -99):
        assert xsv.strerror(code)


def test_create_rejects_bad_configurations_on_the_host(lib):
    good = dict(n_layers=1, n_heads=2, head_dim=64, tokens_per_frame=64, n_special=5, budget=256, kv_bits=4,
                group_size=32, pool_size=16, score_mode=0, softmax_scale=0.0, max_frames=0, value_mode=0)
    def create(**kw):
        cfg = xsv.xsv_config(**{**good, **kw})
        h = C.c_void_p()
        return lib.xsv_create(C.byref(cfg), None, C.byref(h))
    assert create(n_layers=0) == xsv.XSV_ERR_ARG
    assert create(n_heads=0) == xsv.XSV_ERR_ARG
    assert create(kv_bits=3) == xsv.XSV_ERR_ARG
    assert create(budget=-1) == xsv.XSV_ERR_ARG
    assert create(n_special=65) == xsv.XSV_ERR_ARG
    assert create(pool_size=0) == xsv.XSV_ERR_ARG
    assert create(score_mode=2) == xsv.XSV_ERR_ARG
    assert create(value_mode=2) == xsv.XSV_ERR_ARG
    assert create(budget=0, max_frames=0) == xsv.XSV_ERR_ARG
    assert create(head_dim=128) == xsv.XSV_ERR_UNSUPPORTED
    assert create(group_size=16) == xsv.XSV_ERR_UNSUPPORTED
    assert lib.xsv_create(None, None, None) == xsv.XSV_ERR_ARG


def test_null_context_is_rejected(lib):
    t = xsv.xsv_tensor(None, 0, 0)
    assert lib.xsv_step(None, 0, t, t, t, None) == xsv.XSV_ERR_ARG
    assert lib.xsv_reset(None) == xsv.XSV_ERR_ARG
    assert lib.xsv_destroy(None) == xsv.XSV_OK
    assert lib.xsv_cache_len(None, 0, None) == xsv.XSV_ERR_ARG
    assert lib.xsv_quantize_k(None, None, 1, 1, 64, 4, 64, None, None, None) == xsv.XSV_ERR_ARG
    assert lib.xsv_topk_keep(None, None, 4, 5, 0, 0, None) == xsv.XSV_ERR_ARG
    assert lib.xsv_join(None) == xsv.XSV_ERR_ARG
    assert lib.xsv_measure_peaks(None, None, None) == xsv.XSV_ERR_ARG
    assert lib.xsv_frame_attend(None, t, t, t, None) == xsv.XSV_ERR_ARG
    assert lib.xsv_set_overlap(None, 1) == xsv.XSV_ERR_ARG
    assert lib.xsv_set_side_cus(None, 0) == xsv.XSV_ERR_ARG
    assert lib.xsv_set_short_range(None, 0) == xsv.XSV_ERR_ARG
    assert lib.xsv_set_attend_timing(None, 1) == xsv.XSV_ERR_ARG
    assert lib.xsv_attend_times(None, None, None, None, None) == xsv.XSV_ERR_ARG
    assert lib.xsv_chain_times(None, None, None, None) == xsv.XSV_ERR_ARG
    assert lib.xsv_last_attend_workgroups(None, None) == xsv.XSV_ERR_ARG


def test_header_compiles_as_c_and_every_entry_point_links(tmp_path):
    """A C99 program against include/xsv.h and libxsv.so (no GPU needed for what it calls)."""
    import os
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    exe = str(tmp_path / "abi_check")
    libdir = os.path.join(root, "paper_2602_21780_amd")
    cmd = [cc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(root, "include"),
           os.path.join(root, "tests", "c", "abi_check.c"), "-o", exe, "-L", libdir, "-lxsv", "-Wl,-rpath," + libdir,
           "-Wl,-rpath-link,/opt/rocm/lib"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0 and "abi ok" in r.stdout, (r.returncode, r.stdout, r.stderr)


def test_key_ranges_cover_the_tiles_with_equal_cost(lib):
    """The host routine that places the key ranges of an attention launch: the ranges tile [0, tiles) without gaps,
    none is empty, the full ranges cost the same to within one tile, and a short last range costs about its share."""
    import itertools
    for n_ct, n_ft, R, pct, fc in itertools.product((0, 1, 7, 64, 129, 1000), (1, 17, 22), (1, 2, 3, 5, 8, 16), (100, 50, 35, 1),
                                                    (25, 95, 100, 160, 400)):
        tiles = n_ct + n_ft
        if R > tiles:
            assert lib.xsv_key_ranges(n_ct, n_ft, R, pct, fc, (C.c_int32 * (R + 1))()) == xsv.XSV_ERR_ARG
            continue
        b = xsv.key_ranges(n_ct, n_ft, R, pct, fc)
        assert b[0] == 0 and b[-1] == tiles and all(x < y for x, y in zip(b, b[1:])), (n_ct, n_ft, R, pct, fc, b)
        cost = lambda t0, t1: sum(100 if t < n_ct else fc for t in range(t0, t1))
        costs = [cost(b[i], b[i + 1]) for i in range(R)]
        total = sum(costs)
        share = total * 100.0 / (100 * (R - 1) + pct)             # cost of a full range
        biggest = max(100, fc)
        if R > 1 and tiles >= 4 * R:                              # (with very few tiles "one tile each" takes over)
            # (a last range that must hold one whole tile although its share is smaller takes the excess from the others)
            slack = biggest + max(0.0, (100 if tiles - 1 < n_ct else fc) - share * pct / 100.0)
            for c in costs[:-1]:
                assert abs(c - share) <= slack, (n_ct, n_ft, R, pct, fc, b, costs)
            assert abs(costs[-1] - share * pct / 100.0) <= biggest * (R - 1) / 2 + biggest, (n_ct, n_ft, R, pct, fc, b, costs)
    # the benchmark's cut: 64 cache + 22 frame tiles, four long ranges and a half one
    b = xsv.key_ranges(64, 22, 5, 50, 95)
    assert b == sorted(b) and b[-1] == 86 and 17 <= b[1] <= 20 and b[4] - b[3] >= b[5] - b[4]
    for bad in ((-1, 5, 2, 100, 95), (5, 5, 0, 100, 95), (5, 5, 17, 100, 95), (5, 5, 2, 0, 95), (5, 5, 2, 101, 95), (5, 5, 2, 100, 24)):
        assert lib.xsv_key_ranges(*bad, (C.c_int32 * 18)()) == xsv.XSV_ERR_ARG


def test_line_partition_is_a_partition(lib):
    """The (unit, tile) line cut into workgroup pieces: the pieces tile the line in order, differ by at most one item,
    and the workgroups that touch a unit are exactly those whose piece overlaps it."""
    lib.xsv_line_partition.argtypes = [C.c_int64, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                       C.c_int64, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    for units, tiles, wgs in ((48, 86, 224), (48, 86, 256), (1152, 86, 256), (3, 1, 5), (7, 3, 4), (1, 1, 1), (5, 9, 45), (5, 9, 44)):
        b, e = C.c_int64(), C.c_int64()
        pieces = []
        for w in range(wgs):
            assert lib.xsv_line_partition(units, tiles, wgs, w, C.byref(b), C.byref(e), 0, None, None) == xsv.XSV_OK
            pieces.append((b.value, e.value))
        assert pieces[0][0] == 0 and pieces[-1][1] == units * tiles
        assert all(p[1] == q[0] for p, q in zip(pieces, pieces[1:]))
        sizes = [p[1] - p[0] for p in pieces]
        assert max(sizes) - min(sizes) <= 1 and min(sizes) >= 0
        f, l = C.c_int32(), C.c_int32()
        for u in range(units):
            assert lib.xsv_line_partition(units, tiles, wgs, 0, None, None, u, C.byref(f), C.byref(l)) == xsv.XSV_OK
            touching = [w for w, (p0, p1) in enumerate(pieces) if p0 < (u + 1) * tiles and p1 > u * tiles]
            assert (f.value, l.value) == (touching[0], touching[-1]), (units, tiles, wgs, u)
    assert lib.xsv_line_partition(0, 1, 1, 0, None, None, 0, None, None) == xsv.XSV_ERR_ARG
    assert lib.xsv_line_partition(4, 4, 4, 4, None, None, 0, None, None) == xsv.XSV_ERR_ARG


def test_step_plan_follows_the_oracles_cache_lengths(lib, ref):
    """The library's token counting against the oracle stepped on real frames: the same cache length after every step
    (64, 128, 192, 256, 256, .. at the tiny configuration), the same number of kept middle tokens, also where the
    budget is below two frames (k = 0) and without a budget."""
    import numpy as np
    from paper_2602_21780_amd.inputs import CONFIGS, FrameSource, to_u16
    for budget in (256, 200, 100, 0, 64 * 5 + 7):
        spec = CONFIGS[0].with_(budget=budget, n_heads=1)
        cfg = xsv.xsv_config(1, 1, 64, spec.tokens_per_frame, spec.n_special, budget, 4, 32, spec.pool_size, 0, 0.0, 9, 0)
        st = ref.RefStream(1, 1, 64, spec.tokens_per_frame, spec.n_special, budget, 4, 32, spec.pool_size)
        src = FrameSource(spec, "cpu", layers=[0])
        T = 0
        for f in range(8):
            q, k, v = (to_u16(t[0]) for t in src.frame(f))
            mid, keep, new = C.c_int32(), C.c_int32(), C.c_int32()
            assert lib.xsv_step_plan(C.byref(cfg), T, f, C.byref(mid), C.byref(keep), C.byref(new)) == xsv.XSV_OK
            _, T_ref = st.step(0, q, k, v, attend=False)
            assert new.value == T_ref, (budget, f, new.value, T_ref)
            n = spec.tokens_per_frame
            if mid.value:                                            # a pruning step: first + kept middle + current
                assert new.value == n + keep.value + n and mid.value == T + n - 2 * n
                assert keep.value == min(max(0, budget - 2 * n), mid.value)
            T = new.value
        if budget:
            assert T <= max(budget, 2 * spec.tokens_per_frame)
    assert lib.xsv_step_plan(None, 0, 0, None, None, None) == xsv.XSV_ERR_ARG
