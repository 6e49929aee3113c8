"""The static tile schedule of the join kernel, enumerated on the host (csrc/tile_cursor.h compiled with g++):
every tile of the triangle (self-join) or grid (two sets) exactly once, workgroups of an XCD balanced to within
one tile and, step by step, on at most two of the XCD's 8 x 4 rectangles."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def build_schedule(tmp_path_factory, kind):
    out = tmp_path_factory.mktemp("sched") / f"libsched_{kind}.so"
    cmd = ["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-I", os.path.join(ROOT, "paper_2508_21230_amd", "csrc"),
           os.path.join(ROOT, "tests", "host", "schedule_dump.cpp"), "-o", str(out)]
    if kind == "rowmajor_ablation":
        cmd.insert(1, "-DEJOIN_ABL_ROWMAJOR_TILES")
    if kind == "no_fast_path":
        cmd.insert(1, "-DEJOIN_CURSOR_NO_FAST_PATH")
    subprocess.run(cmd, check=True)
    lib = ctypes.CDLL(str(out))
    lib.ejoin_test_schedule.restype = ctypes.c_int64
    lib.ejoin_test_schedule.argtypes = [ctypes.c_uint32] * 4 + [ctypes.c_void_p, ctypes.c_int64]
    lib.ejoin_test_schedule_rows.restype = ctypes.c_int64
    lib.ejoin_test_schedule_rows.argtypes = [ctypes.c_uint32] * 6 + [ctypes.c_void_p, ctypes.c_int64]

    def run(nblocks, self_join, nt_a, nt_b):
        want = nt_a * (nt_a + 1) // 2 if self_join else nt_a * nt_b
        buf = np.zeros((want + 8, 4), dtype=np.uint32)
        m = lib.ejoin_test_schedule(nblocks, int(self_join), nt_a, nt_b, buf.ctypes.data, want + 8)
        return buf[:min(m, want + 8)], m, want
    def run_rows(nblocks, self_join, nt_a, nt_b, row_begin, row_end):
        want = nt_a * (nt_a + 1) // 2 if self_join else nt_a * nt_b
        buf = np.zeros((want + 8, 4), dtype=np.uint32)
        m = lib.ejoin_test_schedule_rows(nblocks, int(self_join), nt_a, nt_b, row_begin, row_end, buf.ctypes.data, want + 8)
        return buf[:min(m, want + 8)], m
    run.kind = kind
    run.rows = run_rows
    return run


@pytest.fixture(scope="module", params=["xcd_rectangles", "rowmajor_ablation"])
def sched(request, tmp_path_factory):
    return build_schedule(tmp_path_factory, request.param)


CASES = [(256, True, t, t) for t in (1, 2, 3, 15, 16, 17, 31, 32, 33, 40, 100, 391)] + \
        [(256, False, a, b) for a, b in ((1, 1), (1, 50), (50, 1), (7, 9), (16, 16), (17, 33), (391, 4), (4, 391), (100, 77))] + \
        [(8, True, 20, 20), (64, True, 45, 45), (304, True, 60, 60), (24, False, 30, 11), (250, True, 130, 130)]


@pytest.mark.parametrize("nblocks,self_join,nt_a,nt_b", CASES)
def test_every_tile_exactly_once(sched, nblocks, self_join, nt_a, nt_b):
    tiles, m, want = sched(nblocks, self_join, nt_a, nt_b)
    assert m == want
    I, J = tiles[:, 2].astype(np.int64), tiles[:, 3].astype(np.int64)
    assert (I < nt_a).all() and (J < nt_b).all()
    if self_join:
        assert (I <= J).all()
    keys = I * (nt_b + 1) + J
    assert np.unique(keys).size == want


@pytest.mark.parametrize("nblocks,self_join,nt_a,nt_b", [c for c in CASES if c[0] == 256])
def test_workgroups_of_an_xcd_stay_together(sched, nblocks, self_join, nt_a, nt_b):
    if sched.kind != "xcd_rectangles":
        pytest.skip("property of the XCD-aware schedule only")
    tiles, m, want = sched(nblocks, self_join, nt_a, nt_b)
    blk, step, I, J = (tiles[:, k].astype(np.int64) for k in range(4))
    xcd = blk % 8
    for x in range(8):
        sel = xcd == x
        counts = np.bincount(blk[sel] // 8, minlength=nblocks // 8)
        assert counts.max() - counts.min() <= 1, "tiles per workgroup of one XCD differ by more than one"
        for s in range(int(step[sel].max()) + 1 if sel.any() else 0):
            now = sel & (step == s)
            # the 8 x 4 rectangle a tile belongs to: (super-block, position inside it)
            rect = set(zip((I[now] // 8).tolist(), (J[now] // 4).tolist()))

            def full(r):  # all 32 cells of the rectangle are tiles of the problem
                i0, j0 = 8 * r[0], 4 * r[1]
                return i0 + 8 <= nt_a and j0 + 4 <= nt_b and (not self_join or i0 + 7 <= j0)
            # 32 consecutive entries of the XCD's list: one full rectangle, or the end of one and the start of the
            # next; partially empty rectangles (diagonal, ragged edge) hold fewer tiles, so more of them fit
            if all(full(r) for r in rect):
                assert len(rect) <= 2, f"XCD {x} step {s}: workgroups spread over {len(rect)} full rectangles"


@pytest.mark.parametrize("nblocks,self_join,nt_a,nt_b", CASES + [(256, True, 1000, 1000), (256, False, 700, 333), (256, True, 784, 784),
                                                                 (248, True, 500, 500), (256, False, 48, 1600)])
def test_fast_step_gives_the_same_sequence_as_the_general_step(tmp_path_factory, nblocks, self_join, nt_a, nt_b):
    """The cursor's shortcut for runs of complete rectangles is an optimisation only: workgroup by workgroup, step by
    step, it yields the tiles the general enumeration yields."""
    global _pair
    try:
        fast, slow = _pair
    except NameError:
        _pair = fast, slow = build_schedule(tmp_path_factory, "xcd_rectangles"), build_schedule(tmp_path_factory, "no_fast_path")
    a, ma, want = fast(nblocks, self_join, nt_a, nt_b)
    b, mb, _ = slow(nblocks, self_join, nt_a, nt_b)
    assert ma == mb == want
    assert np.array_equal(a, b)


@pytest.mark.parametrize("self_join,nt_a,nt_b,cuts", [(True, 100, 100, (0, 2, 3, 7)), (True, 391, 391, (0, 5, 11, 18, 25)), (False, 50, 77, (0, 1, 4)),
                                                     (True, 17, 17, (0, 1, 2)), (True, 40, 40, (0, 9))])
def test_launches_cut_by_rows_of_super_blocks_cover_every_tile_once(sched, self_join, nt_a, nt_b, cuts):
    """A join returned in batches runs one launch per range of super-block rows: the ranges' tiles are disjoint and
    together are all the tiles."""
    if sched.kind != "xcd_rectangles":
        pytest.skip("the row-major ablation enumerates the whole grid in one launch")
    want = nt_a * (nt_a + 1) // 2 if self_join else nt_a * nt_b
    bounds = list(cuts) + [0xFFFFFFFF]
    keys = []
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        tiles, m = sched.rows(256, self_join, nt_a, nt_b, lo, hi)
        I, J = tiles[:, 2].astype(np.int64), tiles[:, 3].astype(np.int64)
        assert m == len(tiles)
        assert ((I // 16 >= lo) & (I // 16 < hi)).all()
        keys.append(I * (nt_b + 1) + J)
    keys = np.concatenate(keys)
    assert keys.size == want and np.unique(keys).size == want
