"""The LDS / packed-copy arrangement of an operand panel (csrc/panel_layout.h compiled with g++): a bijection
inside every group of 32 points, and such that the 16 bytes lane l reads for fragment t are what the operand
layout of v_mfma_f32_16x16x32_f16 wants there: point 16 t + l % 16, coordinates 8 (l / 16) .. + 7.
Also the index algebra of the augmentation step: a 32x32x16 MFMA on the registers of four 16x16 blocks, fed
with the operands of panel_layout.h, adds to every register the two norm terms of the pair it stands for.
The operand and result layouts of the two instructions are taken from AMD's CDNA ISA documentation (the GPU
parity tests are what confirms them on the device)."""
import ctypes
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", params=["swizzled", "no_swizzle_ablation"])
def lay(request, tmp_path_factory):
    out = tmp_path_factory.mktemp("layout") / f"liblayout_{request.param}.so"
    cmd = ["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-I", os.path.join(ROOT, "paper_2508_21230_amd", "csrc"),
           os.path.join(ROOT, "tests", "host", "layout_dump.cpp"), "-o", str(out)]
    if request.param == "no_swizzle_ablation":
        cmd.insert(1, "-DEJOIN_ABL_NOSWIZZLE")
    subprocess.run(cmd, check=True)
    lib = ctypes.CDLL(str(out))
    lib.ejoin_test_stored_at.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32)]
    lib.ejoin_test_stored_at.restype = None
    lib.ejoin_test_place_of.argtypes = [ctypes.c_int64, ctypes.c_int32]
    lib.ejoin_test_place_of.restype = ctypes.c_int64
    lib.ejoin_test_fragment_offset.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.ejoin_test_fragment_offset.restype = ctypes.c_uint32
    for f in (lib.ejoin_test_aug_lds_offset_a, lib.ejoin_test_aug_lds_offset_b):
        f.argtypes = [ctypes.c_int32, ctypes.c_int32]
        f.restype = ctypes.c_uint32

    def stored_at(row, p):
        point, chunk = ctypes.c_int64(), ctypes.c_int32()
        lib.ejoin_test_stored_at(row, p, ctypes.byref(point), ctypes.byref(chunk))
        return point.value, chunk.value
    lib.stored_at = stored_at
    lib.kind = request.param
    return lib


def test_every_chunk_of_every_point_has_exactly_one_place(lay):
    for base in (0, 256, 5 * 256):  # the arrangement repeats per 256-row panel (and per group of 32)
        seen = set()
        for row in range(base, base + 256):
            for p in range(4):
                point, chunk = lay.stored_at(row, p)
                assert point // 32 == row // 32 and 0 <= chunk < 4
                assert lay.ejoin_test_place_of(point, chunk) == row * 4 + p
                seen.add((point, chunk))
        assert seen == {(pt, c) for pt in range(base, base + 256) for c in range(4)}


def test_a_fragment_read_is_the_mfma_operand(lay):
    for t in range(16):  # the 16 fragments of a 256-point panel
        for lane in range(64):
            off = lay.ejoin_test_fragment_offset(lane, t)
            assert off % 16 == 0 and off < 256 * 64
            point, chunk = lay.stored_at(off // 64, (off % 64) // 16)
            assert (point, chunk) == (16 * t + lane % 16, lane // 16)
            assert off == lay.ejoin_test_fragment_offset(lane, t % 2) + (t // 2) * 2048


def test_sixteen_consecutive_lanes_of_a_read_hit_sixteen_bank_groups(lay):
    """What the swizzle is for: lanes 16 q .. 16 q + 15 of a fragment read touch every 16-byte bank group once."""
    if lay.kind != "swizzled":
        pytest.skip("the ablation build stores rows unpermuted")
    for t in range(2):
        for q in range(4):
            groups = {(lay.ejoin_test_fragment_offset(lane, t) % 256) // 16 for lane in range(16 * q, 16 * q + 16)}
            assert len(groups) == 16


def test_the_augmentation_step_adds_each_register_its_own_pairs_norm_terms(lay):
    """Integer stand-ins for the pieces: P(x) = (a_x, b_x, c_x, 0), C = (7, 7, 7, 0).  The step must add
    7 (a + b + c)_i + 7 (a + b + c)_j to the register that holds pair (i, j) of the 32 x 32 region."""
    import numpy as np
    rng = np.random.default_rng(5)
    P = np.zeros((32, 4), dtype=np.int64)
    Q = np.zeros((32, 4), dtype=np.int64)     # the other set's points (two-set join); same layout
    P[:, :3] = rng.integers(-1000, 1000, size=(32, 3))
    Q[:, :3] = rng.integers(-1000, 1000, size=(32, 3))
    C = np.array([7, 7, 7, 0], dtype=np.int64)
    Z = np.zeros(4, dtype=np.int64)

    def rows(pieces):  # the four chunks of every row of a group's augmentation block, 8 numbers each
        out = np.zeros((32, 4, 8), dtype=np.int64)
        for m in range(32):
            x, y = lay.ejoin_test_aug_row_point(m), lay.ejoin_test_aug_col_point(m)
            out[m, 0] = np.concatenate([pieces[x], pieces[x + 4]])
            out[m, 1] = np.concatenate([pieces[y], pieces[y + 16]])
            out[m, 2] = np.concatenate([C, Z])
            out[m, 3] = np.concatenate([Z, C])
        return out
    blockA, blockB = rows(P), rows(Q)
    # operands of v_mfma_f32_32x32x16_f16: lane l supplies row (column) l % 32, k = 8 (l / 32) .. + 7
    A = np.zeros((32, 16), dtype=np.int64)
    B = np.zeros((32, 16), dtype=np.int64)
    for lane in range(64):
        m, k0 = lane % 32, 8 * (lane // 32)
        A[m, k0:k0 + 8] = blockA[m, lay.ejoin_test_aug_chunk_a(lane)]
        B[m, k0:k0 + 8] = blockB[m, lay.ejoin_test_aug_chunk_b(lane)]
    D = A @ B.T
    assert (np.count_nonzero(A[:, None, :] * B[None, :, :], axis=2) <= 6).all()
    seen = set()
    for lane in range(64):
        for q in range(16):
            i, j, m, n = (ctypes.c_int32() for _ in range(4))
            lay.ejoin_test_region_pair(lane, q, ctypes.byref(i), ctypes.byref(j))
            lay.ejoin_test_mfma32_element(lane, q, ctypes.byref(m), ctypes.byref(n))
            assert D[m.value, n.value] == 7 * P[i.value].sum() + 7 * Q[j.value].sum()
            seen.add((i.value, j.value))
    assert len(seen) == 32 * 32  # every pair of the region in exactly one register


def test_the_augmentation_buffer_hands_every_lane_the_chunk_its_operand_needs(lay):
    """The join kernel copies units 0..255 of the row panel's augmentation block and units 256..511 of the column
    panel's to the LDS and keeps the two constant chunks beside them; for every wave tile (rows 128 wm .., columns
    64 wn ..), region t and lane, the 16 bytes at the operand's address must be the chunk the step's operand layout
    asks for (chunk aug_chunk_a / aug_chunk_b of row / column 32 t + lane % 32 of the wave tile)."""
    part, const, step, size = (lay.ejoin_test_aug_const(k) for k in range(4))
    units = {}  # byte offset in the buffer -> what the 16 bytes there are
    for r in range(256):
        ua, ub = lay.ejoin_test_aug_block_unit(r, 0), lay.ejoin_test_aug_block_unit(r, 1)
        assert 0 <= ua < 256 and 256 <= ub < 512  # the first 4 KB and the second 4 KB of the block: what is copied
        units[16 * ua] = ("rowpanel", r, 0)                 # A part: the row panel's units 0..255 land at byte 0
        units[part + 16 * (ub - 256)] = ("colpanel", r, 1)  # B part: the column panel's units 256..511 land at `part`
    for t in range(4):
        units[const + step * t] = ("const", 2)
        units[const + step * t + 16] = ("const", 3)
    assert len(units) == 512 + 8 and max(units) + 16 <= size
    for wm in range(2):
        for wn in range(4):
            for lane in range(64):
                ca, cb = lay.ejoin_test_aug_chunk_a(lane), lay.ejoin_test_aug_chunk_b(lane)
                for t in range(4):
                    got = units[lay.ejoin_test_aug_lds_offset_a(lane, 128 * wm) + step * t]
                    assert got == (("rowpanel", 128 * wm + 32 * t + lane % 32, 0) if ca == 0 else ("const", ca))
                for t in range(2):
                    got = units[lay.ejoin_test_aug_lds_offset_b(lane, 64 * wn) + step * t]
                    assert got == (("colpanel", 64 * wn + 32 * t + lane % 32, 1) if cb == 1 else ("const", cb))
    # 32 consecutive lanes of a data read cover 512 contiguous bytes (no bank conflict); the other 32 read one constant
    offs = [lay.ejoin_test_aug_lds_offset_a(lane, 128) for lane in range(32)]
    assert offs == list(range(offs[0], offs[0] + 512, 16))
