"""The parity checkers themselves, on the CPU: with the oracle's own result in the place of the GPU's they
pass, and a planted mistake (a dropped pair, an extra pair, a shifted squared distance) outside the boundary
band makes them fail.  Also: neighbour lists cut down from a larger epsilon equal the lists computed directly."""
import numpy as np
import pytest

import datagen
from oracle import oracle as orc
from tests import parity
from tests.fullsize import cut_to_eps


@pytest.fixture(scope="module")
def case():
    n, eps = 3000, 0.8
    P = orc.decode(datagen.generate(2, n=n))
    pairs, d2 = orc.selfjoin_pairs(P, eps)
    q = datagen.query_rows(2, 200, n=n)
    rs, nbr, nd2 = orc.rows_join(P, eps, q)
    sel = np.zeros(n, dtype=bool)
    sel[q] = True
    touch = sel[pairs[:, 0]] | sel[pairs[:, 1]]
    return dict(P=P, eps=eps, pairs=pairs, d2=d2, q=q, rs=rs, nbr=nbr, nd2=nd2, touch=touch)


def test_lists_cut_from_a_larger_epsilon_equal_direct_lists(case):
    c = case
    rs, nbr, nd2 = orc.rows_join(c["P"], 0.9, c["q"])
    rs2, nbr2, nd22 = cut_to_eps(rs, nbr, nd2, c["eps"])
    assert np.array_equal(rs2, c["rs"]) and np.array_equal(nbr2, c["nbr"]) and np.array_equal(nd22, c["nd2"])
    rs0, nbr0, _ = cut_to_eps(rs, nbr, nd2, 0.0)
    assert rs0[-1] == 0 and nbr0.size == 0


@pytest.mark.parametrize("strict", [False, True])
def test_row_check_passes_on_the_oracle_and_catches_planted_mistakes(case, strict):
    c = case
    t = c["touch"]
    args = (c["P"], c["eps"], c["q"], c["rs"], c["nbr"], c["nd2"])
    st = parity.check_rows(*args, c["pairs"][t], c["d2"][t].astype(np.float32), strict=strict)
    assert st["mismatches"] == 0 and st["overlap_accuracy"] == 1.0 and st["d2_checked"] == c["nbr"].size and st["floor_used"] == 0
    far = np.where(t & (np.abs(np.sqrt(c["d2"]) - c["eps"]) > 0.05) & (c["pairs"][:, 0] != c["pairs"][:, 1]))[0][0]
    keep = np.ones(len(c["pairs"]), dtype=bool)
    keep[far] = False
    with pytest.raises(AssertionError, match="missed"):
        parity.check_rows(*args, c["pairs"][t & keep], c["d2"][t & keep].astype(np.float32), strict=strict)
    # an extra pair far outside the band: a query row with a point of another cluster
    qrow = int(c["q"][0])
    j = next(j for j in range(c["P"].shape[0]) if orc.dist2(c["P"], qrow, j) > 4 * c["eps"] ** 2)
    extra = np.array([[min(qrow, j), max(qrow, j)]], dtype=np.uint32)
    with pytest.raises(AssertionError, match="reported"):
        parity.check_rows(*args, np.concatenate([c["pairs"][t], extra]), np.concatenate([c["d2"][t], [0.5]]).astype(np.float32), strict=strict)
    bad = c["d2"].astype(np.float32).copy()
    bad[far] *= np.float32(1.01)
    with pytest.raises(AssertionError, match="dist2 off"):
        parity.check_rows(*args, c["pairs"][t], bad[t], strict=strict)
    # a pair inside the band may fall either way, and is counted
    near = np.where(t & orc.boundary_band(c["d2"], c["eps"], 1e-3) & (c["pairs"][:, 0] != c["pairs"][:, 1]))[0]
    if near.size:
        keep[:] = True
        keep[near[0]] = False
        st = parity.check_rows(*args, c["pairs"][t & keep], c["d2"][t & keep].astype(np.float32), strict=strict)
        assert st["mismatches"] >= 1 and st["overlap_accuracy"] < 1.0


@pytest.mark.parametrize("strict", [False, True])
def test_pair_set_check_passes_on_the_oracle_and_catches_planted_mistakes(case, strict):
    c = case
    st = parity.check_pair_sets(c["P"], c["eps"], c["pairs"], c["d2"].astype(np.float32), c["pairs"], c["d2"], strict=strict)
    assert st["mismatches"] == 0 and st["floor_used"] == 0
    far = np.where((np.abs(np.sqrt(c["d2"]) - c["eps"]) > 0.05) & (c["pairs"][:, 0] != c["pairs"][:, 1]))[0][0]
    keep = np.ones(len(c["pairs"]), dtype=bool)
    keep[far] = False
    with pytest.raises(AssertionError, match="missed"):
        parity.check_pair_sets(c["P"], c["eps"], c["pairs"][keep], c["d2"][keep].astype(np.float32), c["pairs"], c["d2"], strict=strict)
    with pytest.raises(AssertionError, match="duplicate"):
        parity.check_pair_sets(c["P"], c["eps"], np.concatenate([c["pairs"], c["pairs"][far:far + 1]]),
                               np.concatenate([c["d2"], c["d2"][far:far + 1]]).astype(np.float32), c["pairs"], c["d2"], strict=strict)
