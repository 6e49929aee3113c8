"""The allocation-free entry point (ejoin_selfjoin_pairs_noalloc) against ejoin_selfjoin_pairs, through the C ABI.

Two calls in a row on the shared static scratch, the second on a smaller input, then one at another
dimensionality: each must give exactly the pair set and squared distances of the existing entry point.
The calls run on a context that has never had a workspace, and the device's free memory is read before
and after them: the entry point must not allocate.
"""
import numpy as np
import pytest
import torch

import datagen

pytestmark = pytest.mark.gpu


def sorted_result(pairs, d2, n_pairs):
    found = int(n_pairs.cpu()[0])
    assert found <= pairs.shape[0]
    p = pairs[:found].to(torch.int64) & 0xFFFFFFFF
    keys = (p[:, 0] << 32) | p[:, 1]
    order = torch.argsort(keys)
    return found, keys[order].cpu().numpy(), d2[:found][order].cpu().numpy().view(np.uint32)


def test_noalloc_entry_point_matches_selfjoin_pairs():
    import paper_2508_21230_amd as pkg
    ref = pkg.EJoin(0)
    ej = pkg.EJoin(0)  # never gets a workspace of its own
    cases = [(2, 100_000, 0.80), (2, 3_001, 0.85), (3, 20_000, 0.95)]
    try:
        for w, n, eps in cases:
            X = datagen.generate(w, n=n)
            Xd = torch.from_numpy(X.view(np.int16)).cuda()
            want_pairs, want_d2, want_n = ref.selfjoin_pairs(Xd, eps, capacity=40_000_000)
            torch.cuda.synchronize()
            found, want_keys, want_bits = sorted_result(want_pairs, want_d2, want_n)
            assert found > n, "the case must produce neighbours"
            del want_pairs, want_d2
            pairs = torch.empty((found + 1000, 2), dtype=torch.int32, device="cuda")
            d2 = torch.empty(found + 1000, dtype=torch.float32, device="cuda")
            n_pairs = torch.full((1,), -1, dtype=torch.int64, device="cuda")
            torch.cuda.synchronize()
            free_before = torch.cuda.mem_get_info()[0]
            print(f"noalloc case w={w} n={n} eps={eps}: {found} pairs expected", flush=True)
            ej.selfjoin_pairs_noalloc(Xd, eps, pairs, d2, n_pairs)
            torch.cuda.synchronize()
            assert torch.cuda.mem_get_info()[0] == free_before, "the allocation-free entry point changed the device's free memory"
            assert ej.status() == 0
            got, keys, bits = sorted_result(pairs, d2, n_pairs)
            assert got == found
            assert np.array_equal(keys, want_keys), "pair set differs from ejoin_selfjoin_pairs"
            assert np.array_equal(bits, want_bits), "squared distances differ from ejoin_selfjoin_pairs"
    finally:
        ej.close()
        ref.close()


def test_noalloc_entry_point_rejects_what_does_not_fit():
    import paper_2508_21230_amd as pkg
    ej = pkg.EJoin(0)
    try:
        n, d = 200_000, 128  # 64 MB of packed copy: beyond the 40 MiB scratch
        Xd = torch.zeros((n, d), dtype=torch.int16, device="cuda")
        pairs = torch.empty((16, 2), dtype=torch.int32, device="cuda")
        n_pairs = torch.full((1,), 7, dtype=torch.int64, device="cuda")
        with pytest.raises(pkg.EJoinError, match="static scratch"):
            ej.selfjoin_pairs_noalloc(Xd, 0.1, pairs, None, n_pairs)
        torch.cuda.synchronize()
        assert int(n_pairs.cpu()[0]) == 7, "nothing may be enqueued on error"
    finally:
        ej.close()
