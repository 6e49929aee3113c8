import hashlib

import numpy as np

import datagen


def test_generator_is_deterministic_and_in_range():
    for w in (1, 2, 3, 4, 5):
        a = datagen.generate(w, n=3000)
        b = datagen.generate(w, n=3000, threads=1)
        assert a.dtype == np.uint16 and a.shape == (3000, datagen.WORKLOADS[w]["d"])
        assert np.array_equal(a, b)
        f = a.view(np.float16).astype(np.float32)
        assert np.isfinite(f).all() and f.min() >= 0.0 and f.max() <= 1.0


def test_multi_chunk_generation_matches_serial():
    n = datagen.CHUNK_ROWS + 1234
    a = datagen.generate(2, n=n, threads=4)
    b = datagen.generate(2, n=n, threads=1)
    assert np.array_equal(a, b)
    # chunk 0 does not depend on how many rows follow it
    c = datagen.generate(2, n=datagen.CHUNK_ROWS)
    assert np.array_equal(a[:datagen.CHUNK_ROWS], c)


def test_mixture_has_cluster_structure():
    w = datagen.WORKLOADS[2]
    x = datagen.generate(2, n=4000).view(np.float16).astype(np.float64)
    # coordinate-wise spread is dominated by the centres (var 1/12), not by sigma^2
    assert 0.05 < x.var(axis=0).mean() < 0.12
    assert w["sigma"] ** 2 < 0.01


def test_sample_indices_distinct_sorted_seeded():
    s = datagen.sample_indices(2)
    assert s.size == 2048 and np.all(np.diff(s) > 0) and s.max() < 100_000
    assert np.array_equal(s, datagen.sample_indices(2))
    assert not np.array_equal(s[:100], datagen.sample_indices(5)[:100])
    q = datagen.query_rows(2, 64)
    assert q.size == 64 and np.all(np.diff(q) > 0)


def test_workload_1_fingerprint_is_stable():
    # guards against silent changes of the recipe (numpy Philox stream + fp16 rounding)
    h = hashlib.sha256(datagen.generate(1).tobytes()).hexdigest()
    assert h == open(__file__.replace("test_datagen.py", "golden/workload1_sha256.txt")).read().split()[0]


def test_stored_eps_reproduced_by_the_oracle():
    # the stored epsilon values are written by oracle/select_eps.py; re-derive the cheap ones
    import json
    import os
    from oracle import oracle as orc
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    stored = json.load(open(os.path.join(root, "paper_2508_21230_amd", "workloads_eps.json")))
    P = orc.decode(datagen.generate(1))
    e = stored["1"]["eps"]["32"]
    eps = orc.select_eps_all_pairs(P, 32)
    assert hex(int(eps.view(np.uint32))) == e["eps_f32_hex"] and float(eps) == e["eps"]
    assert orc.selfjoin_count(P, eps)[1] == e["K"] == 65536
    X = datagen.generate(2)
    Ps = orc.decode(np.ascontiguousarray(X[datagen.sample_indices(2)]))
    e = stored["2"]["eps"]["64"]
    eps = orc.select_eps_sample(Ps, 64, n_full=100_000)
    assert hex(int(eps.view(np.uint32))) == e["eps_f32_hex"]
