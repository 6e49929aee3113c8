"""Writes paper_2508_21230_amd/workloads_eps.json: the epsilon of every synthetic workload.

Epsilon is part of a workload's definition and is chosen by the CPU oracle (this script calls
only oracle/ and the input generator):
  * workload 1: epsilon lies between the K-th and (K+1)-th smallest of all n(n-1)/2 FP64 pair
    distances, K = S*n/2 (mean S neighbours per point over the whole set);
  * workloads 2-5: the same rule on a seeded sample of 2,048 points, with
    K = round(S/(n-1) * m(m-1)/2), i.e. the sample's pair fraction matches S/(n-1).
The paper picks epsilon per data set for target selectivities the same way in spirit
(Section 4.1.3: S = (|R|-|D|)/|D|, epsilon values per data set in the data-set table).

Run:  python -m oracle.select_eps            (about a minute; needs ~6 GB of host memory)
"""
from __future__ import annotations

import json
import os
import sys
import time

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import datagen  # noqa: E402
from oracle import oracle as orc  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2508_21230_amd", "workloads_eps.json")


def main(workloads=(1, 2, 3, 4, 5)):
    res = {}
    if os.path.exists(OUT):
        res = json.load(open(OUT))
    for w in workloads:
        spec = datagen.WORKLOADS[w]
        t0 = time.time()
        X = datagen.generate(w)
        entry = dict(n=spec["n"], d=spec["d"], data_seed=datagen.data_seed(w), sample_seed=datagen.sample_seed(w), eps={})
        if spec["eps_from"] == "all_pairs":
            P = orc.decode(X)
            D2 = orc.all_pairs_dist2(P)
            for S in spec["selectivity"]:
                K = int(round(S * spec["n"] / 2))
                eps = orc.eps_for_pair_rank(D2, K)
                entry["eps"][str(S)] = dict(eps=float(eps), eps_f32_hex=hex(int(np.float32(eps).view(np.uint32))), K=K, pairs_ranked=int(D2.size))
        else:
            idx = datagen.sample_indices(w)
            P = orc.decode(np.ascontiguousarray(X[idx]))
            D2 = orc.all_pairs_dist2(P)
            m = idx.size
            for S in spec["selectivity"]:
                K = max(int(round(S / (spec["n"] - 1) * (m * (m - 1) // 2))), 1)
                eps = orc.eps_for_pair_rank(D2, K)
                entry["eps"][str(S)] = dict(eps=float(eps), eps_f32_hex=hex(int(np.float32(eps).view(np.uint32))), K=K, pairs_ranked=int(D2.size))
        res[str(w)] = entry
        print(f"workload {w}: {entry['eps']}  ({time.time() - t0:.1f}s)", flush=True)
        del X
    with open(OUT, "w") as f:
        json.dump(res, f, indent=1, sort_keys=True)
        f.write("\n")


if __name__ == "__main__":
    main(tuple(int(a) for a in sys.argv[1:]) or (1, 2, 3, 4, 5))
