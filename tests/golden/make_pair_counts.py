"""Writes tests/golden/pair_counts.json: unmasked (query, key) pairs per query head of each workload.

Calls only the oracle's counter (a loop over rows) and the synthetic segment tables.  The closed form
these must equal, sum_t (s C + s (s+1)/2), is half of ((C+s)^2 - C^2) + s, the quadratic term of the
paper's computation-time model (Eq. 1, T_comp).
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402
import synth  # noqa: E402

out = {}
for idx in range(1, 6):
    for sl in (range(8) if idx == 5 else [None]):
        c = synth.case_by_index(idx, sl)
        z = np.zeros((c.total_q, 1, 1)); zk = np.zeros((c.total_kv, 1, 1))
        out[c.name] = oracle.Oracle(c.segs, z, zk, zk).pair_count()
with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "pair_counts.json"), "w") as f:
    json.dump(out, f, indent=1)
print(out)
