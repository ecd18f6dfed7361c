#!/usr/bin/env python3
"""Writes tests/golden/oracle_small_case.json from the CPU oracle alone (datagen + oracle/, no GPU code).

The paper prints no worked numeric example for this path (its tables are model-level accuracy and
latency), so there is no paper value to store here.  This fixture instead freezes the oracle's own
answer on one small seeded case: a change to the oracle's arithmetic, to the generator or to a
tie rule shows up as a diff of this file and has to be justified (the oracle's pins live in
tests/test_oracle_pins.py; this is a change detector, not a pin).

Run from the repository root:  python tests/golden/write_oracle_fixture.py
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import datagen  # noqa: E402
from oracle import ice_oracle as orc  # noqa: E402

CASE = dict(n_tokens=700, n_clusters=12, n_kv_heads=2, group_size=4, page_size=16, n_components=8, seed=11)
T, BUDGET, N_INSERT = 3, 64, 5


def digest(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()[:16]


def compute() -> dict:
    w = datagen.small(**CASE)
    K, V = datagen.keys_values(w)
    init = datagen.init_indices(w)
    q = datagen.queries(w)
    U = w.batch * w.n_kv_heads
    o = orc.OracleIndex(U, w.group_size, w.page_size, w.n_clusters, w.n_tokens + 64)
    inertia = o.build(K, V, init, T)
    stream = datagen.DecodeStream(w, seed=w.seed)
    chosen = []
    for _ in range(N_INSERT):
        k, v, _ = stream.next()
        c, _, _ = o.insert(k, v)
        chosen.append(c.tolist())
    ids, n_sel, scores, _ = o.select(q, BUDGET)
    out = o.attend(q, ids, n_sel)
    return {
        "case": CASE, "lloyd_rounds": T, "token_budget": BUDGET, "inserts": N_INSERT,
        "n_pages": o.n_pages.tolist(),
        "cluster_cnt": o.cluster_cnt.tolist(),
        "inertia": [[float("%.10e" % x) for x in row] for row in inertia],
        "insert_clusters": chosen,
        "page_ids": ids.tolist(), "n_selected": n_sel.tolist(),
        "scores": [[float("%.7e" % x) for x in row] for row in scores],
        "out_head0_first8": [[float("%.6e" % x) for x in out[u, 0, :8]] for u in range(U)],
        "sha256_16": {"assign": digest(o.assign), "page_pos": digest(o.page_pos), "rep": digest(o.rep),
                      "page_sum": digest(o.page_sum), "Kp": digest(o.Kp)},
    }


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small_case.json")
    with open(path, "w") as f:
        json.dump(compute(), f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote", path)
