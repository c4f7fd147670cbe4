#!/usr/bin/env python3
"""Writes tests/golden/oracle_tiny_grid.txt from the CPU checker alone (run from the repository root).

The fixture freezes what the checker returns today for the smallest benchmark configuration, so that a later edit
of the checker that changes its results is noticed even where the analytic pins still pass.  It calls nothing
outside ``oracle/`` and the seeded input generators.
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import grf_oracle  # noqa: E402
from paper_2410_03462_amd import synth  # noqa: E402


def fixture_lines():
    wl = synth.workload("tiny_grid")
    rp, col, val = grf_oracle.sample(wl.graph, wl.f, wl.p_halt, wl.n_walks, wl.walk_seed)
    Q, K, V = wl.qkv()
    res = grf_oracle.masked_linear_attention(Q, K, V, rp, col, val)
    traj = grf_oracle.sample_walks(wl.graph, wl.p_halt, wl.n_walks, wl.f_len, wl.walk_seed)
    yield "# checker results for workload tiny_grid (16x16 4-neighbour grid, n_walks=4, p_halt=0.5, f_len=8, d=32, seed 0)"
    yield "# written by tests/golden/make_oracle_fixtures.py; integers as sha256 of the little-endian int32 bytes, reals as C99 hex floats"
    yield "nnz %d" % int(rp[-1])
    yield "trajectories_sha256 %s" % hashlib.sha256(np.ascontiguousarray(traj, dtype="<i4").tobytes()).hexdigest()
    yield "row_ptr_sha256 %s" % hashlib.sha256(np.ascontiguousarray(rp, dtype="<i4").tobytes()).hexdigest()
    yield "col_sha256 %s" % hashlib.sha256(np.ascontiguousarray(col, dtype="<i4").tobytes()).hexdigest()
    yield "val_sha256 %s" % hashlib.sha256(np.ascontiguousarray(val, dtype="<f4").tobytes()).hexdigest()
    yield "val_first8 " + " ".join(float(x).hex() for x in val[0, :8])
    yield "num_row100_first4 " + " ".join(float(x).hex() for x in res["num"][0, 0, 100, :4])
    yield "den_first4 " + " ".join(float(x).hex() for x in res["den"][0, 0, :4])


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_tiny_grid.txt")
    with open(path, "w") as fh:
        fh.write("\n".join(fixture_lines()) + "\n")
    print("wrote", path)
