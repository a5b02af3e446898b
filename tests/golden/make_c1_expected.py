"""Writes tests/golden/c1_expected.txt from the CPU oracle alone.

Stored so that a later change to the oracle's arithmetic or to the input recipe
shows up as a diff.  Calls only `oracle/` and the input generator; never the HIP
library.  Run from the repository root:  python tests/golden/make_c1_expected.py
"""
import hashlib
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import workloads  # noqa: E402
from oracle import speckv_oracle as orc  # noqa: E402


def expected_lines():
    w = workloads.tiny_fp32()
    t = workloads.generate(w)
    q, k, v = (workloads.to_float64(t[x][0]) for x in ("q", "k", "v"))
    res = orc.speckv_layer(q[0], k, v, w.n_window, w.pool_k, w.c_max, w.sm_scale)
    lines = ["# tiny fp32 workload (seed 0): oracle indices and score summaries; written by make_c1_expected.py"]
    for g in range(w.n_kv_heads):
        idx = res["idx"][g]
        digest = hashlib.sha256(idx.astype("<i4").tobytes()).hexdigest()[:16]
        lines.append("head=%d n_keep=%d idx_sha=%s first8=%s pooled_max=%.12e pooled_sum=%.12e" % (
            g, idx.size, digest, ",".join(str(int(x)) for x in idx[:8]),
            res["pooled"][g].max(), res["pooled"][g].sum()))
    return lines


if __name__ == "__main__":
    with open(os.path.join(HERE, "c1_expected.txt"), "w") as f:
        f.write("\n".join(expected_lines()) + "\n")
