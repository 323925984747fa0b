"""Writes the stored expected values under tests/golden/ -- calls only oracle/ and the
seeded input generators (never the GPU path).

    python tests/golden/make_golden.py

cfg0_evict_idx.txt: the slot index returned by each of the 512 decode steps of the
smallest workload (fp32, 1 x 4/1 heads, head_dim 64, budget 256, empty start).  No value
here comes from the paper, which prints no worked example for this path; the file guards
the oracle and the generators against silent change.
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import longflow_oracle as oracle          # noqa: E402
from paper_2603_11504_amd import workloads as W       # noqa: E402


def cfg0_evict_sequence():
    wl = W.CONFIGS[0]
    c = oracle.OracleCache(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget)
    c.init()
    seq = []
    for t in range(wl.steps):
        q, k, v = W.host_step(wl, t)
        _, idx = c.step(q, k, v)
        seq.append(int(idx[0, 0]))
    return seq


if __name__ == "__main__":
    seq = cfg0_evict_sequence()
    with open(os.path.join(HERE, "cfg0_evict_idx.txt"), "w") as f:
        f.write("# oracle evict_idx per decode step, workload cfg0 (written by make_golden.py): the slot\n"
                "# count while the cache fills, then argmin of the LongFlowScore (eq. 6; Sec. 3.2 last\n"
                "# paragraph; Alg. 1 post-processing). Not a value printed in the paper.\n")
        f.write("\n".join(str(i) for i in seq) + "\n")
    print("wrote", len(seq), "indices")
