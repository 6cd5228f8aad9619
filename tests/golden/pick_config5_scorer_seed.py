"""Picks the seed of workload config 5's scorer inputs (recorded in paper_2601_09093_amd/workloads.py).

Rule: the pruning step of config 5 is bit-exact only if the set of the 64 lowest trace scores does not
depend on the last bits of the step scores, so the scorer inputs (hidden states, weights, prior
running-mean state) are re-drawn, seed 0x5EED0005 + 0x100 j for j = 0, 1, ..., until the float64 chain
(Section 4.1 scorer, Section 4.3 running mean) leaves a gap above 4e-3 between the 64th and the 65th lowest
score.  Calls only the CPU oracle.  Usage: python tests/golden/pick_config5_scorer_seed.py
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import oracle  # noqa: E402
from paper_2601_09093_amd import workloads as wl  # noqa: E402

N, K, MARGIN = 256, 64, 4e-3


def gap_for(seed):
    sc = wl.build_scorer(seed, N, N, 4096, 1024, 26, 0, prior_state=True)
    _, probs = oracle.step_score(sc.hidden, sc.boundary_idx, sc.W1, sc.b1, sc.W2, sc.b2, act=0)
    scores = oracle.running_mean(sc.trace_of, probs.astype(np.float32), sc.score_sum.copy(), sc.score_cnt.copy())
    o = np.sort(scores)
    return float(o[K] - o[K - 1])


if __name__ == "__main__":
    for j in range(64):
        seed = 0x5EED0005 + 0x100 * j
        g = gap_for(seed)
        print("j = %d  seed = %#x  gap = %.3e" % (j, seed, g))
        if g > MARGIN:
            print("chosen: %#x" % seed)
            break
