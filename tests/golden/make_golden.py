"""Writes tests/golden/tiny_pure_samples.txt from the CPU oracle alone.

Run: python tests/golden/make_golden.py
The paper prints no numeric example of the operator, so these values are not the
paper's: they are the oracle's own output on the seeded "tiny" workload
(batch 1, 1 head, 14x14 tokens, d = 32, 7x7 agents pooled from Q, fp32 inputs,
pure mode; Sec. 4.1 Eq. (3) with A = Pooling(Q), Sec. 4.2), kept so that a later
edit of the oracle that changes its results is noticed.
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import agent_attn_oracle as oracle            # noqa: E402
from paper_2312_08874_amd import inputs                   # noqa: E402  (generator only)


def main():
    wl = inputs.WORKLOADS["tiny"]
    t = inputs.make_qkv(wl)
    O = oracle.agent_attn_fwd(inputs.to_float64(t["Q"], wl.dtype), inputs.to_float64(t["K"], wl.dtype),
                              inputs.to_float64(t["V"], wl.dtype), heads=wl.heads, grid=wl.grid,
                              agent_grid=wl.agent_grid)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_pure_samples.txt")
    with open(out, "w") as f:
        f.write("# oracle output O[0, token, channel] on workload 'tiny' (seed %d), pure mode\n" % inputs.BASE_SEED)
        f.write("# source: oracle/agent_attn_oracle.c via tests/golden/make_golden.py; not values printed by the paper\n")
        f.write("# token channel value\n")
        for i in range(0, wl.N, 13):
            for c in (0, 7, 31):
                f.write("%d %d %.17g\n" % (i, c, O[0, i, c]))
    print("wrote", out)


if __name__ == "__main__":
    main()
