"""Writes tests/golden/oracle_tiny_rows.txt.  Calls only the CPU oracle and the
seeded input generator (never the GPU library).  The paper prints no numeric
example of the attention computation, so this file is a regression record of
the pinned oracle on the smallest benchmark configuration (B=1, Hq=4, Hkv=1,
N=1024, D=64, W=128, S=4), not a value from the paper.

    python tests/golden/make_golden.py
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import swaa_attn_oracle  # noqa: E402
from paper_2512_10411_amd.inputs import WORKLOADS, make_workload  # noqa: E402

ROWS = [0, 1, 3, 4, 5, 126, 127, 128, 129, 130, 131, 132, 133, 511, 512, 1022, 1023]


def main():
    w = WORKLOADS["tiny"]
    q, k, v = make_workload(w)
    out, lse = swaa_attn_oracle(q, k, v, w.window, w.n_sink, w.scale, rows=ROWS)
    path = os.path.join(HERE, "oracle_tiny_rows.txt")
    with open(path, "w") as f:
        f.write("# written by tests/golden/make_golden.py from oracle/ only; workload 'tiny'\n")
        f.write("# head row lse o[0] o[1] o[31] o[63]\n")
        for h in (0, 3):
            for r, i in enumerate(ROWS):
                o = out[0, h, r]
                f.write("%d %d %.17g %.17g %.17g %.17g %.17g\n" % (h, i, lse[0, h, r], o[0], o[1], o[31], o[63]))
    print("wrote", path)


if __name__ == "__main__":
    main()
