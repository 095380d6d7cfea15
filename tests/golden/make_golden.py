"""Writes tests/golden/cfg1_oracle.txt: what the fp64 oracle computes for the tiny fp32 stream.

Calls only the oracle and the seeded input generator (never the HIP library).  The file is a
regression pin for the oracle itself: the paper prints no worked numerical example (Alg. 1 is
symbolic), so there are no paper values to store.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import OracleStream                                     # noqa: E402
from paper_2409_09086_amd.workloads import CONFIGS, ChunkStream           # noqa: E402


def compute(bias):
    cfg = CONFIGS["cfg1"]
    s = OracleStream(cfg.budget, cfg.recent, cfg.heads, cfg.kv_heads, cfg.head_dim,
                     bias=float(np.float32(bias)), scale=float(np.float32(1.0 / np.sqrt(cfg.head_dim))))
    sums = []
    for _, (q, k, v) in zip(range(cfg.steps), ChunkStream(cfg)):
        out, _ = s.step(q.double().numpy(), k.double().numpy(), v.double().numpy())
        sums.append(float(out.sum()))
    return s.export()[2], sums


def main():
    lines = ["# cfg1 (4 heads x 64, budget 256, recent 64, 8 chunks of 64, seed 1): oracle output sums per step and",
             "# final stream positions per head.  Written by tests/golden/make_golden.py (oracle only)."]
    for bias in (1e-4, 1e-2):
        pos, sums = compute(bias)
        lines.append("bias %g" % bias)
        lines.append("sums " + " ".join("%.12e" % x for x in sums))
        for h in range(pos.shape[0]):
            lines.append("pos %d " % h + " ".join(str(int(x)) for x in pos[h]))
    with open(os.path.join(ROOT, "tests", "golden", "cfg1_oracle.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
