"""Writes the table workloads.py steers its logit scale with: mean full-vocabulary entropy (nats) of
softmax(beta * z), z ~ N(0,1)^152064 stored as bf16, per scale beta, over six seeds.

    python tests/golden/make_entropy_scale_table.py        # prints the (entropy, beta) pairs

Calls only the CPU oracle (O1) and the seeded input generator.  The table shapes inputs; it is not an expected
value of any test (the kernels and the oracle report what the entropy of a row actually is).
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

import oracle  # noqa: E402
from paper_2602_00523_amd import workloads as wl  # noqa: E402

BETAS = [0.5, 1.0, 1.5, 2.0, 2.5, 3.0, 3.25, 3.5, 3.75, 4.0, 4.25, 4.5, 4.75, 5.0, 5.5, 6.0, 6.5, 7.0, 8.0, 9.0, 10.0, 12.0,
         14.0, 17.0, 20.0, 25.0, 30.0, 60.0]
SEEDS = 6
VOCAB = 152064


def main():
    pairs = []
    for beta in BETAS:
        rows = np.concatenate([wl.draft_logits(9000 + s, 1, VOCAB, "bf16", beta) for s in range(SEEDS)])
        h = oracle.entropy_topk(rows, 1)["entropy"]
        pairs.append((round(float(np.mean(h)), 2), beta))
    print("_ENTROPY_TO_SCALE_152064 = [")
    for i in range(0, len(pairs), 8):
        print("    " + " ".join(f"({h:.2f}, {b})," for h, b in pairs[i:i + 8]))
    print("]")


if __name__ == "__main__":
    main()
