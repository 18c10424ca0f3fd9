"""Writes tests/golden/tiny_reference.txt from the fp64 oracle alone (never from the GPU library).

The paper prints no worked numeric example of the head (no small tensor with its loss), so nothing here is
a value quoted from it.  The file is a regression anchor: the oracle's outputs on the seeded `tiny` workload
(64 positions, d=64, V=512, n=2, r=2, fp32) at the time its pins were established.  A test checks that the
oracle still reproduces them, and the GPU tests of the plain path may compare against the same numbers.

Run from the repository root:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import cp_oracle  # noqa: E402
from paper_2410_17765_amd import synth  # noqa: E402


def main():
    cp_oracle.build()
    cfg = synth.CONFIGS["tiny"]
    inp = synth.make_inputs(cfg)
    args = (inp["H"], inp["W"], inp["U"], inp["G"], inp["X"])
    loss = cp_oracle.loss_fwd(*args)
    g = cp_oracle.loss_bwd(*args, np.full(cfg.T, 1.0 / cfg.T))
    lines = ["# oracle on synth.CONFIGS['tiny'] (seeds in synth.py); written by tests/golden/make_golden.py",
             "# loss[t] for t = 0..7, then mean loss, then Frobenius norms of dH, dW, dU, dG for dloss = 1/T"]
    lines += [f"loss {t} {loss[t]:.15e}" for t in range(8)]
    lines.append(f"mean_loss {loss.mean():.15e}")
    for k in ("dH", "dW", "dU", "dG"):
        lines.append(f"norm_{k} {np.linalg.norm(g[k].ravel()):.15e}")
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_reference.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
