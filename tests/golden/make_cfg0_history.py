"""Writes tests/golden/cfg0_history.txt: the fp64 oracle's loss and gradient-norm
trajectory on the smallest benchmark configuration (logistic regression,
4096 x 128, lambda 1e-4, step 0.1, 50 iterations, seed 0, inputs drawn on the
CPU).  Calls only the seeded input generator and the oracle; no value in the
file comes from the GPU library.

Run from the repository root:  python tests/golden/make_cfg0_history.py
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_1802_04819_amd import synth  # noqa: E402


def main():
    p = synth.config0(device="cpu")
    lh, gh, _, _ = oracle.run(p.loss, p.X.numpy(), p.y.numpy(), p.w0.numpy().astype("float64"),
                              p.lam, p.eta, p.K)
    out = os.path.join(ROOT, "tests", "golden", "cfg0_history.txt")
    with open(out, "w") as f:
        f.write("# oracle (fp64, sequential) on synth.config0(): iteration, loss L(w_k), |grad L(w_k)|_2\n")
        f.write("# source: tests/golden/make_cfg0_history.py (oracle only); not a value printed by the paper\n")
        for k in range(p.K):
            f.write(f"{k} {float(lh[k])!r} {float(gh[k])!r}\n")
    print("wrote", out)


if __name__ == "__main__":
    main()
