"""Writes tests/golden/config0_oracle_samples.txt from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_golden.py
The file stores a few oracle outputs of the tiny fp32 configuration so that a later
change to the oracle's arithmetic (or to the seeded inputs) cannot pass unnoticed.
Nothing here touches the GPU library.
"""

import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

from helpers import config0_oracle  # noqa: E402

SAMPLES_PREFILL = [(0, 0, 0), (0, 63, 1), (0, 64, 2), (0, 65, 3), (0, 128, 0), (0, 255, 3)]  # (b, i, head)
SAMPLES_DECODE = [(0, 0), (0, 3)]  # (b, head)


def main():
    pre_out, dec_out, _ = config0_oracle()
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config0_oracle_samples.txt")
    with open(path, "w") as f:
        f.write("# oracle outputs, tiny fp32 configuration (4 layers, prefill 256, 16 decode steps)\n")
        f.write("# written by tests/golden/make_golden.py from oracle/ only; first 4 components of each row\n")
        for li, out in enumerate(pre_out):
            for (b, i, j) in SAMPLES_PREFILL:
                f.write("prefill %d %d %d %d " % (li, b, i, j) + " ".join("%.17g" % x for x in out[b, i, j, :4]) + "\n")
        for t, outs in enumerate(dec_out):
            for li, out in enumerate(outs):
                for (b, j) in SAMPLES_DECODE:
                    f.write("decode %d %d %d %d " % (t, li, b, j) + " ".join("%.17g" % x for x in out[b, j, :4]) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
