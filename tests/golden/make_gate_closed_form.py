#!/usr/bin/env python3
"""Writes gate_closed_form.txt: closed-form gate cases for two verdict tokens.

Nothing under test is imported: the confidence is the closed form 1 / (1 + exp(-|z0 - z1|)) of a
two-way softmax (Section 4.2, Eq. 3) evaluated with math.exp in double precision, and the gate bits are
the comparison conf >= gamma (Eq. 4) at the thresholds of the paper's ablation on verification strategy
(Table 3).  Run from anywhere: python tests/golden/make_gate_closed_form.py
"""
import math
import os

GAMMAS = (0.8, 0.9, 0.95)
HEADER = """# Closed-form gate cases for two verdict tokens.
# With logits (z0, z1) the softmax over the two verdict tokens gives
#   conf = 1 / (1 + exp(-|z0 - z1|))
# (Section 4.2, Eq. 3: the softmax probability of the emitted verification token), and the
# verifier's own decision is kept iff conf >= gamma (Section 4.2, Eq. 4).  The thresholds are
# the three the paper sweeps in its ablation on verification strategy (Table 3): 0.8, 0.9, 0.95.
# |z0 - z1| = ln(p / (1 - p)) -+ 0.05 puts conf clearly on either side of threshold p.
# conf values are the closed form evaluated in double precision, not an output of any code
# under test.
# columns: z0  z1  verdict  conf  accept@0.8  accept@0.9  accept@0.95
"""


def rows():
    out = []
    for p, base in zip(GAMMAS, (0.0, 0.0, 0.5)):
        gap = math.log(p / (1.0 - p))
        # just below the threshold, the second token ahead; just above it, the first token ahead
        for z0, z1 in ((base, base + gap - 0.05), (base + gap + 0.05, base)):
            out.append((z0, z1))
    return out


def line(z0, z1):
    conf = 1.0 / (1.0 + math.exp(-abs(z0 - z1)))
    verdict = 0 if z0 >= z1 else 1                      # lowest index on ties
    bits = " ".join(str(int(conf >= g)) for g in GAMMAS)
    return f"{z0!r} {z1!r} {verdict} {conf!r} {bits}\n"


def main():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "gate_closed_form.txt")
    with open(path, "w") as f:
        f.write(HEADER)
        for z0, z1 in rows():
            f.write(line(z0, z1))
        f.write("# tie: lowest index wins, conf = 1/2\n")
        f.write(line(0.25, 0.25))
    print("wrote", path)


if __name__ == "__main__":
    main()
