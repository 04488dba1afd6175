"""Writes mlp_speedup_closed_forms.txt: the two simplified closed forms that
Section 5 of the paper prints for the GPT-3 MLP shapes, evaluated for d = 1..4.
Uses nothing but those printed expressions (no code of this repository)."""
import os

HEADER = """\
# Section 5 prints the speed-up of msGeMM over the naive GeMM for the two GPT-3
# MLP shapes in simplified closed form (the plotted figure is not available):
#   MLP1 = 12288 x 49152 x b : 49152 / (16^d * 4 + (49152/d - 1))
#   MLP2 = 49152 x 12288 x b : 49152 / (16^d + (12288/d - 1) * 4)
# The numbers below are those two expressions evaluated for d = 1..4 (6 digits),
# written by make_mlp_speedup.py.  The text's "about 2.5x at d = 3" matches MLP2 only.
# name d value
"""


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "mlp_speedup_closed_forms.txt")
    with open(out, "w") as f:
        f.write(HEADER)
        for d in range(1, 5):
            f.write("mlp1 %d %.6f\n" % (d, 49152 / (16 ** d * 4 + (49152 / d - 1))))
        for d in range(1, 5):
            f.write("mlp2 %d %.6f\n" % (d, 49152 / (16 ** d + (12288 / d - 1) * 4)))


if __name__ == "__main__":
    main()
