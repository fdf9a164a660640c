"""Writes the expected values of mf_step_3x3.txt: one pass of per-entry SGD over five revealed entries of a 3 x 3
matrix, rank 2, in exact rational arithmetic (Python's fractions only - nothing of the oracle or the library is
imported).  The step is that of the latent-factor model of Sec. 4.1 "Matrix factorization":
    e = v - <w_i, h_j>;  w_i += lr (e h_j - lambda w_i);  h_j += lr (e w_i - lambda h_j),  both from the old rows.
Run it to check the stored file: `python tests/golden/make_mf_step_3x3.py` prints the lines `after1_W0`,
`after1_H0`, `W` and `H` of the file, and with --check compares them with what the file holds."""
import os
import sys
from fractions import Fraction as F

LR, LAM = F(1, 2), F(1, 4)
W0 = [[F(1), F(1, 2)], [F(-1, 2), F(1, 4)], [F(1, 4), F(-1)]]
H0 = [[F(1, 2), F(2)], [F(-1), F(1, 2)], [F(3, 2), F(1, 4)]]
ENTRIES = [(0, 0, F(5, 2)), (0, 1, F(-1)), (2, 1, F(1, 2)), (1, 2, F(2)), (2, 0, F(-3, 2))]


def fmt(rows):
    return " ; ".join(" ".join(str(x) for x in r) for r in rows)


def lines():
    W, H = [list(r) for r in W0], [list(r) for r in H0]
    out = []
    for step, (i, j, v) in enumerate(ENTRIES):
        w, h = W[i], H[j]
        e = v - sum(a * b for a, b in zip(w, h))
        W[i] = [wk + LR * (e * hk - LAM * wk) for wk, hk in zip(w, h)]
        H[j] = [hk + LR * (e * wk - LAM * hk) for wk, hk in zip(w, h)]
        if step == 0:
            out.append("after1_W0 " + fmt([W[0]]))
            out.append("after1_H0 " + fmt([H[0]]))
    out.append("W " + fmt(W))
    out.append("H " + fmt(H))
    return out


if __name__ == "__main__":
    got = lines()
    print("\n".join(got))
    if "--check" in sys.argv:
        stored = [l.strip() for l in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "mf_step_3x3.txt"))]
        missing = [l for l in got if l not in stored]
        if missing:
            print("differs from mf_step_3x3.txt:", missing, file=sys.stderr)
            sys.exit(1)
        print("mf_step_3x3.txt agrees")
