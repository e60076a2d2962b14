"""Writes closed_form_zero_weights.txt: 40-digit values of the zero-weight LSTM recurrence.

With every weight matrix zero the gate values are constants of the biases (cell equations,
Section 4 of the paper): f = sigmoid(b_f), i = sigmoid(b_i), o = sigmoid(b_o), g = tanh(b_g),
so c_t = f^t c_0 + i g (1 - f^t)/(1 - f) and h_t = o tanh(c_t).  Evaluated here with Python's
`decimal` module only (no LSTM code, no numpy), exp by decimal's own routine.

Run:  python tests/golden/make_closed_form.py
"""
import os
from decimal import Decimal, getcontext

getcontext().prec = 60


def sigmoid(z):
    return Decimal(1) / (Decimal(1) + (-z).exp())


def tanh(z):
    e2 = (2 * z).exp()
    return (e2 - 1) / (e2 + 1)


CASES = [
    # name, b_f, b_i, b_o, b_g, c0
    ("forget1", "1", "0", "0", "0", "0.5"),          # biases of the small dense config
    ("distinct", "0.3", "-0.7", "1.1", "0.45", "-0.25"),
]


def main():
    out = []
    out.append("# zero-weight closed form of the LSTM cell (paper Section 4 cell equations)")
    out.append("# columns: case t c_t h_t   (40 significant digits)")
    for name, bf, bi, bo, bg, c0 in CASES:
        f, i, o, g = sigmoid(Decimal(bf)), sigmoid(Decimal(bi)), sigmoid(Decimal(bo)), tanh(Decimal(bg))
        c0 = Decimal(c0)
        for t in range(0, 8):
            ft = f ** t
            c = ft * c0 + i * g * (1 - ft) / (1 - f)
            h = o * tanh(c)
            out.append(f"{name} {t} {c:.40e} {h:.40e}")
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "closed_form_zero_weights.txt")
    with open(path, "w") as fh:
        fh.write("\n".join(out) + "\n")
    print(path)


if __name__ == "__main__":
    main()
