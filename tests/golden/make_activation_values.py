"""Writes activation_values.txt: reference values of the epilogue activations.

Independent of the oracle and of libm: evaluated with Python's arbitrary
precision `decimal` arithmetic (50 digits) from the standard published forms
    ReLU(x)      = max(x, 0)
    GELU_tanh(x) = 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))),  tanh u = (e^{2u}-1)/(e^{2u}+1)
    SiLU(x)      = x / (1 + e^{-x})
and rounded once to double.  The paper (PRAGMA, Section 4.2) only names the
activation category; these are the usual definitions of the named functions.
Run:  python tests/golden/make_activation_values.py
"""
import os
from decimal import Decimal, getcontext

getcontext().prec = 50

# pi to 50 digits (Machin-like series evaluated in Decimal)
def _arctan_inv(n: int) -> Decimal:
    x = Decimal(1) / n
    x2 = x * x
    term, total, k = x, x, 1
    while abs(term) > Decimal(10) ** -55:
        term = -term * x2
        k += 2
        total += term / k
    return total

PI = 16 * _arctan_inv(5) - 4 * _arctan_inv(239)


def gelu_tanh(x: Decimal) -> Decimal:
    c = (Decimal(2) / PI).sqrt()
    u = c * (x + Decimal("0.044715") * x ** 3)
    e2u = (2 * u).exp()
    return Decimal("0.5") * x * (1 + (e2u - 1) / (e2u + 1))


def silu(x: Decimal) -> Decimal:
    return x / (1 + (-x).exp())


def relu(x: Decimal) -> Decimal:
    return x if x > 0 else Decimal(0)


XS = ["-8", "-5", "-3", "-2", "-1", "-0.5", "-0.125", "0.125", "0.5", "1", "2", "3", "5", "8"]

if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "activation_values.txt")
    with open(out, "w") as fh:
        fh.write("# name x value   (standard published forms; 50-digit decimal arithmetic rounded to double;\n")
        fh.write("# written by make_activation_values.py; the paper, Section 4.2, names the category only)\n")
        for name, fn in (("gelu_tanh", gelu_tanh), ("silu", silu), ("relu", relu)):
            for xs in XS:
                fh.write(f"{name} {xs} {float(fn(Decimal(xs)))!r}\n")
    print("wrote", out)
