"""Writes activation_points.txt: closed-form values of the two activations.

Independent of the oracle and of libm: 40-digit decimal arithmetic.
  GELU_tanh(z) = z/2 * (1 + tanh(sqrt(2/pi) * (z + 0.044715 z^3)))   (tanh-form GELU)
  SiLU(z)      = z / (1 + exp(-z))
tanh(x) is evaluated as (e^{2x} - 1) / (e^{2x} + 1) with Decimal.exp().
Citations: the MLP pattern's GELU epilogue (paper Section 5.2.4) and the SwiGLU
pattern's SiLU(gate) x up (Section 5.2.5); the tanh form is the workload's.
"""
import os
from decimal import Decimal, getcontext

getcontext().prec = 40
PI = Decimal("3.14159265358979323846264338327950288419716939937510")


def tanh(x):
    e = (2 * x).exp()
    return (e - 1) / (e + 1)


def gelu(z):
    return z / 2 * (1 + tanh((2 / PI).sqrt() * (z + Decimal("0.044715") * z ** 3)))


def silu(z):
    return z / (1 + (-z).exp())


POINTS = ["-6", "-3", "-2", "-1", "-0.5", "-0.125", "0", "0.125", "0.5", "1", "2", "3", "6"]

if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "activation_points.txt")
    with open(out, "w") as f:
        f.write("# name z value   (40-digit decimal arithmetic, printed to 20 significant digits;\n")
        f.write("# written by make_activation_points.py; GELU is the tanh form, paper Section 5.2.4;\n")
        f.write("# SiLU is the gate activation of Section 5.2.5)\n")
        for p in POINTS:
            z = Decimal(p)
            f.write(f"gelu_tanh {p} {gelu(z):.20e}\n")
        for p in POINTS:
            z = Decimal(p)
            f.write(f"silu {p} {silu(z):.20e}\n")
    print(out)
