"""Recompute the tanh-form GELU anchors of gelu_values.txt with 40-digit decimal arithmetic
(no oracle, no HIP code involved): tanh(z) = (e^{2z}-1)/(e^{2z}+1)."""
from decimal import Decimal, getcontext

getcontext().prec = 40
PI = Decimal("3.14159265358979323846264338327950288419716939937510")


def gelu_tanh(x: Decimal) -> Decimal:
    z = (Decimal(2) / PI).sqrt() * (x + Decimal("0.044715") * x ** 3)
    e = (2 * z).exp()
    return x / 2 * (1 + (e - 1) / (e + 1))


if __name__ == "__main__":
    for x in ("1.0", "-1.0", "2.0", "0.5", "3.0", "0.0"):
        print("tanh", x, float(gelu_tanh(Decimal(x))))
