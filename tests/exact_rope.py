"""Rotary rotation of one head with cos/sin from 80-digit decimal arithmetic: a reference that is independent of
any double-precision range reduction, for position deltas of any size (test helper)."""
import numpy as np

import oracle as O


def exact_rotation(x_bits, delta, theta, D):
    """Half-split rotation of one head by `delta` positions with cos/sin from 80-digit decimal arithmetic
    (the frequency is the double theta^(-2j/D), taken as exact; the angle delta * frequency is then an exact
    decimal product, reduced modulo 2 pi and summed as a Taylor series).  bf16 bits in, bf16 bits out."""
    from decimal import Decimal, getcontext

    getcontext().prec = 80
    two_pi = 2 * Decimal("3.14159265358979323846264338327950288419716939937510582097494459230781640628620899862803482534")
    x = [Decimal(O.bf16_to_double(int(b))) for b in x_bits]
    out = [0] * D
    for j in range(D // 2):
        phi = (Decimal(int(delta)) * Decimal(float(theta) ** (-2.0 * j / D))) % two_pi
        c, s, term, k = Decimal(1), Decimal(0), Decimal(1), 0
        while abs(term) > Decimal(10) ** -70:
            k += 1
            term = term * phi / k
            if k % 2:
                s += term if k % 4 == 1 else -term
            else:
                c += term if k % 4 == 0 else -term
        out[j] = O.double_to_bf16(float(x[j] * c - x[j + D // 2] * s))
        out[j + D // 2] = O.double_to_bf16(float(x[j + D // 2] * c + x[j] * s))
    return np.array(out, np.uint16)
