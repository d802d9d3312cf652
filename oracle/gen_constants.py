"""Prints the constants of the oracle's exp(-y) evaluation.

TEST INFRASTRUCTURE.  The values are defined mathematically and computed
here with 60-digit decimal arithmetic:
  EXPC[j+3] = round(exp(-2^j) * 2^31), j = -3..4
  TAYLOR_C3 = round(2^31 / 6), TAYLOR_C4 = round(2^31 / 24)
Run: python oracle/gen_constants.py
"""
from decimal import Decimal, getcontext, ROUND_HALF_EVEN

getcontext().prec = 60


def rnd(d):
    return int(d.to_integral_value(rounding=ROUND_HALF_EVEN))


def constants():
    two31 = Decimal(2) ** 31
    expc = [rnd((-(Decimal(2) ** j)).exp() * two31) for j in range(-3, 5)]
    return expc, rnd(two31 / 6), rnd(two31 / 24)


if __name__ == "__main__":
    expc, c3, c4 = constants()
    print("EXPC =", expc)
    print("TAYLOR_C3 =", c3)
    print("TAYLOR_C4 =", c4)
