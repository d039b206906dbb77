"""Writes eq3_values.txt: Eq. 3 of the paper evaluated from its printed formulas in 40-digit
decimal arithmetic (no implementation under test is involved)."""
import os
from decimal import Decimal, getcontext

getcontext().prec = 40
ROWS = [(0, 1), (1, 1), (5, 5), (10, 5), (50, 100), (300, 100), (7, 2), (90, 90), (12, 0), (1, 2),
        (64, 64), (175, 175)]
HEADER = """# Closed-form values of the MRI-centric importance I = H1 + H2 (Sec. 4, Eq. 3 of arXiv 2506.15969),
# H1 = 2*sigmoid(-(t-TS)/MRI), H2 = 2*sigmoid(-1/(MRI-1)) as printed; H2 = 0 for MRI <= 1; for MRI = 0
# and t > TS the score is 0 (the token was never re-activated).  Evaluated from the printed formulas in
# 40-digit decimal arithmetic by tests/golden/make_eq3_values.py; nothing here comes from any
# implementation under test.  Columns: t-TS  MRI  I (12 decimals)
"""


def f(x: Decimal) -> Decimal:
    return Decimal(2) / (Decimal(1) + x.exp())


def main():
    lines = []
    for dt, m in ROWS:
        if m == 0:
            v = Decimal(1) if dt == 0 else Decimal(0)
        else:
            v = f(Decimal(dt) / Decimal(m))
            if m > 1:
                v += f(Decimal(1) / Decimal(m - 1))
        lines.append("%d %d %.12f" % (dt, m, v))
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "eq3_values.txt"), "w") as fh:
        fh.write(HEADER + "\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
