"""Writes tests/golden/oracle_table.txt: the oracle's 16 representatives and
derivative levels (S2A Sec. 3.2, GeLU paragraph, Eq. 9 and Eq. 12) at full
double precision.  Calls only oracle/.  Run from the repository root:

    python tests/golden/make_oracle_table.py
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))

import oracle  # noqa: E402


def main():
    xhat, deriv, _ = oracle.table()
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_table.txt")
    with open(out, "w") as fh:
        fh.write("# code  xhat (Eq. 9)  derivative (Eq. 12 at xhat)  -- written by make_oracle_table.py from oracle/ only\n")
        for k in range(16):
            fh.write(f"{k} {float(xhat[k])!r} {float(deriv[k])!r}\n")


if __name__ == "__main__":
    main()
