"""Writes tests/golden/bessel_series.txt: the kernel of two single linear segments.

For x, y single segments with increments a, b the signatures are tensor exponentials (paper
Proposition 2.1), so k = sum_n <a,b>^n / (n!)^2 (Section 3.1), i.e. I0(2 sqrt z) for z = <a,b> > 0 and
J0(2 sqrt |z|) for z < 0.  Evaluated with mpmath at 40 digits straight from the series; calls nothing
from this repository.
"""
import os

import mpmath as mp

mp.mp.dps = 40
ZS = ["-2", "-1", "-0.5", "-0.1", "0", "0.01", "0.1", "0.25", "0.5", "1", "2", "3"]


def series(z):
    return mp.nsum(lambda n: z ** n / mp.factorial(n) ** 2, [0, mp.inf])


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    with open(os.path.join(here, "bessel_series.txt"), "w") as f:
        f.write("# z   sum_n z^n/(n!)^2   (paper Prop. 2.1 + Section 3.1; mpmath, 40 digits)\n")
        for zs in ZS:
            f.write("%s %s\n" % (zs, mp.nstr(series(mp.mpf(zs)), 25)))
