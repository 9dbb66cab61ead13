"""Writes normal_quantiles.txt: upper-tail standard-normal quantiles z(q), P(Z > z) = q.

These are fixed by the mathematics (the standard normal table), not by any implementation
under test: each is z = sqrt(2) * erfinv(1 - 2q) in 40-digit arithmetic with mpmath, checked by
substituting back into erfc(z/sqrt(2))/2 = q,
and printed to 17 significant digits.  The q list covers the table values usually quoted
(q = 0.025, 0.01, 0.005, 0.001, 0.0005) and the tail masses k/(2d) of the benchmark
configurations (Algorithm 1, step 3, with the two-sided reading) plus k/d (as printed).
Run: python tests/golden/make_normal_quantiles.py
"""
import os

import mpmath as mp

mp.mp.dps = 40

CASES = [("table", "0.025"), ("table", "0.01"), ("table", "0.005"), ("table", "0.001"),
         ("table", "0.0005"), ("table", "0.25"), ("table", "1e-9")]
for d, k in [(269722, 270), (14728266, 14729), (25557032, 25558), (25557032, 255571),
             (66034000, 66034), (64, 1)]:
    CASES.append((f"k/(2d) d={d} k={k}", mp.mpf(k) / (2 * d)))
    CASES.append((f"k/d d={d} k={k}", mp.mpf(k) / d))

here = os.path.dirname(os.path.abspath(__file__))
with open(os.path.join(here, "normal_quantiles.txt"), "w") as f:
    f.write("# q (upper-tail mass, 25 digits)   z (17 digits)   # label\n")
    for label, q in CASES:
        q = mp.mpf(q)
        z = mp.sqrt(2) * mp.erfinv(1 - 2 * q)
        assert abs(mp.erfc(z / mp.sqrt(2)) / 2 - q) < q * mp.mpf(10) ** -30
        f.write(f"{mp.nstr(q, 25)} {mp.nstr(z, 17)} # {label}\n")
