"""Inputs chosen to sit where a plausible shortcut in the quantize step goes wrong.  Test-side helper: it is used by
the oracle's pins and, as page contents, by the GPU parity tests."""
from fractions import Fraction

import numpy as np


def near_half_products(n_amax: int = 600, seed: int = 21):
    """(amax, x, q) triples, FP16 values and the correctly rounded code, for which the exact product x * s^-1 lies so
    close to k + 1/2 that rounding it to binary32 first lands exactly on k + 1/2 and the tie rule then picks the
    wrong neighbour.  s = amax / 127 and s^-1 = 1 / s are binary32 quotients; q is taken by exact rational
    arithmetic."""
    rng = np.random.default_rng(seed)
    finite = np.arange(1, 0x7C00, dtype=np.uint16).view(np.float16)
    out = []
    for amax in rng.choice(finite[finite >= np.float16(2.0 ** -10)], n_amax, replace=False):
        s = np.float32(np.float32(amax) / np.float32(127.0))
        s_inv = np.float32(np.float32(1.0) / s)
        x = finite[finite <= amax]
        p = x.astype(np.float64) * np.float64(s_inv)  # exact: 11 x 24 significant bits
        p32 = p.astype(np.float32).astype(np.float64)
        lands_on_tie = (p32 - np.floor(p32) == 0.5) & (p32 != p)
        wrong = lands_on_tie & (np.rint(p32) != np.rint(p))
        for xv in x[wrong]:
            pe = Fraction(float(xv)) * Fraction(float(s_inv))
            fl = pe.numerator // pe.denominator
            r = pe - fl
            q = fl + (1 if r > Fraction(1, 2) or (r == Fraction(1, 2) and fl % 2 == 1) else 0)
            out.append((np.float16(amax), np.float16(xv), int(q)))
    return out
