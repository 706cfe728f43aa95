"""TEST INFRASTRUCTURE -- exact-rational brute force of the same definitions, for tiny inputs.

Every binary floating-point input is an exact rational, so with fractions.Fraction the sums
G_i = (sum_k b_k g_ki)/B, n_k = sum_i g_ki^2, A = sum_i G_i^2, d_k = sum_i (g_ki - G_i)^2 and
T = (sum_k b_k d_k)/(K-1) are computed with no rounding at all.  Used to pin the C oracle on
P <= 64.  Pure Python loops; shares nothing with the C oracle or the HIP path.
"""
from fractions import Fraction


def exact_record(cols, b, lo, hi):
    """cols[k][i] are Python floats (exact values of the inputs); returns Fractions."""
    K = len(cols)
    B = sum(int(x) for x in b)
    G = []
    for i in range(lo, hi):
        s = Fraction(0)
        for k in range(K):
            s += int(b[k]) * Fraction(cols[k][i])
        G.append(s / B)
    A = sum((x * x for x in G), Fraction(0))
    n = [sum((Fraction(cols[k][i]) ** 2 for i in range(lo, hi)), Fraction(0)) for k in range(K)]
    d = [sum(((Fraction(cols[k][i]) - G[i - lo]) ** 2 for i in range(lo, hi)), Fraction(0))
         for k in range(K)]
    T = sum((int(b[k]) * d[k] for k in range(K)), Fraction(0)) / (K - 1) if K > 1 else Fraction(0)
    return {"G": G, "A": A, "n": n, "d": d, "T": T, "B": B, "A_unb": A - T / B}
