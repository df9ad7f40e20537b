"""Lloyd's k-means rounds for one row in exact rational arithmetic (a pin for the codebook oracle).

k = 16 centres start on the uniform grid min + k*(max-min)/15; each round assigns every value to
its nearest centre (lowest index among equal distances) and moves each non-empty cluster's centre
to the mean of its members.  Python `Fraction`s throughout, so nothing is rounded.  The caller
uses small integer rows whose range is a multiple of 15: there every binary32 distance comparison
of the oracle agrees with the exact one unless two DIFFERENT centres are exactly equidistant from a
value, which this code reports so that such rows can be left out.
"""
from fractions import Fraction

K = 16


def lloyd(X, rounds):
    X = [Fraction(int(v)) for v in X]
    lo, hi = min(X), max(X)
    c = [lo + k * (hi - lo) / 15 for k in range(K)]
    exact_tie = False

    def assign(x):
        nonlocal exact_tie
        d = [abs(x - ck) for ck in c]
        m = min(d)
        first = d.index(m)
        if any(dk == m and c[k] != c[first] for k, dk in enumerate(d)):
            exact_tie = True
        return first

    for _ in range(rounds):
        labels = [assign(x) for x in X]
        for k in range(K):
            members = [x for x, a in zip(X, labels) if a == k]
            if members:
                c[k] = sum(members, Fraction(0)) / len(members)
    labels = [assign(x) for x in X]
    return c, labels, exact_tie
