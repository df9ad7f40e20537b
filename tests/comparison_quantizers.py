"""The comparison quantizers of Section 2 and Table 2, CPU side only (plain NumPy, float64).

They are the paper's baselines, not its method: nothing here is part of the library or of the
oracle; `test_comparison_quantizers.py` uses them to reproduce the qualitative ordering of Fig. 1
and Table 2 on synthetic rows.  Each function returns the clipping range (xmin, xmax) it chooses for
one row X; `uniform_roundtrip` is Eq. 1 followed by its de-quantizer, over the reals (float64, no
binary16 storage).

  SYM    symmetric range-based: xmax = max|X|, xmin = -xmax                          (Table 2, row SYM)
  ASYM   range-based: xmin = min X, xmax = max X                                    (Section 2)
  TABLE  ASYM with the range of the whole table instead of the row                  (Fig. 1)
  GSS    symmetric, threshold found by golden section search on the row's error     (Section 2, GSS)
  ACIQ   Laplace closed form for 4 bits: E X -+ 5.03 * E|X - E X|                    (Section 2, ACIQ)

Readings: GSS searches the threshold over (0, max|X|]; golden section search assumes a unimodal
objective, which the rounding makes only approximately true, so it may stop in a local minimum --
that is the method.  ACIQ's thresholds are intersected with [min X, max X] (a clip beyond the data
changes nothing but wastes levels; Table 2 prints ACIQ equal to ASYM at d = 8, 16, 32, which is what
the intersection gives when alpha exceeds the row's spread).
"""
import numpy as np

GOLDEN = (np.sqrt(5.0) - 1.0) / 2.0


def uniform_roundtrip(X, xmin, xmax, nbits=4):
    """x_float of Eq. 1's quantizer and de-quantizer for the clipping range [xmin, xmax]."""
    X = np.asarray(X, dtype=np.float64)
    levels = 2 ** nbits - 1
    scale = (xmax - xmin) / levels
    if scale <= 0:
        return np.full_like(X, xmin)
    q = np.rint((np.clip(X, xmin, xmax) - xmin) / scale)
    return scale * q + xmin


def sq_error(X, xmin, xmax, nbits=4):
    X = np.asarray(X, dtype=np.float64)
    return float(((X - uniform_roundtrip(X, xmin, xmax, nbits)) ** 2).sum())


def asym(X):
    return float(np.min(X)), float(np.max(X))


def sym(X):
    m = float(np.max(np.abs(X)))
    return -m, m


def table_range(table):
    return float(np.min(table)), float(np.max(table))


def gss(X, nbits=4, tol=1e-6, max_steps=200):
    """Golden section search for the symmetric threshold that minimises the row's squared error."""
    hi = float(np.max(np.abs(X)))
    if hi == 0.0:
        return 0.0, 0.0
    a, b = 0.0, hi
    f = lambda t: sq_error(X, -t, t, nbits)  # noqa: E731
    c, d = b - GOLDEN * (b - a), a + GOLDEN * (b - a)
    fc, fd = f(c), f(d)
    for _ in range(max_steps):
        if b - a <= tol * hi:
            break
        if fc < fd:
            b, d, fd = d, c, fc
            c = b - GOLDEN * (b - a)
            fc = f(c)
        else:
            a, c, fc = c, d, fd
            d = a + GOLDEN * (b - a)
            fd = f(d)
    t = (a + b) / 2
    return -t, t


def aciq_laplace(X):
    X = np.asarray(X, dtype=np.float64)
    mean = float(X.mean())
    alpha = 5.03 * float(np.abs(X - mean).mean())
    return max(float(X.min()), mean - alpha), min(float(X.max()), mean + alpha)


def normalized_l2(table, recon):
    """||X - Q(X)||_2 / ||X||_2 over the whole table (the quantity of Fig. 1 and Table 2)."""
    table = np.asarray(table, dtype=np.float64)
    return float(np.linalg.norm(table - recon) / np.linalg.norm(table))


def rowwise(table, chooser, nbits=4):
    """Reconstruction of a table when `chooser(row)` picks each row's clipping range."""
    return np.stack([uniform_roundtrip(row, *chooser(row), nbits=nbits) for row in np.asarray(table, dtype=np.float64)])
