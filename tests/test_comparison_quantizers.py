"""Fig. 1's synthetic setup on the CPU: tables of 10 rows with standard normal entries, the
embedding dimension swept, 4-bit codes, normalized l2 error ||X - Q(X)|| / ||X||.

The comparison quantizers (SYM, GSS, ACIQ's Laplace formula, TABLE) live in
`comparison_quantizers.py`; GREEDY, GREEDY(opt) and ASYM are the oracle's.  The paper prints no
numbers for the figure (only the plot), so what is asserted is the ordering that Section 2 ("Their
Limitations") and Table 2 state in words."""
import numpy as np
import pytest

import comparison_quantizers as cq


def errors(oracle, d, seed):
    rng = np.random.default_rng(1000 * d + seed)
    t = rng.standard_normal((10, d)).astype(np.float32)
    r = {"ASYM(real)": cq.normalized_l2(t, cq.rowwise(t, cq.asym)),
         "SYM": cq.normalized_l2(t, cq.rowwise(t, cq.sym)),
         "GSS": cq.normalized_l2(t, cq.rowwise(t, cq.gss)),
         "ACIQ": cq.normalized_l2(t, cq.rowwise(t, cq.aciq_laplace))}
    whole = cq.table_range(t)
    r["TABLE"] = cq.normalized_l2(t, cq.rowwise(t, lambda row: whole))
    for name, (b, ratio) in {"GREEDY": (200, 0.16), "GREEDY(opt)": (1000, 0.5), "ASYM": (200, 0.0)}.items():
        codes, scale, bias = oracle.quantize_rowwise_greedy(t, b, ratio)
        r[name] = cq.normalized_l2(t, oracle.dequantize(codes, scale, bias, d))
    return r


@pytest.mark.parametrize("d", [8, 16, 32, 64, 128, 256, 1024, 4096])
def test_ordering_of_fig1_on_normal_rows(oracle_lib, d):
    runs = [errors(oracle_lib, d, seed) for seed in range(4)]
    mean = {k: float(np.mean([r[k] for r in runs])) for k in runs[0]}
    for r in runs:
        # the oracle's ASYM (binary32, binary16 parameters) is the textbook min/max quantizer
        assert abs(r["ASYM"] - r["ASYM(real)"]) <= 0.01 * r["ASYM(real)"]
        # GREEDY starts from ASYM's range and keeps the best range it meets
        assert r["GREEDY"] <= r["ASYM"] and r["GREEDY(opt)"] <= r["ASYM"]
        # row-wise ranges beat one range for the whole table; a symmetric range wastes levels
        assert r["TABLE"] > r["ASYM"] and r["SYM"] > r["ASYM"]
    # GREEDY(opt) walks a finer grid much further: never noticeably worse, clearly better on long rows
    assert mean["GREEDY(opt)"] <= 1.01 * mean["GREEDY"]
    if d >= 1024:
        assert mean["GREEDY(opt)"] < 0.98 * mean["GREEDY"]
    assert mean["GREEDY"] < 0.95 * mean["ASYM"]
    if d <= 64:
        # short rows: the clipping baselines have lost their advantage; GSS is worse than ASYM
        assert mean["GSS"] > mean["ASYM"]
        assert mean["ACIQ"] >= 0.999 * mean["ASYM"]
    if d >= 1024:
        # long rows: GSS and ACIQ are no worse than ASYM any more, GSS clearly better
        assert mean["GSS"] < 0.9 * mean["ASYM"] and mean["ACIQ"] <= mean["ASYM"]
    # GREEDY is the best 4-bit uniform quantizer up to the dimensions embedding tables use (Table 2)
    if d <= 256:
        assert mean["GREEDY"] < min(mean[k] for k in ("SYM", "GSS", "ASYM", "ACIQ", "TABLE"))


def test_comparison_quantizers_on_hand_checked_rows():
    """The helpers themselves: a row on an exact 16-point grid is reproduced by ASYM; SYM's range is
    symmetric; ACIQ's alpha for a two-point row; GSS lands inside (0, max|X|]."""
    grid = -1.5 + 0.2 * np.arange(16)
    assert np.allclose(cq.uniform_roundtrip(grid, *cq.asym(grid)), grid, atol=1e-12)
    assert cq.sym(np.array([-1.0, 3.0])) == (-3.0, 3.0)
    lo, hi = cq.aciq_laplace(np.array([-1.0, 1.0] * 50 + [40.0]))  # mean 0.396, E|X - mean| = 1.77
    x = np.array([-1.0, 1.0] * 50 + [40.0])
    alpha = 5.03 * np.abs(x - x.mean()).mean()
    assert lo == -1.0 and np.isclose(hi, x.mean() + alpha) and hi < 40.0
    rng = np.random.default_rng(0)
    row = rng.standard_normal(4096)
    a, b = cq.gss(row)
    assert a == -b and 0 < b <= np.abs(row).max()
    assert cq.sq_error(row, a, b) < cq.sq_error(row, *cq.sym(row))
