"""Shared test helpers: the error metric and tolerances of the parity bar."""
import numpy as np

# max relative error allowed against the float64 oracle, per storage dtype
TOL = {"f32": 1e-5, "bf16": 2e-2}


def rel_err(a, r):
    """max_i |a_i - r_i| / max(|r_i|, rms(r)): relative error with the reference's RMS as
    floor, so that entries where the exact result crosses zero (GELU' at the minimum,
    LayerNorm cancellation) do not make the ratio meaningless."""
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    r = np.asarray(r, dtype=np.float64).reshape(-1)
    assert a.shape == r.shape
    if r.size == 0:
        return 0.0
    assert not np.isnan(a[~np.isnan(r)]).any(), "NaN where the reference is finite"
    ok = np.isfinite(r)
    same_nonfinite = np.array_equal(a[~ok], r[~ok], equal_nan=True)
    assert same_nonfinite, "non-finite entries differ"
    if not ok.any():
        return 0.0
    rms = float(np.sqrt(np.mean(r[ok] ** 2)))
    floor = np.maximum(np.abs(r[ok]), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(a[ok] - r[ok]) / floor))
