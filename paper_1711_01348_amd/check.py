"""Error measures used when a result is compared with a reference (no reference is computed here)."""
from __future__ import annotations

import numpy as np

# acceptance limits: (floored element-wise relative error, normwise relative error)
LIMITS = {"f64": (1e-12, 1e-13), "f32": (1e-4, 1e-5)}


def errors(got, ref) -> dict:
    """Three error figures for one tensor.

    ``floored``  max_i |g_i - r_i| / max(|r_i|, 1e-2 * max|r|): element-wise relative error whose
                 denominator is floored, because sums of terms of random sign leave individual
                 elements arbitrarily close to zero where a pure relative bound cannot hold in fp32;
    ``normwise`` ||g - r||_2 / ||r||_2;
    ``raw``      max_i |g_i - r_i| / |r_i| over r_i != 0 (information only).
    """
    g = np.asarray(got, dtype=np.float64).reshape(-1)
    r = np.asarray(ref, dtype=np.float64).reshape(-1)
    assert g.shape == r.shape, (g.shape, r.shape)
    if r.size == 0:
        return dict(floored=0.0, normwise=0.0, raw=0.0)
    diff = np.abs(g - r)
    rmax = float(np.max(np.abs(r)))
    if rmax == 0.0:
        bad = float(np.max(diff))
        return dict(floored=bad, normwise=bad, raw=bad)
    floored = float(np.max(diff / np.maximum(np.abs(r), 1e-2 * rmax)))
    normwise = float(np.linalg.norm(g - r) / np.linalg.norm(r))
    nz = r != 0
    raw = float(np.max(diff[nz] / np.abs(r[nz]))) if nz.any() else 0.0
    return dict(floored=floored, normwise=normwise, raw=raw)


def within(got, ref, dtype: str) -> bool:
    e = errors(got, ref)
    lim = LIMITS[dtype]
    zero_ok = bool(np.all(np.asarray(got)[np.asarray(ref) == 0] == 0)) if dtype == "f64" else True
    return e["floored"] <= lim[0] and e["normwise"] <= lim[1] and zero_ok
