"""Helpers shared by the tests (no layer arithmetic)."""
import numpy as np


def rel_err(got, ref):
    """max_i |g_i - r_i| / max(|r_i|, rms(r)): element-wise relative error with
    the denominator floored at the tensor's RMS, so zero crossings of the
    reference do not blow it up."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(got - ref) / den))


def vec_rel_err(got, ref):
    """max over vectors (last axis) of ||g - r||_2 / ||r||_2: the relative error
    of each output hidden-state (or cached K/V head) vector."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    num = np.sqrt(np.sum((got - ref) ** 2, axis=-1))
    den = np.maximum(np.sqrt(np.sum(ref * ref, axis=-1)), 1e-300)
    return float(np.max(num / den))


def rms_err(got, ref):
    """rms(g - r) / rms(r): the typical (rather than worst-element) error."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.sqrt(np.mean((got - ref) ** 2)) / max(np.sqrt(np.mean(ref * ref)), 1e-300))


def read_golden(path):
    vals = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            vals[parts[0]] = np.array([float(p) for p in parts[1:]], dtype=np.float64)
    return vals
