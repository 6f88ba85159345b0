"""What 16-bit storage alone costs: the feed-forward half of the 8B-shaped layer evaluated
with the fp64 checker's own arithmetic, rounding to bf16 only where ANY bf16 layer has to
(the normalised activations that feed the matrix units, the SwiGLU intermediate, the
result), against the same without rounding.  No kernel is involved; this is the floor
under the element-wise tolerance of the GPU tests (tests/util.py, BF16_ELEM_TOL), and it
shows that the stated 2e-2 cannot be an element-wise bound at the workloads' sizes."""
import math

import numpy as np

from oracle import layer as O


def to_bf16(a):
    """Round-to-nearest-even to bf16, returned as float64."""
    u = np.asarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def test_bf16_rounding_helper():
    assert to_bf16(np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -0.1], dtype=np.float32)).tolist() == \
        [1.0, 1.0, 1.0 + 2.0 ** -6, float(np.float32(-0.10009765625))]


def test_storage_rounding_floor_of_the_dense_ffn_half():
    rng = np.random.default_rng(3)
    R, d, F = 64, 4096, 14336
    h = to_bf16(rng.standard_normal((R, d)))                       # the residual stream, as drawn for the workloads
    wg = to_bf16(0.02 * rng.standard_normal((F, d)))
    wu = to_bf16(0.02 * rng.standard_normal((F, d)))
    wd = to_bf16(0.02 * rng.standard_normal((d, F)))
    g = np.ones(d)
    m = O.rmsnorm(h, g, 1e-5)
    y = h + O.swiglu_ffn(m, wg, wu, wd)
    mr = to_bf16(m)
    act = to_bf16(O.silu(mr @ wg.T) * (mr @ wu.T))
    yr = to_bf16(h + act @ wd.T)
    rms_y = math.sqrt(np.mean(y * y))
    err = np.abs(yr - y) / np.maximum(np.abs(y), rms_y)
    rms_err = math.sqrt(np.mean((yr - y) ** 2)) / rms_y
    n = y.size
    print("floor: rms error %.3e, worst of %d elements %.3e = %.1f sigma" % (rms_err, n, err.max(), err.max() / rms_err))
    # three storage roundings of unit roundoff 2^-8 (rms relative error ~ 1.6e-3 each) in series
    assert 2.2e-3 < rms_err < 4.5e-3
    # the largest of n such errors: ~ sqrt(2 ln n) sigma.  At n = 2.6e5 that is already > 1.2e-2;
    # the workloads compare 1e5 .. 1e8 elements (sqrt(2 ln 1e8) = 6.1 sigma -> 2e-2 and more).
    assert err.max() > 4.0 * rms_err
    assert math.sqrt(2 * math.log(1e8)) * rms_err > 1.6e-2
