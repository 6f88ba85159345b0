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


# bf16 storage mode, whole-layer outputs against the fp64 checker (the derivation is in
# tests/test_gpu_layer_bf16.py): per output vector, per element (floored at the tensor's
# rms), and pooled rms per kind of output.  The pooled bound sits between what storage rounding alone
# gives (3.4e-3, tests/test_bf16_floor.py) plus the kernels' own roundings (measured 4.2e-3 .. 5.2e-3) and
# what a dropped term or a bias would produce (1e-2 and up).
BF16_VEC_TOL = 2e-2
BF16_ELEM_TOL = 3e-2
BF16_RMS_TOL = 6e-3
FP32_TOL = 1e-5


class ErrLog:
    """Collects the three error measures per compared tensor and asserts them together.

    vec:  max over vectors of ||g - r|| / ||r||
    elem: max |g - r| / max(|r|, rms(r))           (the contract's element-wise measure)
    rms:  sqrt(sum |g - r|^2 / sum |r|^2) pooled over all tensors of one kind (the tag up
          to its first digit), so that a systematic bias cannot hide under a maximum."""

    def __init__(self, vec_tol=BF16_VEC_TOL, elem_tol=BF16_ELEM_TOL, rms_tol=BF16_RMS_TOL):
        self.vec_tol, self.elem_tol, self.rms_tol = vec_tol, elem_tol, rms_tol
        self.vec, self.elem, self.pool = {}, {}, {}

    @classmethod
    def for_depth(cls, n_layers):
        """A depth of layers: every layer adds its own storage roundings to the stream, independent
        of the earlier ones, so the element and rms errors grow like sqrt(n_layers); the per-vector
        bound is kept."""
        f = float(n_layers) ** 0.5
        return cls(BF16_VEC_TOL, BF16_ELEM_TOL * f, BF16_RMS_TOL * f)

    def cmp(self, tag, got, ref):
        got = np.asarray(got, dtype=np.float64)
        ref = np.asarray(ref, dtype=np.float64)
        assert got.shape == ref.shape, (tag, got.shape, ref.shape)
        if ref.size == 0:
            return
        assert np.all(np.isfinite(got)), tag
        self.vec[tag] = vec_rel_err(got, ref)
        self.elem[tag] = rel_err(got, ref)
        kind = tag.rstrip("0123456789_")
        while kind and kind[-1].isdigit():
            kind = kind[:-1].rstrip("_")
        num, den = self.pool.get(kind, (0.0, 0.0))
        self.pool[kind] = (num + float(np.sum((got - ref) ** 2)), den + float(np.sum(ref * ref)))

    def rms(self):
        return {k: (n / max(d, 1e-300)) ** 0.5 for k, (n, d) in self.pool.items()}

    def check(self, label=""):
        assert self.vec, "nothing was compared"
        wv, we = max(self.vec, key=self.vec.get), max(self.elem, key=self.elem.get)
        rms = self.rms()
        wr = max(rms, key=rms.get)
        print(label, "tensors compared: %d | worst vector error %s %.3e | worst element error %s %.3e | worst pooled rms error %s %.3e"
              % (len(self.vec), wv, self.vec[wv], we, self.elem[we], wr, rms[wr]))
        assert self.vec[wv] < self.vec_tol, {k: "%.2e" % v for k, v in self.vec.items() if v >= self.vec_tol}
        assert self.elem[we] < self.elem_tol, {k: "%.2e" % v for k, v in self.elem.items() if v >= self.elem_tol}
        assert rms[wr] < self.rms_tol, {k: "%.2e" % v for k, v in rms.items()}


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
