"""Plain definition of the block-scaled 4-bit weight format the paper's largest
model is served in ("mxfp4 weights", Sec. IV-B), as laid down by the OCP
Microscaling Formats (MX) specification v1.0: elements in FP4 E2M1, one shared
E8M0 scale per block of 32 consecutive elements along the contraction index.

TEST INFRASTRUCTURE ONLY (see oracle/layer.py); shares no code with the HIP
library.  All arithmetic is float64; every representable product of an element
and a scale is exact in float64 (and in bf16, which is why the library may
expand the weights without loss).

Element (4 bits, S E1 E0 M, exponent bias 1):
    E = 0      : (-1)^S * M * 0.5                (zero and the one subnormal)
    E = 1..3   : (-1)^S * (1 + M/2) * 2^(E - 1)
  i.e. magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6; no infinities, no NaN.
Scale (8 bits, E8M0): 2^(e - 127) for e = 0..254; e = 255 is NaN (not produced
by the seeded inputs and rejected here).

Packing (a convention of this repository, stated in include/compact.h, not
fixed by the paper): two elements per byte, the element with the even index in
the low nibble; element k of a row sits in byte k // 2; its scale in byte
k // 32 of the row's scale array.

Pins (tests/test_oracle_pins.py): the sixteen code values against the
specification's value set (tests/golden/fp4_e2m1_values.txt), scales against
powers of two, the packing order by planting single codes, and round trips of
exactly representable matrices.  Parity unpinned: the nibble order (convention).
"""
import numpy as np

BLOCK = 32


def e2m1_value(code):
    """Value of one 4-bit code (0..15), by the field definition above."""
    code = int(code)
    s = (code >> 3) & 1
    e = (code >> 1) & 3
    m = code & 1
    mag = m * 0.5 if e == 0 else (1.0 + 0.5 * m) * 2.0 ** (e - 1)
    return -mag if s else mag


def e8m0_value(byte):
    byte = int(byte)
    if byte == 255:
        raise ValueError("E8M0 scale 255 is NaN")
    return 2.0 ** (byte - 127)


def dequantize(codes, scales):
    """codes uint8 [..., K/2] (two elements per byte, even index in the low nibble),
    scales uint8 [..., K/32]  ->  float64 [..., K]."""
    codes = np.asarray(codes, dtype=np.uint8)
    scales = np.asarray(scales, dtype=np.uint8)
    K = codes.shape[-1] * 2
    assert K % BLOCK == 0 and scales.shape[-1] == K // BLOCK and codes.shape[:-1] == scales.shape[:-1]
    table = np.array([e2m1_value(c) for c in range(16)], dtype=np.float64)
    out = np.empty(codes.shape[:-1] + (K,), dtype=np.float64)
    out[..., 0::2] = table[codes & 0x0F]
    out[..., 1::2] = table[codes >> 4]
    if (scales == 255).any():
        raise ValueError("E8M0 scale 255 is NaN")
    sc = np.exp2(scales.astype(np.float64) - 127.0)
    return out * np.repeat(sc, BLOCK, axis=-1)
