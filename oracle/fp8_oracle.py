"""CPU checker for the 8-bit floating point GEMM variant -- TEST INFRASTRUCTURE ONLY.

The paper computes in 16-bit floating point and says nothing of 8-bit formats; this variant is
an extension of the projections' GEMM for hardware with 8-bit matrix instructions, and what it
computes is DEFINED here (the format by the Open Compute Project's "OCP 8-bit Floating Point
Specification (OFP8)", the recipe by this module):

  * Format E4M3 (OFP8): 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits; exponent field 0
    holds subnormals m/8 * 2^-6; there are no infinities; S.1111.111 is NaN; the largest finite
    value is S.1111.110 = 448.
  * Encoding rounds to nearest, ties to the even code, and saturates: magnitudes above 448 give
    +-448.  NaN gives the NaN code.
  * A matrix is quantised row by row: scale = max|row| / 448 computed in binary32 (1 for an
    all-zero row), code = encode(x / scale) with the division in binary32.  Both GEMM operands are
    K-contiguous, so "row" is a token for the activations and an output feature for the weights.
  * The product is  C[m, n] = sa[m] * sw[n] * sum_k dec(a[m, k]) * dec(w[n, k]).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module; it
shares no code with the HIP path.  Pins live in tests/test_oracle_fp8.py: the code points the
specification names, a library's independent conversion (torch.float8_e4m3fn on the CPU) over
all codes and over random and halfway values, error bounds of the row quantisation, and the
product against exact rational arithmetic on small cases.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0
NAN_CODE = 0x7F


def e4m3_decode(code: np.ndarray) -> np.ndarray:
    """Value of every E4M3 code (uint8) as float64."""
    code = np.asarray(code, dtype=np.uint8).astype(np.int64)
    sign = np.where(code & 0x80, -1.0, 1.0)
    e = (code >> 3) & 0xF
    m = (code & 0x7).astype(np.float64)
    normal = np.ldexp(1.0 + m / 8.0, (e - 7).astype(np.int64))
    sub = np.ldexp(m / 8.0, -6)
    val = sign * np.where(e == 0, sub, normal)
    return np.where((code & 0x7F) == 0x7F, np.nan, val)


# the 127 finite non-negative values in code order (strictly increasing)
_POS = e4m3_decode(np.arange(0x7F, dtype=np.uint8))


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code of every element: ties to the even code, saturating at +-448."""
    x = np.asarray(x, dtype=np.float64)
    mag = np.abs(x)
    hi = np.searchsorted(_POS, mag, side="left")           # first code whose value >= mag
    hi = np.clip(hi, 1, 0x7E)
    lo = hi - 1
    d_lo, d_hi = mag - _POS[lo], _POS[hi] - mag
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo)
    code = np.where(mag >= E4M3_MAX, 0x7E, code)           # saturate
    code = np.where(np.signbit(x), code | 0x80, code)
    code = np.where(np.isnan(x), NAN_CODE, code)
    return code.astype(np.uint8)


def quantize_rows(x: np.ndarray):
    """Row-wise scaled quantisation.  Returns (codes uint8 [M, K], scale float32 [M])."""
    x32 = np.asarray(x, dtype=np.float32)
    amax = np.max(np.abs(x32), axis=1) if x32.shape[1] > 0 else np.zeros(x32.shape[0], np.float32)
    scale = (amax / np.float32(E4M3_MAX)).astype(np.float32)
    scale = np.where(amax == 0, np.float32(1.0), scale).astype(np.float32)
    codes = np.empty(x32.shape, dtype=np.uint8)
    step = max(1, (1 << 22) // max(1, x32.shape[1]))       # row blocks: bounds the temporaries, nothing else
    for r0 in range(0, x32.shape[0], step):
        y = (x32[r0:r0 + step] / scale[r0:r0 + step, None]).astype(np.float32)      # binary32 division
        codes[r0:r0 + step] = e4m3_encode(y)
    return codes, scale


def gemm_fp8(a_codes: np.ndarray, sa: np.ndarray, w_codes: np.ndarray, sw: np.ndarray) -> np.ndarray:
    """C[m, n] = sa[m] sw[n] sum_k dec(a[m, k]) dec(w[n, k]) in float64."""
    a = e4m3_decode(a_codes)
    w = e4m3_decode(w_codes)
    return (a @ w.T) * np.asarray(sa, dtype=np.float64)[:, None] * np.asarray(sw, dtype=np.float64)[None, :]
