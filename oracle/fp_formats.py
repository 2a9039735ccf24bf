"""Storage formats of the MoE-layer oracle: OCP e4m3 ("FN") and bfloat16.

TEST INFRASTRUCTURE ONLY.  Nothing outside tests/, the smoke check and the
benchmark's cpu_baseline leg may import this module; the HIP path shares no
code, table or constant with it.

FP8 rollout (section 3.1.2 of the paper) stores weights and activations in
FP8.  The paper names no variant; the workload's scale rule amax/448 fixes
the OCP e4m3 "FN" format: 1 sign, 4 exponent (bias 7), 3 mantissa bits, no
infinities, the two all-ones codes 0x7F/0xFF are NaN, largest finite value
448.  Encoding is round-to-nearest-even on the value grid with saturation to
+-448, done by searching the explicit 256-entry value table below.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def _build_e4m3_table() -> np.ndarray:
    t = np.empty(256, dtype=np.float64)
    for c in range(256):
        sign = -1.0 if (c >> 7) else 1.0
        e = (c >> 3) & 15
        m = c & 7
        if e == 15 and m == 7:
            t[c] = np.nan
        elif e == 0:
            t[c] = sign * (m / 8.0) * 2.0 ** -6          # subnormal
        else:
            t[c] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return t


#: value of every e4m3 code (index = code byte); NaN at 0x7F and 0xFF
E4M3_TABLE = _build_e4m3_table()
#: the 127 non-negative finite values, codes 0x00..0x7E, strictly increasing
_POS = E4M3_TABLE[:127].copy()


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """uint8 codes -> float64 values (table lookup)."""
    return E4M3_TABLE[np.asarray(codes, dtype=np.uint8)]


def e4m3_encode(r: np.ndarray) -> np.ndarray:
    """Nearest e4m3 code of each real r: ties to the even code, |r|>448 -> +-448.

    The sign of r is kept even when the magnitude rounds to zero (so -0.0 and
    tiny negatives give 0x80).  NaN input is not defined for the layer and
    maps to 0x7F.
    """
    r = np.asarray(r, dtype=np.float64)
    a = np.abs(r)
    a = np.where(np.isnan(a), 0.0, a)
    a = np.minimum(a, E4M3_MAX)
    hi = np.searchsorted(_POS, a, side="left")          # first table value >= a
    hi = np.minimum(hi, 126)
    lo = np.maximum(hi - 1, 0)
    dlo = a - _POS[lo]
    dhi = _POS[hi] - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & ((hi & 1) == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    code = code | (np.signbit(r).astype(np.uint8) << 7)
    return np.where(np.isnan(r), np.uint8(0x7F), code).astype(np.uint8)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64 values (exact)."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return b.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(v: np.ndarray) -> np.ndarray:
    """Round float64 to bfloat16 (nearest, ties to even), return uint16 patterns.

    bfloat16 keeps 8 significant bits.  The value is split as m*2^e with
    0.5<=|m|<1, m is rounded to a multiple of 2^-8 with numpy's rint (ties to
    even), and the result -- exactly representable in float32 -- is read back
    through the float32 bit pattern.  Magnitudes beyond the bfloat16 range do
    not occur in the layer; subnormal results use the fixed quantum 2^-133.
    """
    v = np.asarray(v, dtype=np.float64)
    m, e = np.frexp(v)
    e = np.maximum(e, -125)                       # below 2^-126 the quantum stays 2^-133
    q = np.rint(np.ldexp(v, 8 - e))               # |q| <= 256
    r32 = np.ldexp(q, e - 8).astype(np.float32)   # exact
    return (r32.view(np.uint32) >> 16).astype(np.uint16)
