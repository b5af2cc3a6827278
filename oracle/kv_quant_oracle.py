"""CPU oracle for 8-bit cache slots and for temporal eviction: the two compositions with depth-wise
cache sharing that the paper names as open (Sec. 5, "Limitations": KV quantization and temporal
eviction methods).

THIS IS TEST INFRASTRUCTURE, NOT A COMPUTE PATH (same rules as skv_oracle.py: only tests, the smoke
check and the benchmark's cpu_baseline may import it; it shares nothing with the HIP library).

The paper defines neither, so what is computed here is this build's reading, stated in the design
document and restated in include/skv.h:

Quantised slots.  A K or V row piece of one (position, kv head) -- head_dim values x -- is stored as
head_dim 8-bit codes plus one 8-bit scale exponent:
    amax = max |x|;  e = the smallest integer with amax * 2^-e <= 448, clamped to [-127, 127]
           (e = 0 if amax == 0);
    code_i = the e4m3 number nearest to x_i * 2^-e, ties to the even code (x_i * 2^-e is exact: the
           scale is a power of two);  the stored exponent byte is e + 127.
e4m3 is the 8-bit float of the OCP 8-bit floating point specification ("E4M3": 1 sign, 4 exponent
bits of bias 7, 3 mantissa bits, subnormals, no infinity, S.1111.111 = NaN, largest finite 448); the
exponent byte is that specification family's E8M0 scale.  Attention then runs over the DEQUANTISED
values code * 2^e, which are exact in bfloat16/float16 (3 mantissa bits; a float16 result needs
|code * 2^e| inside float16's range) and in float64: quantisation changes what the cache holds, not
how Eq. (3.1) is evaluated on it.

Temporal eviction.  Each sequence keeps a set of cached positions; the others have been dropped
from every slot (depth-wise sharing and temporal eviction compose: one dropped block frees its
rows in |S| slots instead of L).  The reading built here is the sliding-window-with-sinks family
at block granularity: positions [0, sink_b) and [first_b, n_b) survive, where sink_b and first_b
are multiples of the block size.  Attention of Eq. (3.1) runs over the surviving positions only
(causal: a surviving key j is visible to the query at absolute position p iff j <= p).
"""
from __future__ import annotations

import math

import numpy as np

E4M3_MAX = 448.0


def e4m3_value(code: int) -> float:
    """Value of one e4m3 code, from the format's definition (NaN for S.1111.111)."""
    s = -1.0 if code & 0x80 else 1.0
    e = (code >> 3) & 0xF
    m = code & 0x7
    if e == 0xF and m == 0x7:
        return float("nan")
    if e == 0:
        return s * (m / 8.0) * 2.0 ** -6
    return s * (1.0 + m / 8.0) * 2.0 ** (e - 7)


E4M3_TABLE = np.array([e4m3_value(c) for c in range(256)], dtype=np.float64)
_POS = E4M3_TABLE[:0x7F]          # the 127 non-negative finite values, ascending, code == index


def scale_exponent(amax: float) -> int:
    """Smallest integer e with amax * 2^-e <= 448, clamped to [-127, 127]; 0 for amax == 0."""
    if amax == 0.0:
        return 0
    f, k = math.frexp(amax)              # amax = f * 2^k, 0.5 <= f < 1; 448 = 0.875 * 2^9
    e = k - 9 if f <= 0.875 else k - 8
    return max(-127, min(127, e))


def scale_exponents(amax: np.ndarray) -> np.ndarray:
    """scale_exponent for an array of row maxima (the same rule, element by element)."""
    amax = np.asarray(amax, dtype=np.float64)
    f, k = np.frexp(amax)
    e = np.where(f <= 0.875, k - 9, k - 8)
    return np.where(amax == 0.0, 0, np.clip(e, -127, 127)).astype(np.int64)


def round_to_e4m3(y: np.ndarray) -> np.ndarray:
    """Nearest e4m3 code of every element of y (|y| <= 448), ties to the even code."""
    y = np.asarray(y, dtype=np.float64)
    a = np.abs(y)
    assert (a <= E4M3_MAX).all()
    hi = np.searchsorted(_POS, a, side="left")           # first grid point >= a
    hi = np.minimum(hi, len(_POS) - 1)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - _POS[lo], _POS[hi] - a
    code = np.where(d_lo < d_hi, lo, np.where(d_hi < d_lo, hi, np.where(lo % 2 == 0, lo, hi)))
    code = np.where(_POS[hi] == a, hi, code)
    return (code | np.where(np.signbit(y), 0x80, 0)).astype(np.uint8)


def quantise_rows(x: np.ndarray):
    """x: float64 [..., head_dim] -> (codes uint8 [..., head_dim], exponent bytes uint8 [...])."""
    x = np.asarray(x, dtype=np.float64)
    lead = x.shape[:-1]
    flat = x.reshape(-1, x.shape[-1])
    e = scale_exponents(np.abs(flat).max(axis=1))
    codes = round_to_e4m3(np.ldexp(flat, -e[:, None]))
    return codes.reshape(x.shape), (e + 127).astype(np.uint8).reshape(lead)


def dequantise_rows(codes: np.ndarray, ebyte: np.ndarray) -> np.ndarray:
    """float64 values code * 2^e of quantise_rows' output."""
    e = ebyte.astype(np.int64) - 127
    return np.ldexp(E4M3_TABLE[codes], e[..., None])


def surviving_positions(n: int, sink: int, first: int) -> np.ndarray:
    """Positions of a sequence of n cached positions that survived eviction: [0, sink) and [first, n)."""
    assert 0 <= sink <= first <= n
    return np.concatenate([np.arange(0, sink), np.arange(first, n)]).astype(np.int64)


def attn_over_positions(q, K, V, positions, scale):
    """Eq. (3.1) for one query vector over the listed cached positions only (two-pass softmax).
    q [d]; K, V [n][d] (all positions, evicted rows are never touched); returns [d]."""
    Ks, Vs = K[positions], V[positions]
    s = scale * (Ks @ q)
    w = np.exp(s - s.max())
    return (w / w.sum()) @ Vs
