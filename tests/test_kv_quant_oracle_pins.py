"""Pins of oracle/kv_quant_oracle.py (CPU only): the e4m3 grid against the format's defining facts
and against torch's own float8_e4m3fn conversion, the scale rule against closed forms, round-trip
error bounds, identity on representable rows, and the eviction reading against the full-attention
special case and a direct softmax."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import kv_quant_oracle as Q
from oracle import skv_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_e4m3_table_matches_the_format():
    for line in open(os.path.join(ROOT, "tests", "golden", "e4m3_format.txt")):
        if line.startswith("#") or not line.strip():
            continue
        code, val = line.split()
        assert Q.E4M3_TABLE[int(code, 16)] == float(val), code
    t = Q.E4M3_TABLE
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and np.isfinite(np.delete(t, [0x7F, 0xFF])).all()
    assert (np.diff(t[:0x7F]) > 0).all()                      # ascending: code order is value order
    assert (t[0x80:0xFF] == -t[:0x7F]).all()
    assert np.nanmax(t) == Q.E4M3_MAX == 448.0


def test_e4m3_table_and_rounding_match_torch_float8():
    """torch.float8_e4m3fn is a library's implementation of the same format: decode all codes, and
    round a dense set of values in range with it."""
    codes = torch.arange(256, dtype=torch.uint8)
    dec = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ours = Q.E4M3_TABLE
    assert np.array_equal(np.isnan(dec), np.isnan(ours))
    assert np.array_equal(dec[~np.isnan(dec)], ours[~np.isnan(ours)])
    rng = np.random.default_rng(3)
    y = np.concatenate([rng.uniform(-448, 448, 20000), rng.normal(0, 1, 20000), rng.normal(0, 0.01, 20000),
                        ours[:0x7F], (ours[:0x7E] + ours[1:0x7F]) / 2])          # grid points and exact ties
    y32 = y.astype(np.float32).astype(np.float64)
    got = Q.round_to_e4m3(y32)
    want = torch.from_numpy(y32.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    zero = y32 == 0
    assert np.array_equal(got[~zero], want[~zero])
    assert ((got[zero] & 0x7F) == 0).all()


def test_ties_go_to_the_even_code():
    t = Q.E4M3_TABLE
    for c in range(0, 0x7E):
        mid = (t[c] + t[c + 1]) / 2
        assert Q.round_to_e4m3(np.array([mid]))[0] == (c if c % 2 == 0 else c + 1)
        assert Q.round_to_e4m3(np.array([-mid]))[0] == 0x80 | (c if c % 2 == 0 else c + 1)


def test_scale_exponent_closed_forms():
    assert Q.scale_exponent(0.0) == 0
    assert Q.scale_exponent(448.0) == 0 and Q.scale_exponent(448.0001) == 1 and Q.scale_exponent(224.0) == -1
    assert Q.scale_exponent(1.0) == -8           # 2^8 = 256 <= 448 < 2^9
    assert Q.scale_exponent(3.5) == -7 and Q.scale_exponent(3.5000001) == -6     # 3.5 = 448 / 128
    rng = np.random.default_rng(0)
    for amax in np.exp(rng.uniform(-60, 60, 2000)):
        e = Q.scale_exponent(float(amax))
        assert amax * 2.0 ** -e <= 448.0 < amax * 2.0 ** -(e - 1)               # smallest such integer
    assert Q.scale_exponent(1e-45) == -127                                       # clamped
    amax = np.concatenate([np.exp(rng.uniform(-100, 100, 500)), [0.0, 448.0, 3.5, 1e-45]])
    assert Q.scale_exponents(amax).tolist() == [Q.scale_exponent(float(a)) for a in amax]


@pytest.mark.parametrize("sigma", [1e-3, 0.5, 1.0, 300.0])
def test_round_trip_error_bounds(sigma):
    rng = np.random.default_rng(5)
    x = torch.from_numpy(rng.normal(0, sigma, (200, 128))).to(torch.bfloat16).to(torch.float64).numpy()
    codes, eb = Q.quantise_rows(x)
    back = Q.dequantise_rows(codes, eb)
    e = eb.astype(np.int64) - 127
    step_sub = np.ldexp(1.0, e - 9)[:, None]                  # spacing of the scaled subnormal grid
    # half an ulp of a 3-bit mantissa: 2^-4 relative for normal codes, half a subnormal step below
    bound = np.maximum(np.abs(x) * 2.0 ** -4, step_sub / 2)
    assert (np.abs(back - x) <= bound).all()
    amax = np.abs(x).max(axis=1)
    assert (np.abs(back).max(axis=1) <= amax * (1 + 2.0 ** -4)).all()
    # the largest element uses the top binade and a half of the code range
    top = np.abs(Q.E4M3_TABLE[codes]).max(axis=1)
    assert ((top >= 224) & (top <= 448)).all()
    # sign symmetry and idempotence
    c2, e2 = Q.quantise_rows(-x)
    assert np.array_equal(e2, eb) and np.array_equal(c2 & 0x7F, codes & 0x7F)
    # (a row whose largest code is exactly 224 re-quantises with the exponent one lower: same values)
    assert np.array_equal(Q.dequantise_rows(*Q.quantise_rows(back)), back)


def test_identity_on_representable_rows():
    rng = np.random.default_rng(8)
    for e in (-20, -3, 0, 5):
        codes = rng.integers(0, 0x7F, size=(50, 64)).astype(np.uint8) | (rng.integers(0, 2, size=(50, 64)) << 7).astype(np.uint8)
        codes[:, 0] = 0x7E                                     # every row reaches the top of the range
        x = np.ldexp(Q.E4M3_TABLE[codes], e)
        c, eb = Q.quantise_rows(x)
        assert (eb == e + 127).all()
        assert np.array_equal(Q.dequantise_rows(c, eb), x)
    z, ez = Q.quantise_rows(np.zeros((2, 16)))
    assert (z == 0).all() and (ez == 127).all() and (Q.dequantise_rows(z, ez) == 0).all()


def test_dequantised_values_are_exact_in_bfloat16():
    rng = np.random.default_rng(2)
    x = torch.from_numpy(rng.normal(0, 0.5, (64, 128))).to(torch.bfloat16).to(torch.float64).numpy()
    back = Q.dequantise_rows(*Q.quantise_rows(x))
    assert np.array_equal(torch.from_numpy(back).to(torch.bfloat16).to(torch.float64).numpy(), back)
    assert np.array_equal(torch.from_numpy(back).to(torch.float16).to(torch.float64).numpy(), back)


def test_eviction_reading():
    rng = np.random.default_rng(4)
    n, d = 300, 32
    K, V, q = rng.normal(size=(n, d)), rng.normal(size=(n, d)), rng.normal(size=d)
    # nothing evicted: the plain definition
    full = Q.attn_over_positions(q, K, V, Q.surviving_positions(n, 0, 0), 0.3)
    assert np.allclose(full, O.attn_one(q, K, V, 0.3), rtol=0, atol=1e-13)
    assert np.array_equal(Q.surviving_positions(n, 64, 64), np.arange(n))         # sink meets window: nothing dropped
    pos = Q.surviving_positions(n, 32, 128)
    assert len(pos) == 32 + (n - 128) and pos[31] == 31 and pos[32] == 128 and pos[-1] == n - 1
    got = Q.attn_over_positions(q, K, V, pos, 0.3)
    s = 0.3 * (K[pos] @ q)
    w = np.exp(s) / np.exp(s).sum()
    assert np.allclose(got, w @ V[pos], rtol=0, atol=1e-13)
    # evicted rows never matter: poison them
    K2, V2 = K.copy(), V.copy()
    K2[32:128], V2[32:128] = np.nan, np.nan
    assert np.array_equal(Q.attn_over_positions(q, K2, V2, pos, 0.3), got)
    # a key that dominates inside the evicted range is gone, one in the sink stays
    K3 = K.copy()
    K3[100] = 50 * q
    assert np.allclose(Q.attn_over_positions(q, K3, V, pos, 0.3), got)
    K3[5] = 50 * q
    assert np.allclose(Q.attn_over_positions(q, K3, V, pos, 0.3), V[5], atol=1e-9)
