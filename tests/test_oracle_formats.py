"""Pins of the oracle's e4m3 and bf16 formats against the format definitions,
stored spot values and torch's own float8/bfloat16 casts (CPU only)."""
import os

import numpy as np
import torch

from oracle import fp_formats as ff

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_pairs(name):
    out = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                a, b = line.split()
                out.append((a, b))
    return out


def test_e4m3_spot_values():
    for code, val in _read_pairs("e4m3_spot_values.txt"):
        assert ff.E4M3_TABLE[int(code, 16)] == float(val), code
    assert np.signbit(ff.E4M3_TABLE[0x80]) and ff.E4M3_TABLE[0x80] == 0.0


def test_e4m3_table_structure():
    t = ff.E4M3_TABLE
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF])
    assert np.isfinite(t).sum() == 254
    pos = t[:0x7F]
    assert np.all(np.diff(pos) > 0)                      # strictly increasing over 0x00..0x7E
    assert np.array_equal(t[0x80:0xFF], -pos)            # sign symmetry
    assert pos.max() == 448.0
    assert pos[1] == 2.0 ** -9                           # smallest subnormal
    assert pos[8] == 2.0 ** -6                           # smallest normal


def test_e4m3_table_matches_torch_decode():
    codes = torch.arange(256, dtype=torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ours = ff.e4m3_decode(codes.numpy())
    assert np.array_equal(np.isnan(ref), np.isnan(ours))
    m = ~np.isnan(ref)
    assert np.array_equal(ref[m], ours[m])
    assert np.array_equal(np.signbit(ref[m]), np.signbit(ours[m]))


def test_e4m3_roundtrip_all_finite_codes():
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    assert np.array_equal(ff.e4m3_encode(ff.e4m3_decode(codes)), codes)


def test_e4m3_rounding_cases():
    for real, code in _read_pairs("e4m3_rounding_cases.txt"):
        got = int(ff.e4m3_encode(np.array([float(real)]))[0])
        assert got == int(code, 16), (real, hex(got))


def test_e4m3_ties_to_even_at_every_midpoint():
    pos = ff.E4M3_TABLE[:0x7F]
    for c in range(126):
        mid = 0.5 * (pos[c] + pos[c + 1])                # exact in fp64
        want = c if c % 2 == 0 else c + 1
        assert ff.e4m3_encode(np.array([mid]))[0] == want
        assert ff.e4m3_encode(np.array([-mid]))[0] == (want | 0x80)
        # just off the midpoint goes to the nearer neighbour
        assert ff.e4m3_encode(np.array([np.nextafter(mid, 0.0)]))[0] == c
        assert ff.e4m3_encode(np.array([np.nextafter(mid, 1e9)]))[0] == c + 1


def test_e4m3_never_emits_nan_codes_and_saturates():
    v = np.array([448.0, 448.0001, 463.99, 464.0, 480.0, 1e30, np.inf, -np.inf, -500.0])
    c = ff.e4m3_encode(v)
    assert np.array_equal(c, np.array([0x7E] * 7 + [0xFE, 0xFE], dtype=np.uint8))


def test_e4m3_encode_matches_torch_cast_in_range():
    rng = np.random.default_rng(7)
    # dense in every binade of the format, plus subnormal range, both signs
    mag = np.exp2(rng.uniform(-12, np.log2(448.0), size=400_000))
    v = (mag * rng.choice([-1.0, 1.0], size=mag.size)).astype(np.float32)
    v = v[np.abs(v) <= 448.0]
    ref = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(ff.e4m3_encode(v.astype(np.float64)), ref)


def test_bf16_roundtrip_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    val = ff.bf16_bits_to_f64(bits)
    finite = np.isfinite(val)
    back = ff.f64_to_bf16_bits(val[finite])
    assert np.array_equal(back, bits[finite])


def test_bf16_ties_to_even():
    cases = {1.0 + 2.0 ** -8: 1.0, 1.0 + 3 * 2.0 ** -8: 1.0 + 2.0 ** -6,
             1.0 + 2.0 ** -8 + 2.0 ** -30: 1.0 + 2.0 ** -7, -(1.0 + 2.0 ** -8): -1.0}
    for v, want in cases.items():
        got = ff.bf16_bits_to_f64(ff.f64_to_bf16_bits(np.array([v])))[0]
        assert got == want, (v, got)


def test_bf16_matches_torch_cast():
    rng = np.random.default_rng(3)
    v = (rng.standard_normal(300_000) * np.exp2(rng.uniform(-20, 20, 300_000))).astype(np.float32)
    ref = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ff.f64_to_bf16_bits(v.astype(np.float64)), ref)
